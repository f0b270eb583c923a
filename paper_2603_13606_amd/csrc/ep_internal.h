// Internal declarations shared by the translation units of libep_mi355x.so.
// Host-side structs and the launch functions each kernel file exports.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ep.h"

namespace ep {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kMaxExperts = 1024;
constexpr int kMaxTopK = 64;
constexpr int kMaxWaveChunks = 512;        // wave-chunks per layout
constexpr int kMaxChunks = 256;            // workgroups (chunks) per layout, and rows of the published bin sums
constexpr int kLayoutWavesPerBlock = 16;   // wavefronts per workgroup (chunk); fewer when the bin tables are large
constexpr int kLayoutOneBlockEntries = 4096;  // inputs up to this size are laid out by one workgroup
constexpr int kTotalsWords = 16;
constexpr int kLayoutCtlWords = 4;

// indices into the device totals block
enum { TOT_KEPT = 0, TOT_DROPPED, TOT_MASKED, TOT_INVALID, TOT_SORTED, TOT_MSGS, TOT_STATUS,
       TOT_ROWS_END };

enum { STATUS_INVALID_IDS = 1, STATUS_CAPACITY_DROP = 2, STATUS_OUTPUT_OVERFLOW = 4, STATUS_TIMEOUT = 8 };

// Everything the layout kernels need.  All pointers are device pointers.
struct LayoutArgs {
    const int32_t* topk;      // [T, K], row stride topk_stride
    int64_t topk_stride;
    const int32_t* expert_base;  // [E] or nullptr
    int T, K, E, R, L;
    int L_shift;              // log2(L) if L is a power of two, else -1
    int K_shift;              // log2(K) if K is a power of two, else -1
    int padded;               // 1 = [E, C, H] layout
    int C;                    // slots per (expert, source) sub-region
    int C_rank;               // staging slots per destination rank in padded mode
    int n;                    // T * K
    int passes;               // a wave-chunk is 64 * passes consecutive entries
    int nwc;                  // number of wave-chunks
    int W;                    // histogram width: E experts + masked + invalid + R ranks
    int bits_e, bits_r;       // key widths for the in-wave match
    uint32_t* pub;            // [kMaxChunks, W] scratch: per-chunk bin sums, each tagged with its launch
    uint32_t* ctl;            // [kLayoutCtlWords] scratch: generation and arrival count (see ep_layout.hip);
                              // pub and ctl start out zero and are kept consistent by the kernel itself
    int32_t* expert_count;    // [E]
    int32_t* expert_kept;     // [E]
    int32_t* expert_offset;   // [E+1]
    int32_t* own_prefix;      // [E+1]
    int32_t* rank_pair_count; // [R]
    int32_t* rank_token_count;// [R]
    int32_t* rank_offset;     // [R+1]
    int32_t* totals;          // [kTotalsWords]
    int32_t* slot;            // [n]
    int32_t* dst_row;         // [n]
    int32_t* rank_row;        // [n]
    int32_t* entry_rank;      // [n] destination rank of the entry, -1 if not routed (may be nullptr)
    int32_t* sorted_token;    // [n]
    int32_t* sorted_k;        // [n]
    int32_t* sorted_row;      // [n]
    // optional: token rows to read into the memory-side cache on otherwise idle compute units
    const uint16_t* warm_x;   // [warm_rows, H] bf16, row stride warm_stride elements, or nullptr
    int64_t warm_stride;
    int warm_rows, warm_units;  // rows to read, 16-byte units per row
    uint8_t* quant_out;       // or nullptr: rows [0, warm_rows) are also quantised to FP8 into this staging copy,
    int64_t quant_pitch;      // row t at quant_out + t * quant_pitch: H codes, then H/128 float scales
    int nchunks;              // workgroups of the slot kernel that lay out (set by launch_layout)
    int64_t rows_cap;         // a launch that also dispatches: rows its output takes (more are flagged); else -1
    int32_t* recv_count;      // such a launch: where the caller wants the rows placed per expert [E]; else nullptr
    int64_t* drop_hint;       // mapped host word or nullptr: gets kept | dropped << 32 (rows of padded windows)
    int32_t* run_start;       // [nwc+1, E] or nullptr: first sorted position of expert e among the entries
                              // of wave-chunks >= c (row c); only the histogram kernels fill it
};

// Addressing of the receive windows: element offset of logical row r is
//   padded: (r / C) * stride0 + (r % C) * stride1      (3-D [E, C, H])
//   concat:  r * stride0                               (2-D [rows, H])
// (the quantising dispatch reuses it for one-byte elements: base is then a byte pointer)
struct WindowDesc {
    uint16_t* base;
    int64_t stride0, stride1;
    int64_t rows_cap;  // rows addressable through this descriptor
    int padded;
    int C;
};

// Element offset of logical row `row` of a window (see WindowDesc).
__device__ __forceinline__ int64_t window_offset(const WindowDesc& w, int row) {
    if (w.padded) {
        const int e = row / w.C;
        const int s = row - e * w.C;
        return (int64_t)e * w.stride0 + (int64_t)s * w.stride1;
    }
    return (int64_t)row * w.stride0;
}

struct DispatchArgs {
    const uint16_t* x;
    int64_t x_stride;
    const float* w;          // [T, K] or nullptr
    int64_t w_stride;
    const int32_t* dst_row;  // [T, K] contiguous
    WindowDesc win;
    float* recv_w;           // [rows] or nullptr
    int32_t* recv_src;       // [rows] or nullptr
    int32_t* recv_count;     // [E] or nullptr
    const int32_t* expert_kept;
    int32_t* totals;
    int T, K, H, E;
    // run-ordered kernel only (see launch_dispatch): the expert-sorted entry list of the
    // layout and the table of where each wave-chunk's entries start inside it
    const int32_t* sorted_token;  // [n]
    const int32_t* sorted_k;      // [n]
    const int32_t* sorted_row;    // [n]
    const int32_t* own_prefix;    // [E+1] first sorted position of each expert
    const int32_t* run_start;     // [nwc+1, E], or nullptr: the layout did not produce one
    int nwc;                      // wave-chunks of the layout
    int chunk_entries;            // entries per wave-chunk
    int order;                    // EP_ORDER_*
    int prefetched_rows;          // leading token rows the layout launch has already read into cache
};

struct CombineArgs {
    WindowDesc win;          // y
    const float* w;          // [T, K] or nullptr
    int64_t w_stride;
    const int32_t* dst_row;
    uint16_t* out;
    int64_t out_stride;
    int T, K, H;
    int staged;              // 1: y is the (t,k)-indexed staging, entry (t,k) sits in row t*K + k
    const int32_t* entry_rank;  // [T, K] destination rank per entry (two-level order only)
    int ranks_per_node;      // > 0: sum per node first, then across nodes; 0: flat k order
    int nodes;
};

struct DedupSendArgs {
    const uint16_t* x;
    int64_t x_stride;
    const int32_t* topk;
    int64_t topk_stride;
    const float* w;           // [T, K] or nullptr (header then carries 1.0)
    int64_t w_stride;
    const int32_t* rank_row;  // [T, K] staging slot for the first k naming a rank, else -1
    uint8_t* staging;
    int64_t msg_stride;       // bytes from one staging slot to the next
    int64_t msg_lead;         // bytes between the start of a slot and its message
    int64_t staging_slots;
    int hdr_units;            // header size in 16-byte units
    int32_t* totals;
    int T, K, H;
};

struct DedupFanoutArgs {
    const uint8_t* staging;
    int64_t msg_stride, msg_lead, hdr_bytes;
    int64_t staging_slots;
    int slots_per_rank;            // > 0: fixed-size window per rank; 0: compact windows
    const int32_t* rank_offset;    // [R+1]
    const int32_t* rank_count;     // [R]
    const int32_t* recv_dst_row;   // [staging_slots, K]
    const int32_t* recv_kept;      // [E]
    WindowDesc win;
    float* recv_w;
    int32_t* recv_src;
    int32_t* recv_count;
    int32_t* totals;
    int K, H, E, R;
};

// Receiving side of the once-per-rank path: ranks the header entries of every staging
// window among the entries of the same expert, in slot order.
struct DedupRankArgs {
    const uint8_t* staging;
    int64_t msg_stride, msg_lead;
    int64_t staging_slots;
    int slots_per_rank;              // > 0: fixed-size window per rank; 0: compact windows
    const int32_t* rank_offset;      // [R+1] first slot of each rank's window
    const int32_t* rank_count;       // [R]   messages in each rank's window
    const int32_t* expert_offset;    // [E+1] first row of each expert (concat layout)
    int32_t* recv_dst_row;           // [staging_slots, K] out: row of each header entry, -1 if none
    int32_t* recv_count;             // [E] out: entries per expert
    int32_t* recv_kept;              // [E] out: rows per expert (capped at C in the padded layout)
    int K, E, R, L, L_shift, K_shift;
    int bits_l;                      // bits of a local expert index
    int padded, C;
};

hipError_t launch_layout(const LayoutArgs& a, hipStream_t s);
// Layout and direct dispatch of a small input in one launch (see ep_layout.hip); `fusable` says
// whether the pair qualifies.
bool layout_dispatch_fusable(const LayoutArgs& a, const DispatchArgs& d);
hipError_t launch_layout_dispatch(const LayoutArgs& a, const DispatchArgs& d, hipStream_t s);
hipError_t launch_dedup_rank(const DedupRankArgs& a, hipStream_t s);
hipError_t launch_dedup_send(const DedupSendArgs& a, hipStream_t s);
hipError_t launch_dedup_fanout(const DedupFanoutArgs& a, hipStream_t s);
hipError_t launch_dispatch(const DispatchArgs& a, hipStream_t s);
hipError_t launch_dispatch_fp8(const DispatchArgs& a, float* recv_scales, hipStream_t s);
// The quantising dispatch from rows already quantised into a staging copy (LayoutArgs::quant_out),
// in destination order.  False when this input is not walked in destination order.
bool dispatch_fp8_staged_possible(const DispatchArgs& a);
hipError_t launch_dispatch_fp8_staged(const DispatchArgs& a, float* recv_scales, const uint8_t* staged, int64_t pitch,
                                      hipStream_t s);
// Bytes between two rows of the staging copy for hidden size H (a multiple of 128).
constexpr int64_t quant_row_pitch(int H) { return (int64_t)H + (((int64_t)H / 32 + 15) / 16) * 16; }
hipError_t launch_combine(const CombineArgs& a, hipStream_t s);
// How a combine of T tokens of H channels is cut into wavefronts on a GPU of `compute_units`
// units (host arithmetic; launch_combine plans with the current device's count).
struct CombinePlan {
    int segments;   // 1 KiB segments of a token row per wavefront: 1, 2, or the whole row
    int whole_row;  // 1: one wavefront per token
    int64_t workgroups;
};
void plan_combine(int64_t T, int H, int ranks_per_node, int compute_units, CombinePlan* out);
// Backward of the weighted combine: a.win = expert outputs y (base may be nullptr: no grad_w), a.w, a.dst_row,
// T, K, H as for the forward; g = gradient of the combined output [T, H]; gy = windows for grad_y.
hipError_t launch_combine_backward(const CombineArgs& a, const uint16_t* g, int64_t g_stride, const WindowDesc& gy,
                                   float* grad_w, int64_t gw_stride, hipStream_t s);
hipError_t launch_publish_counts(int32_t* sig, const int32_t* counts, int n, hipStream_t s);
hipError_t launch_await_counts(int32_t* sig, int n, int spin_limit, int32_t* count_out, int32_t* offset_out,
                               int32_t* totals, hipStream_t s);
hipError_t launch_clear_counts(int32_t* sig, int n, hipStream_t s);
hipError_t launch_combine_pack(const CombineArgs& a, uint16_t* stage, hipStream_t s);
hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_calibration_fill(void* dst, size_t bytes, hipStream_t s);
hipError_t launch_calibration_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s);

// Host-side planning helpers (pure functions, testable without a GPU).
void plan_layout(int n, int* passes, int* nwc);

// How launch_dispatch walks an input (see ep_dispatch.hip).
struct DispatchPlan {
    int run_order;          // 1: destination order; 0: token order (nothing else is set then)
    int group;              // wave-chunks of the layout per block
    int blocks;             // blocks of the input
    int block_entries;      // routed entries per block
    int splits;             // workgroups that share the run of one (block, expert)
    int piece;              // 16-byte units of a row per XCD slice
    int tpr_shift;          // log2(threads that share one row piece)
    int blocks_per_launch;  // blocks per copy launch
    int launches;           // copy launches
    int read_passes;        // token read passes (at most one per copy launch)
};
bool plan_dispatch(int T, int K, int H, int E, int order, bool have_runs, int prefetched_rows, DispatchPlan* out);
// True when launch_layout fills LayoutArgs::run_start for this plan.
bool layout_writes_runs(const LayoutArgs& a);
// True when launch_layout reads LayoutArgs::warm_x for this plan.
bool layout_prefetches(const LayoutArgs& a);
// Token bytes one read pass of the destination-ordered dispatch covers.
constexpr int64_t kWarmBytes = 64ll << 20;
// Inputs from this many routed entries on may be dispatched in destination order.
constexpr int kRunOrderMinEntries = 8192;

}  // namespace ep
