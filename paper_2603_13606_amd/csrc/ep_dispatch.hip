// Dispatch pack, direct path (Sec. IV-C "Send Tokens"; row format of Sec. IV-B
// with the source index and gate weight kept in side arrays so rows are pure
// token data, ready for a grouped GEMM as Sec. III-E asks).
//
// Pure data movement, bound by HBM: a token row of 2H bytes is read once and
// written to up to K destination rows.  Work unit = one wavefront moving one
// 1 KiB segment of one token row: every lane loads 16 bytes once and stores
// them K times, so all global accesses are full 64-lane x 16-byte bursts.  The
// routing entries of the token are wave-uniform and come through scalar loads.
#include "ep_internal.h"
#include "ep_fp8.h"

#include <algorithm>

namespace ep {
namespace {

// One wavefront copies one 1 KiB segment (16-byte unit `seg * 64 + lane` of every lane) of
// token t to the token's destination rows, in two halves so that a caller can put other
// work between the loads and the stores.  Both must be called by all 64 lanes.
struct TokenSegment {
    u32x4 v;     // the 16 bytes of this lane
    int my_row;  // lane k: destination row of the token's k-th entry
};

__device__ __forceinline__ TokenSegment load_token_segment(const DispatchArgs& a, int t, int seg, int units, int lane) {
    TokenSegment s;
    const int unit = seg * kWave + lane;
    s.v = (u32x4){0u, 0u, 0u, 0u};
    if (unit < units) s.v = __builtin_nontemporal_load((const u32x4*)(a.x + (int64_t)t * a.x_stride) + unit);
    // lane k fetches the k-th destination row of the token: one load for all K entries
    s.my_row = lane < a.K ? a.dst_row[(int64_t)t * a.K + lane] : -1;
    return s;
}

__device__ __forceinline__ void store_token_segment(const DispatchArgs& a, const TokenSegment& s, int t, int seg, int units,
                                                    int lane) {
    const int unit = seg * kWave + lane;
    const bool active = unit < units;
    for (int k = 0; k < a.K; ++k) {
        const int row = __builtin_amdgcn_readlane(s.my_row, k);
        if (row < 0) continue;
        if (row >= a.win.rows_cap) {
            if (seg == 0 && lane == 0) atomicOr(&a.totals[TOT_STATUS], STATUS_OUTPUT_OVERFLOW);
            continue;
        }
        uint16_t* dst = a.win.base + window_offset(a.win, row);
        if (active) __builtin_nontemporal_store(s.v, (u32x4*)dst + unit);
        if (seg == 0 && lane == 0) {
            if (a.recv_w) a.recv_w[row] = a.w ? a.w[(int64_t)t * a.w_stride + k] : 1.0f;
            if (a.recv_src) a.recv_src[row] = t;
        }
    }
}

__device__ __forceinline__ void copy_token_segment(const DispatchArgs& a, int t, int seg, int units, int lane) {
    const TokenSegment s = load_token_segment(a, t, seg, units, lane);
    store_token_segment(a, s, t, seg, units, lane);
}

__global__ __launch_bounds__(256) void dispatch_direct_kernel(DispatchArgs a, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (blockIdx.x == 0 && a.recv_count) {
        for (int e = threadIdx.x; e < a.E; e += blockDim.x) a.recv_count[e] = a.expert_kept[e];
    }
    if (u >= (int64_t)a.T * nseg) return;
    const int t = (int)(u / nseg);
    copy_token_segment(a, t, (int)(u - (int64_t)t * nseg), units, lane);
}

// ---- run-ordered variant for large inputs
//
// Writes that land next to each other within a short time are served much faster by the
// memory system than rows scattered at random (measured on this part: 6.3 TB/s against
// 4.9 TB/s), so large inputs are walked in the order of the destination rows instead of
// the order of the tokens.  The layout's expert-sorted entry list is cut into runs: the
// entries of one expert that come from one block of consecutive wave-chunks of the input
// (the layout records where those start).  A run is copied by `splits` workgroups, a few
// rows each per step; consecutive workgroups take the runs of one block expert by expert,
// so the copy sweeps over all expert regions once per block and every region grows by about
// a dozen adjacent rows each time.
//
// A row is read once from HBM and up to K-1 more times from the L2 cache: the 16-byte
// units of a row are split into kSlices equal pieces and workgroup index mod kSlices picks
// the piece, which on this part is also the accelerator die the workgroup runs on, so each
// die's L2 only ever holds its own piece of the tokens of the current block.
constexpr int kSlices = 8;
constexpr int kRunUnroll = 2;

struct RunPlan {
    int group;      // wave-chunks per block
    int nblocks;    // blocks of the input
    int piece;      // 16-byte units per slice
    int units;      // 16-byte units per row
    int tpr_shift;  // log2(threads that share one row piece)
    int first_block;  // this launch covers blocks first_block .. first_block + gridDim.y - 1
    int splits;       // workgroups that share one run
};

// What the walk copies when the rows were quantised ahead of the dispatch (FP8 codes and scales
// in a staging copy, row t at staged + t * pitch: H bytes of codes, then H/128 floats): unit col
// of a staged row goes to the code row of the output window while col < code_units and to the
// row of the scales array after that.  A staged row is half as long as a token row, so it is cut
// into 4 slices instead of 8 (two dies share a slice): the bytes per workgroup stay what they are
// for bf16 rows.  Window strides are in one-byte elements then.
constexpr int kFp8Slices = 4;

struct StagedRows {
    const uint8_t* staged;
    int64_t pitch;
    float* recv_scales;  // [rows, groups]
    int code_units;      // H / 16
    int groups;          // H / 128
};

// TPR_SHIFT = log2(threads that share one row piece); PADDED = window addressing mode; FP8 =
// rows come from a staging copy of quantised rows instead of the bf16 tokens.
//
// The vector-memory counter of this part counts loads and stores alike, in order, and the
// compiler waits for it to reach zero wherever control flow stands between an access and the
// use of its result -- which, between two row stores, means waiting for the first store to
// reach memory before the second is issued.  So the rows of a step are copied by straight-line
// code (loads, then stores, nothing conditional in between) whenever every lane of the wave has
// all its rows, with the general code kept for the ragged end of a run, and the side arrays
// are read before the rows and written after them.
template <int TPR_SHIFT, bool PADDED, bool FP8>
__global__ __launch_bounds__(256) void dispatch_runs_kernel(DispatchArgs a, RunPlan p, StagedRows f) {
    if (blockIdx.x == 0 && blockIdx.y == 0 && p.first_block == 0 && a.recv_count) {
        for (int e = threadIdx.x; e < a.E; e += blockDim.x) a.recv_count[e] = a.expert_kept[e];
    }
    constexpr int tpr = 1 << TPR_SHIFT, nsub = 256 >> TPR_SHIFT;
    constexpr int slices = FP8 ? kFp8Slices : kSlices;
    constexpr int elem_bytes = FP8 ? 1 : 2;  // size of the elements the window strides count
    // grid = (slices * splits * E, blocks): x runs fastest, so workgroups are handed out
    // slice by slice, then share by share of a run, expert by expert, block by block
    const int xs = blockIdx.x & (slices - 1);
    const int es = blockIdx.x / slices;
    const int e = es / p.splits, sp = es - e * p.splits;
    const int blk = p.first_block + blockIdx.y;
    const int c0 = blk * p.group, c1 = min(c0 + p.group, a.nwc);
    // wave-uniform: the run of expert e in block blk, as positions of the sorted entry list
    const int lo = __builtin_amdgcn_readfirstlane(max(a.run_start[(int64_t)c0 * a.E + e], 0));
    int hi = __builtin_amdgcn_readfirstlane(min(a.run_start[(int64_t)c1 * a.E + e], a.T * a.K));
    // padded windows keep the first C entries of an expert: the rest of its sorted range has no row
    if (PADDED) hi = min(hi, __builtin_amdgcn_readfirstlane(a.own_prefix[e]) + a.win.C);
    if (lo >= hi) return;
    const int sub = threadIdx.x >> TPR_SHIFT, u = threadIdx.x & (tpr - 1);
    const int u0 = xs * p.piece, u1 = min(p.units, u0 + p.piece);
    const int cend = FP8 ? min(u1, f.code_units) : u1;  // units of the row proper end here
    const bool side = xs == 0 && u == 0;  // one lane per row fills the side arrays
    const uint8_t* src_base = FP8 ? f.staged : (const uint8_t*)a.x;
    const int64_t src_pitch = FP8 ? f.pitch : a.x_stride * 2;
    uint8_t* dst_base = (uint8_t*)a.win.base;
    for (int pos0 = lo + sp * (nsub * kRunUnroll) + sub; pos0 < hi; pos0 += p.splits * nsub * kRunUnroll) {
        int t[kRunUnroll], row[kRunUnroll];
#pragma unroll
        for (int q = 0; q < kRunUnroll; ++q) {
            const int pos = pos0 + q * nsub;
            t[q] = 0;
            row[q] = -1;
            if (pos < hi) {
                t[q] = a.sorted_token[pos];
                row[q] = a.sorted_row[pos];
                if (row[q] >= a.win.rows_cap) {
                    if (side) atomicOr(&a.totals[TOT_STATUS], STATUS_OUTPUT_OVERFLOW);
                    row[q] = -1;
                }
            }
            if (TPR_SHIFT >= 6) {  // a row piece takes whole waves: token and row, and with them the row
                                   // addresses, are the same for every lane and live in scalar registers
                t[q] = __builtin_amdgcn_readfirstlane(t[q]);
                row[q] = __builtin_amdgcn_readfirstlane(row[q]);
            }
        }
        float wq[kRunUnroll];
        if (side && a.recv_w) {
#pragma unroll
            for (int q = 0; q < kRunUnroll; ++q) {
                wq[q] = 1.0f;
                if (row[q] >= 0 && a.w) wq[q] = a.w[(int64_t)t[q] * a.w_stride + a.sorted_k[pos0 + q * nsub]];
            }
        }
        const uint8_t* src[kRunUnroll];
        uint8_t* dst[kRunUnroll];
        bool have_all = true;
#pragma unroll
        for (int q = 0; q < kRunUnroll; ++q) {
            const int r = max(row[q], 0);
            const int64_t off = PADDED ? window_offset(a.win, r) : (int64_t)r * a.win.stride0;
            src[q] = src_base + (int64_t)t[q] * src_pitch;
            dst[q] = dst_base + off * elem_bytes;
            have_all = have_all && row[q] >= 0;
        }
        if (FP8 && u1 > f.code_units) {  // the slice that holds the scales (workgroup-uniform), a few lanes of it
            for (int col = max(u0, f.code_units) + u; col < u1; col += tpr) {
                const int j = (col - f.code_units) * 4;  // up to four scales; the last unit may be part padding
#pragma unroll
                for (int q = 0; q < kRunUnroll; ++q) {
                    if (row[q] < 0) continue;
                    const u32x4 v = *((const u32x4*)src[q] + col);
                    float* sdst = f.recv_scales + (int64_t)row[q] * f.groups + j;
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        if (j + c < f.groups) sdst[c] = __uint_as_float(v[c]);
                }
            }
        }
        if (__builtin_amdgcn_ballot_w64(!have_all) == 0) {
            for (int col = u0 + u; col < cend; col += tpr) {
                u32x4 v[kRunUnroll];
#pragma unroll
                for (int q = 0; q < kRunUnroll; ++q) v[q] = *((const u32x4*)src[q] + col);
#pragma unroll
                for (int q = 0; q < kRunUnroll; ++q) __builtin_nontemporal_store(v[q], (u32x4*)dst[q] + col);
            }
        } else {
            for (int col = u0 + u; col < cend; col += tpr) {
                u32x4 v[kRunUnroll];
#pragma unroll
                for (int q = 0; q < kRunUnroll; ++q)
                    if (row[q] >= 0) v[q] = *((const u32x4*)src[q] + col);
#pragma unroll
                for (int q = 0; q < kRunUnroll; ++q)
                    if (row[q] >= 0) __builtin_nontemporal_store(v[q], (u32x4*)dst[q] + col);
            }
        }
        if (side) {
#pragma unroll
            for (int q = 0; q < kRunUnroll; ++q) {
                if (row[q] < 0) continue;
                if (a.recv_src) a.recv_src[row[q]] = t[q];
                if (a.recv_w) a.recv_w[row[q]] = wq[q];
            }
        }
    }
}

// Reads token rows [t0, t1) (and, when asked, the index arrays of the layout) once, front
// to back, with ordinary cached loads, so that the run-ordered copy that follows finds
// them in the memory-side cache and the DRAM sees a read phase and then a write phase.
__global__ __launch_bounds__(256) void dispatch_warm_kernel(DispatchArgs a, int units, int t0, int t1, int with_index) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc = 0;
    const int64_t total = (int64_t)(t1 - t0) * units;
    for (int64_t i = gid; i < total; i += stride) {
        const int64_t t = i / units;
        const int col = (int)(i - t * units);
        const u32x4 v = *((const u32x4*)(a.x + (t0 + t) * a.x_stride) + col);
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (with_index) {
        const int n = a.T * a.K, table = (a.nwc + 1) * a.E;
        for (int64_t i = gid; i < n; i += stride) acc ^= (uint32_t)(a.sorted_token[i] ^ a.sorted_row[i]);
        for (int64_t i = gid; i < table; i += stride) acc ^= (uint32_t)a.run_start[i];
    }
    asm volatile("" ::"v"(acc));  // the loads are the point: keep them
}

template <int TPR_SHIFT>
void launch_runs(const DispatchArgs& a, const RunPlan& p, int nblocks, hipStream_t s) {
    const dim3 grid((unsigned)(kSlices * a.E * p.splits), (unsigned)nblocks);
    const StagedRows none = {nullptr, 0, nullptr, 0, 0};
    if (a.win.padded) hipLaunchKernelGGL((dispatch_runs_kernel<TPR_SHIFT, true, false>), grid, dim3(256), 0, s, a, p, none);
    else hipLaunchKernelGGL((dispatch_runs_kernel<TPR_SHIFT, false, false>), grid, dim3(256), 0, s, a, p, none);
}

// ---- quantising dispatch: FP8 (OCP E4M3) rows with one float scale per 128 channels
//
// The paper lets dispatch quantise tokens (Sec. I) and sizes the FP8 row at H bytes
// plus H/128 float scales (Sec. IV-B payload); format and scale rule are fixed by this
// library: per token and 128-channel group amax = max|x|, scale = amax / 448,
// q = e4m3(float(x) * (448 / amax)) rounded to nearest even and saturated at 448;
// amax == 0 gives scale 1.  Work unit = one wavefront x 1024 channels of one token:
// a lane owns 16 consecutive channels (32 bytes in, 16 bytes out), a group is 8 lanes.
// The row is quantised once and stored K times.

__global__ __launch_bounds__(256) void dispatch_fp8_kernel(DispatchArgs a, float* recv_scales, int nseg) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (blockIdx.x == 0 && a.recv_count) {
        for (int e = threadIdx.x; e < a.E; e += blockDim.x) a.recv_count[e] = a.expert_kept[e];
    }
    if (u >= (int64_t)a.T * nseg) return;
    const int t = (int)(u / nseg);
    const int seg = (int)(u - (int64_t)t * nseg);
    const int ch0 = seg * 1024 + lane * 16;  // first channel of this lane
    const bool active = ch0 < a.H;
    u32x4 in0 = {0u, 0u, 0u, 0u}, in1 = {0u, 0u, 0u, 0u};
    if (active) {
        const u32x4* src = (const u32x4*)(a.x + (int64_t)t * a.x_stride + ch0);
        in0 = __builtin_nontemporal_load(src);
        in1 = __builtin_nontemporal_load(src + 1);
    }
    float scale;
    const u32x4 q = quantize16(in0, in1, &scale);
    const int groups = a.H >> 7;
    const int my_row = lane < a.K ? a.dst_row[(int64_t)t * a.K + lane] : -1;
    uint8_t* base = (uint8_t*)a.win.base;  // window strides are in one-byte elements here
    for (int k = 0; k < a.K; ++k) {
        const int row = __builtin_amdgcn_readlane(my_row, k);
        if (row < 0) continue;
        if (row >= a.win.rows_cap) {
            if (seg == 0 && lane == 0) atomicOr(&a.totals[TOT_STATUS], STATUS_OUTPUT_OVERFLOW);
            continue;
        }
        if (active) {
            __builtin_nontemporal_store(q, (u32x4*)(base + window_offset(a.win, row) + ch0));
            if ((lane & 7) == 0) recv_scales[(int64_t)row * groups + (ch0 >> 7)] = scale;
        }
        if (seg == 0 && lane == 0) {
            if (a.recv_w) a.recv_w[row] = a.w ? a.w[(int64_t)t * a.w_stride + k] : 1.0f;
            if (a.recv_src) a.recv_src[row] = t;
        }
    }
}

// Plain streaming copy, 16 bytes per lane, grid-stride: the yardstick the hardware
// counters and the achievable copy bandwidth are calibrated against.
__global__ __launch_bounds__(256) void calibration_copy_kernel(u32x4* dst, const u32x4* src, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// The two halves of that copy on their own, four 16-byte accesses per lane and trip: what this
// part's memory sustains for reads alone and for writes alone (a row kernel that mostly writes,
// or mostly reads, is bounded by these and not by the mixed copy).
__global__ __launch_bounds__(256) void calibration_fill_kernel(u32x4* dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * 1024;
    const u32x4 v = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += stride) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i + j * 256 < n16) __builtin_nontemporal_store(v, dst + i + j * 256);
    }
}

__global__ __launch_bounds__(256) void calibration_read_kernel(const u32x4* src, int64_t n16, uint32_t* sink) {
    const int64_t stride = (int64_t)gridDim.x * 1024;
    uint32_t acc = 0;
    for (int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x; i < n16; i += stride) {
        u32x4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(src + min(i + j * 256, n16 - 1));
#pragma unroll
        for (int j = 0; j < 4; ++j) acc ^= v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
    }
    // the loads must not be dropped: the word is written only if the lane's checksum is one particular value
    if (acc == 0x9e3779b9u) *sink = acc;
}

}  // namespace

hipError_t launch_calibration_fill(void* dst, size_t bytes, hipStream_t s) {
    const int64_t n16 = (int64_t)(bytes / 16);
    if (n16 == 0) return hipSuccess;
    int64_t nblk = (n16 + 1023) / 1024;
    if (nblk > 256 * 64) nblk = 256 * 64;
    hipLaunchKernelGGL(calibration_fill_kernel, dim3((unsigned)nblk), dim3(256), 0, s, (u32x4*)dst, n16);
    return hipGetLastError();
}

hipError_t launch_calibration_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s) {
    const int64_t n16 = (int64_t)(bytes / 16);
    if (n16 == 0) return hipSuccess;
    int64_t nblk = (n16 + 1023) / 1024;
    if (nblk > 256 * 64) nblk = 256 * 64;
    hipLaunchKernelGGL(calibration_read_kernel, dim3((unsigned)nblk), dim3(256), 0, s, (const u32x4*)src, n16, sink);
    return hipGetLastError();
}

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const int64_t n16 = (int64_t)(bytes / 16);
    if (n16 == 0) return hipSuccess;
    int64_t nblk = (n16 + 255) / 256;
    if (nblk > 256 * 64) nblk = 256 * 64;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)nblk), dim3(256), 0, s, (u32x4*)dst,
                       (const u32x4*)src, n16);
    return hipGetLastError();
}

// Inputs from kRunOrderMinEntries entries on can be copied in run order (when the layout
// recorded the runs); smaller ones are bound by latency and keep the shorter token-ordered
// kernel.  A read pass covers kWarmBytes of tokens: a piece must stay in the 256 MiB
// memory-side cache, next to whatever else lives there, while the copy of that piece runs.
//
// A block holds about 12 rows per expert, and no more tokens than keep one slice of them
// (2H/8 bytes each) within 2 MiB, half of an XCD's L2.  Longer runs are rewarded by the
// memory system when the routing is even (32 rows per expert: 86 instead of 88 us at the
// prefill shape) but lose more when a few experts are hot, because the workgroups of a long
// hot run then loop while the others idle; 8 to 16 rows are within 1 % of the best on every
// shape measured.  A workgroup copies nsub * kRunUnroll rows at a time, so a run of average
// length is shared by `splits` workgroups, one step each.
// `units` 16-byte units per copied row, cut into `slices` slices; H = channels of a token row
// (what a read pass reads).
static bool plan_rows(int T, int K, int H, int units, int slices, int E, int order, bool have_runs, int prefetched_rows,
                      DispatchPlan* out) {
    DispatchPlan d = {};
    const int64_t n = (int64_t)T * K;
    d.run_order = order != EP_ORDER_TOKEN && have_runs && n >= kRunOrderMinEntries && units >= slices;
    if (!d.run_order) { *out = d; return false; }
    int passes = 0, nwc = 0;
    plan_layout((int)n, &passes, &nwc);
    const int chunk_entries = passes * kWave;
    const int64_t l2_tokens = (2ll << 20) / std::max(16 * units / slices, 1);
    const int want = (int)std::max<int64_t>(768, std::min<int64_t>(12ll * E, l2_tokens * K));
    d.group = std::max(1, want / chunk_entries);
    d.blocks = (nwc + d.group - 1) / d.group;
    d.piece = (units + slices - 1) / slices;
    if (d.piece >= 8) d.piece = (d.piece + 7) / 8 * 8;  // whole 128-byte lines per slice (the last slices get less)
    d.tpr_shift = 4;
    while ((1 << d.tpr_shift) < d.piece && d.tpr_shift < 8) ++d.tpr_shift;
    const int rows_per_step = (256 >> d.tpr_shift) * kRunUnroll;
    const int avg_run = (int)(((int64_t)d.group * chunk_entries + E - 1) / E);
    d.splits = std::max(1, (avg_run + rows_per_step - 1) / rows_per_step);
    d.block_entries = d.group * chunk_entries;
    // blocks per launch: all of them, or as many as cover kWarmBytes of tokens
    d.blocks_per_launch = d.blocks;
    if (order == EP_ORDER_DESTINATION) {
        const int64_t block_bytes = ((int64_t)d.block_entries + K - 1) / K * H * 2;
        d.blocks_per_launch = (int)std::max<int64_t>(1, std::min<int64_t>(d.blocks, kWarmBytes / std::max<int64_t>(block_bytes, 1)));
    }
    for (int b0 = 0; b0 < d.blocks; b0 += d.blocks_per_launch) {
        const int nb = std::min(d.blocks_per_launch, d.blocks - b0);
        const int t1 = (int)std::min<int64_t>(T, ((int64_t)(b0 + nb) * d.block_entries + K - 1) / K);
        d.launches += 1;
        if (order == EP_ORDER_DESTINATION && t1 > prefetched_rows) d.read_passes += 1;
    }
    *out = d;
    return true;
}

bool plan_dispatch(int T, int K, int H, int E, int order, bool have_runs, int prefetched_rows, DispatchPlan* out) {
    return plan_rows(T, K, H, H / 8, kSlices, E, order, have_runs, prefetched_rows, out);
}

// The copy launches of the run order (with their read passes): `launch(plan, blocks)` starts
// the copy of `blocks` blocks from plan.first_block on.
template <typename Launch>
static void launch_run_order(const DispatchArgs& a, const DispatchPlan& d, RunPlan p, hipStream_t s, Launch launch) {
    const int units = a.H / 8;
    for (int b0 = 0; b0 < d.blocks; b0 += d.blocks_per_launch) {
        const int nb = std::min(d.blocks_per_launch, d.blocks - b0);
        const int t0 = (int)std::min<int64_t>(a.T, (int64_t)b0 * d.block_entries / a.K);
        const int t1 = (int)std::min<int64_t>(a.T, ((int64_t)(b0 + nb) * d.block_entries + a.K - 1) / a.K);
        // a read pass, unless the layout launch has read these rows already
        if (a.order == EP_ORDER_DESTINATION && t1 > a.prefetched_rows)
            hipLaunchKernelGGL(dispatch_warm_kernel, dim3(2048), dim3(256), 0, s, a, units, t0, t1, b0 == 0 ? 1 : 0);
        p.first_block = b0;
        launch(p, nb);
    }
}

hipError_t launch_dispatch(const DispatchArgs& a, hipStream_t s) {
    const int units = a.H / 8;  // 16-byte units per row
    DispatchPlan d;
    if (plan_dispatch(a.T, a.K, a.H, a.E, a.order, a.run_start != nullptr, a.prefetched_rows, &d)) {
        RunPlan p;
        p.group = d.group; p.nblocks = d.blocks; p.units = units; p.piece = d.piece; p.tpr_shift = d.tpr_shift;
        p.splits = d.splits;
        launch_run_order(a, d, p, s, [&](const RunPlan& q, int nb) {
            switch (q.tpr_shift) {
                case 4: launch_runs<4>(a, q, nb, s); break;
                case 5: launch_runs<5>(a, q, nb, s); break;
                case 6: launch_runs<6>(a, q, nb, s); break;
                case 7: launch_runs<7>(a, q, nb, s); break;
                default: launch_runs<8>(a, q, nb, s); break;
            }
        });
        return hipGetLastError();
    }
    const int nseg = (units + kWave - 1) / kWave;
    const int64_t nwaves = (int64_t)a.T * nseg;
    int64_t nblk = (nwaves + 3) / 4;
    if (nblk < 1) nblk = 1;  // block 0 also copies the per-expert counts
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dispatch_direct_kernel, dim3((unsigned)nblk), dim3(256), 0, s, a, nseg, units);
    return hipGetLastError();
}

// The quantising dispatch in token order: a row is quantised once for all its destinations.
// (Measured at the prefill shape, 61 us this way.  In the order of the destination rows:
// quantising a row piece again for every destination row is bound by arithmetic, 129 us;
// quantising once into a staging copy by a kernel of its own and copying that in run order,
// 90 us for the two.  Only when the staging copy is made while the layout runs -- see
// launch_dispatch_fp8_staged -- does the copy, 56 us, come out ahead, and the layout launch
// then takes 7 us longer.)
hipError_t launch_dispatch_fp8(const DispatchArgs& a, float* recv_scales, hipStream_t s) {
    const int nseg = (a.H + 1023) / 1024;
    const int64_t nwaves = (int64_t)a.T * nseg;
    int64_t nblk = (nwaves + 3) / 4;
    if (nblk < 1) nblk = 1;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dispatch_fp8_kernel, dim3((unsigned)nblk), dim3(256), 0, s, a, recv_scales, nseg);
    return hipGetLastError();
}

// Units of a staged FP8 row: H/16 of codes, then the scales rounded up to whole units.
static int fp8_code_units(int H) { return H / 16; }
static int fp8_row_units(int H) { return H / 16 + (H / 32 + 15) / 16; }

bool dispatch_fp8_staged_possible(const DispatchArgs& a) {
    DispatchPlan d;
    return a.H % 128 == 0 && plan_rows(a.T, a.K, a.H, fp8_row_units(a.H), kFp8Slices, a.E, EP_ORDER_DESTINATION_RESIDENT,
                                       a.run_start != nullptr, 0, &d);
}

template <int TPR_SHIFT>
static void launch_runs_fp8(const DispatchArgs& a, const RunPlan& p, int nblocks, const uint8_t* staged, int64_t pitch,
                            float* recv_scales, hipStream_t s) {
    const dim3 grid((unsigned)(kFp8Slices * a.E * p.splits), (unsigned)nblocks);
    const StagedRows f = {staged, pitch, recv_scales, fp8_code_units(a.H), a.H / 128};
    if (a.win.padded) hipLaunchKernelGGL((dispatch_runs_kernel<TPR_SHIFT, true, true>), grid, dim3(256), 0, s, a, p, f);
    else hipLaunchKernelGGL((dispatch_runs_kernel<TPR_SHIFT, false, true>), grid, dim3(256), 0, s, a, p, f);
}

hipError_t launch_dispatch_fp8_staged(const DispatchArgs& a, float* recv_scales, const uint8_t* staged, int64_t pitch,
                                      hipStream_t s) {
    DispatchPlan d;
    if (a.H % 128 != 0 || !plan_rows(a.T, a.K, a.H, fp8_row_units(a.H), kFp8Slices, a.E, EP_ORDER_DESTINATION_RESIDENT,
                                     a.run_start != nullptr, 0, &d))
        return hipErrorInvalidValue;
    RunPlan p;
    p.group = d.group; p.nblocks = d.blocks; p.units = fp8_row_units(a.H); p.piece = d.piece; p.tpr_shift = d.tpr_shift;
    p.splits = d.splits; p.first_block = 0;
    switch (p.tpr_shift) {  // every block in one launch: the staged rows were written just before, nothing to read ahead
        case 4: launch_runs_fp8<4>(a, p, d.blocks, staged, pitch, recv_scales, s); break;
        case 5: launch_runs_fp8<5>(a, p, d.blocks, staged, pitch, recv_scales, s); break;
        case 6: launch_runs_fp8<6>(a, p, d.blocks, staged, pitch, recv_scales, s); break;
        case 7: launch_runs_fp8<7>(a, p, d.blocks, staged, pitch, recv_scales, s); break;
        default: launch_runs_fp8<8>(a, p, d.blocks, staged, pitch, recv_scales, s); break;
    }
    return hipGetLastError();
}

}  // namespace ep
