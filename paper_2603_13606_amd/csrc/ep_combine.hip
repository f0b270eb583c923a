// Combine: gather the K expert outputs of every token and reduce them with the
// gate weights (Sec. II-B "Combine"; Sec. IV-B receive phase; Sec. IV-C
// "Combine/recv"; the (t, k)-indexed addressing of Sec. IV-D).
//
//   out[t, h] = bf16_rne( sum_{k = 0..K-1, in order} w[t,k] * f32(y[dst_row[t,k], h]) )
//
// float32 multiply and float32 add are separate, each rounded to nearest even
// (no fused multiply-add), so the result does not depend on the launch shape.
// Bound by HBM: K rows read, one row written per token.  Work unit = one
// wavefront reducing one 1 KiB segment of one token: every lane issues up to 8
// independent 16-byte loads before it starts to accumulate.
#include <atomic>

#include "ep_internal.h"

namespace ep {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int KB = 8;  // rows gathered per batch of loads

__device__ __forceinline__ float bf16_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }

// Two float32 -> two bfloat16 packed low, high: round to nearest even, every NaN becomes 0x7FC0.
// The conversion instruction of this part rounds exactly as the integer rule
// (u + 0x7FFF + bit 16) >> 16 does -- compared over all 2^32 inputs -- and leaves only the
// NaN payload to be made canonical here.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    uint32_t u = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    if (lo != lo) u = (u & 0xffff0000u) | 0x7fc0u;
    if (hi != hi) u = (u & 0x0000ffffu) | 0x7fc00000u;
    return u;
}

__device__ __forceinline__ void accumulate(float (&acc)[8], const u32x4& v, float w) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        acc[2 * c] = __fadd_rn(acc[2 * c], __fmul_rn(w, bf16_lo(v[c])));
        acc[2 * c + 1] = __fadd_rn(acc[2 * c + 1], __fmul_rn(w, bf16_hi(v[c])));
    }
}

// Byte offset of entry (t, k)'s row in the window, or -1 when the entry has no row: computed once
// per entry by the lane that holds it (the division of the padded addressing included), so that
// the loop over the entries only moves it into scalar registers.
__device__ __forceinline__ int64_t entry_row_offset(const CombineArgs& a, int t, int k, int row) {
    if (row < 0 || row >= a.win.rows_cap) return -1;
    const int64_t elems = a.staged ? (int64_t)(t * a.K + k) * a.H : window_offset(a.win, row);  // (t,k)-indexed staging (Sec. IV-D)
    return elems * 2;
}

__device__ __forceinline__ int64_t readlane64(int64_t v, int lane) {
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, lane);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)((uint64_t)v >> 32), lane);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// The next N entries that have rows (the set bits of `mask`, lowest first: ascending k), gathered
// and added to the sums.  Straight-line code for a count known at compile time: all N * SEGS loads
// are in flight before the first is waited for -- behind a branch the compiler may wait for the
// earlier loads before it issues the next -- and an entry without a row costs nothing, not even a
// test.  SEGS = 2: the wave reduces two adjacent 1 KiB segments of the token (`base` points into
// the first; the second lies 1 KiB behind it in every row).
template <int N, bool DENSE, int SEGS>
__device__ __forceinline__ void gather_rows(uint64_t& mask, int& first, int64_t my_off, float my_w, const uint8_t* base,
                                            int second, float (&acc)[SEGS][8]) {
    u32x4 v[N][SEGS];
    float wk[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
        int src;  // wave-uniform: the lane that holds the entry
        if (DENSE) {  // every entry has a row: the lanes in turn
            src = first + j;
        } else {
            src = __builtin_ctzll(mask);
            mask &= mask - 1;
        }
        wk[j] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), src));
        const uint8_t* p = base + readlane64(my_off, src);
        v[j][0] = __builtin_nontemporal_load((const u32x4*)p);
        if (SEGS == 2) v[j][1] = __builtin_nontemporal_load((const u32x4*)(p + second));
    }
    first += N;
#pragma unroll
    for (int j = 0; j < N; ++j)
#pragma unroll
        for (int q = 0; q < SEGS; ++q) accumulate(acc[q], v[j][q], wk[j]);
}

template <bool DENSE, int SEGS>
__device__ __forceinline__ void gather_all(uint64_t mask, int left, int64_t my_off, float my_w, const uint8_t* base, int second,
                                           float (&acc)[SEGS][8]) {
    int first = 0;
    for (; left >= KB; left -= KB) gather_rows<KB, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc);
    switch (left) {
        case 1: gather_rows<1, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc); break;
        case 2: gather_rows<2, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc); break;
        case 3: gather_rows<3, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc); break;
        case 4: gather_rows<4, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc); break;
        case 5: gather_rows<5, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc); break;
        case 6: gather_rows<6, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc); break;
        case 7: gather_rows<7, DENSE, SEGS>(mask, first, my_off, my_w, base, second, acc); break;
        default: break;
    }
}

// SEGS segments of 1 KiB per wavefront.  Two segments per wavefront (nseg even) halve the number
// of wavefronts and of index fetches and put 16 loads per lane in flight: a few per cent faster
// once the launch is long enough to be bound by the memory and not by its latency.
template <int SEGS>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nper = nseg / SEGS;  // work units per token
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (u >= (int64_t)a.T * nper) return;
    const int t = (int)(u / nper);
    const int seg = (int)(u - (int64_t)t * nper) * SEGS;
    const int unit = seg * kWave + lane;
    // lanes beyond the end of the row read its last unit (and store nothing)
    const int unit0 = min(unit, units - 1);
    const uint8_t* base = (const uint8_t*)a.win.base + (int64_t)unit0 * 16;
    const int second = SEGS == 2 ? (min(unit + kWave, units - 1) - unit0) * 16 : 0;
    float acc[SEGS][8];
#pragma unroll
    for (int q = 0; q < SEGS; ++q)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[q][c] = 0.0f;
    for (int k0 = 0; k0 < a.K; k0 += kWave) {  // the entries of the token, 64 at a time in the lanes of the wave
        // lane j fetches row index and weight of entry k0 + j (one load each for up to 64 entries) and works
        // out where the row lies
        const int kk = k0 + lane;
        const int my_row = kk < a.K ? a.dst_row[(int64_t)t * a.K + kk] : -1;
        const float my_w = (a.w && kk < a.K) ? a.w[(int64_t)t * a.w_stride + kk] : 1.0f;
        const int64_t my_off = entry_row_offset(a, t, kk, my_row);
        const uint64_t mask = __ballot(my_off >= 0);  // the entries that have rows
        const int left = (int)__popcll(mask), nk = min(kWave, a.K - k0);
        if (left == nk) gather_all<true, SEGS>(mask, left, my_off, my_w, base, second, acc);  // all of them: the usual case
        else gather_all<false, SEGS>(mask, left, my_off, my_w, base, second, acc);
    }
#pragma unroll
    for (int q = 0; q < SEGS; ++q) {
        if (unit + q * kWave < units) {
            u32x4 o;
#pragma unroll
            for (int c = 0; c < 4; ++c) o[c] = pack_bf16(acc[q][2 * c], acc[q][2 * c + 1]);
            __builtin_nontemporal_store(o, (u32x4*)(a.out + (int64_t)t * a.out_stride) + unit + q * kWave);
        }
    }
}

// One wavefront reduces a whole token row of NSEG segments of 1 KiB (rows of exactly that length;
// NSEG = 14 is the 14 336-byte row of Sec. IV-B): one index fetch per token instead of one per
// segment, and the output row leaves in one piece.  112 accumulators and the 14 loads of a row
// fill the registers, so the entries are taken one after the other; the compiler moves the next
// row's loads up as far as they fit (straight-line code for the usual token: eight entries, all
// with rows).  A few per cent faster than the segment kernels once the launch has thousands of
// tokens; anything else -- other row lengths, short launches -- uses those.
template <int NSEG>
__device__ __forceinline__ void add_row(float (&acc)[NSEG][8], const uint8_t* p, float wk) {
    u32x4 v[NSEG];
#pragma unroll
    for (int q = 0; q < NSEG; ++q) v[q] = __builtin_nontemporal_load((const u32x4*)(p + q * 1024));
#pragma unroll
    for (int q = 0; q < NSEG; ++q) accumulate(acc[q], v[q], wk);
}

template <int NSEG>
__global__ __launch_bounds__(256) void combine_row_kernel(CombineArgs a) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int t = blockIdx.x * 4 + wave;
    if (t >= a.T) return;
    const uint8_t* base = (const uint8_t*)a.win.base + lane * 16;
    // lane j holds row index and weight of entry j (K <= 64) and works out where the row lies
    const int my_row = lane < a.K ? a.dst_row[(int64_t)t * a.K + lane] : -1;
    const float my_w = (a.w && lane < a.K) ? a.w[(int64_t)t * a.w_stride + lane] : 1.0f;
    const int64_t my_off = entry_row_offset(a, t, lane, my_row);
    uint64_t mask = __ballot(my_off >= 0);  // the entries that have rows
    float acc[NSEG][8];
#pragma unroll
    for (int q = 0; q < NSEG; ++q)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[q][c] = 0.0f;
    if (mask == 0xffu) {  // entries 0..7 and no others: straight-line
#pragma unroll
        for (int j = 0; j < 8; ++j)
            add_row<NSEG>(acc, base + readlane64(my_off, j), __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), j)));
    } else {
        while (mask) {  // lowest k first
            const int src = __builtin_ctzll(mask);
            mask &= mask - 1;
            add_row<NSEG>(acc, base + readlane64(my_off, src), __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), src)));
        }
    }
    u32x4* o = (u32x4*)(a.out + (int64_t)t * a.out_stride) + lane;
#pragma unroll
    for (int q = 0; q < NSEG; ++q) {
        u32x4 r;
#pragma unroll
        for (int c = 0; c < 4; ++c) r[c] = pack_bf16(acc[q][2 * c], acc[q][2 * c + 1]);
        __builtin_nontemporal_store(r, o + q * kWave);
    }
}

// Two-level summation order (Sec. V-A: partial results are accumulated within a node
// first, then reduced across nodes): for every node in ascending order the products of
// the entries whose expert lives in that node are summed in ascending k, and the node
// sums are added in ascending node order; all in float32, one rounding to bf16 at the
// end.  Same bytes moved as the flat kernel.
__global__ __launch_bounds__(256) void combine_hier_kernel(CombineArgs a, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (u >= (int64_t)a.T * nseg) return;
    const int t = (int)(u / nseg);
    const int seg = (int)(u - (int64_t)t * nseg);
    const int unit = seg * kWave + lane;
    const bool active = unit < units;
    int my_row = lane < a.K ? a.dst_row[(int64_t)t * a.K + lane] : -1;
    if (my_row >= a.win.rows_cap) my_row = -1;
    const float my_w = (a.w && lane < a.K) ? a.w[(int64_t)t * a.w_stride + lane] : 1.0f;
    const int my_rank = lane < a.K ? a.entry_rank[(int64_t)t * a.K + lane] : -1;
    const int my_node = (my_row >= 0 && my_rank >= 0) ? my_rank / a.ranks_per_node : -1;
    float total[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) total[c] = 0.0f;
    for (int n = 0; n < a.nodes; ++n) {
        uint64_t members = __ballot(my_node == n);  // the k's of this node, ascending = bit order
        if (members == 0) continue;
        float part[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) part[c] = 0.0f;
        while (members) {
            u32x4 v[KB];
            float wk[KB];
            bool has[KB];
#pragma unroll
            for (int j = 0; j < KB; ++j) {
                has[j] = members != 0;
                v[j] = (u32x4){0u, 0u, 0u, 0u};
                wk[j] = 0.0f;
                if (has[j]) {
                    const int k = __builtin_ctzll(members);
                    members &= members - 1;
                    int r = __builtin_amdgcn_readlane(my_row, k);
                    wk[j] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), k));
                    if (a.staged) r = t * a.K + k;
                    const int64_t off = a.staged ? (int64_t)r * a.H : window_offset(a.win, r);
                    if (active) v[j] = __builtin_nontemporal_load((const u32x4*)(a.win.base + off) + unit);
                }
            }
#pragma unroll
            for (int j = 0; j < KB; ++j)
                if (has[j]) accumulate(part, v[j], wk[j]);
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) total[c] = __fadd_rn(total[c], part[c]);
    }
    if (active) {
        u32x4 o;
#pragma unroll
        for (int c = 0; c < 4; ++c) o[c] = pack_bf16(total[2 * c], total[2 * c + 1]);
        __builtin_nontemporal_store(o, (u32x4*)(a.out + (int64_t)t * a.out_stride) + unit);
    }
}

// Backward pass of the weighted combine (Sec. III-F training pattern: the handle of the
// forward pass is reused).  With out[t] = sum_k w[t,k] * y[row(t,k)], the gradient g = d/d out
// gives
//   grad_y[row(t,k), h] = bf16_rne( w[t,k] * f32(g[t,h]) )      (a dispatch of g scaled per entry)
//   grad_w[t,k]         = sum_h f32(y[row(t,k), h]) * f32(g[t,h])
// One workgroup per token.  Its threads walk the row 256 16-byte units at a time; a thread
// loads its unit of g once and then, for up to 8 entries together, issues the loads of the
// entries' y rows before it uses any of them (8 independent 16-byte loads in flight per
// lane, as in the forward kernel), stores the scaled gradient to the entries' rows and adds
// its products to one float32 sum per entry.  The sums of an entry batch are reduced once:
// the 64 lanes of a wave by a fixed exchange tree, the four waves in order through LDS -- a
// fixed order, so the result does not depend on timing.  Entries without a row get
// grad_w = 0 and write nothing.  Bound by HBM: per entry one row read and one written.
constexpr int KBB = 8;  // entries handled together

__global__ __launch_bounds__(256) void combine_backward_kernel(CombineArgs a, const uint16_t* g, int64_t g_stride,
                                                               WindowDesc gy, float* grad_w, int64_t gw_stride, int units) {
    __shared__ float part[4][KBB];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const u32x4* grow = (const u32x4*)(g + (int64_t)t * g_stride);
    for (int k0 = 0; k0 < a.K; k0 += kWave) {  // the entries of the token, 64 at a time in the lanes of a wave
        const int kk = k0 + lane;
        int my_row = kk < a.K ? a.dst_row[(int64_t)t * a.K + kk] : -1;
        if (my_row >= a.win.rows_cap) my_row = -1;
        const float my_w = (a.w && kk < a.K) ? a.w[(int64_t)t * a.w_stride + kk] : 1.0f;
        const int nk = min(kWave, a.K - k0);
        for (int j0 = 0; j0 < nk; j0 += KBB) {
            // wave-uniform per entry of the batch: row, weight, the row's addresses
            int row[KBB];
            float w[KBB];
            const u32x4* yrow[KBB];
            u32x4* gyrow[KBB];
            float dot[KBB];
#pragma unroll
            for (int b = 0; b < KBB; ++b) {
                const int j = j0 + b;  // lanes >= nk hold no row
                row[b] = __builtin_amdgcn_readlane(my_row, j & (kWave - 1));
                if (j >= nk) row[b] = -1;
                w[b] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), j & (kWave - 1)));
                const int r = max(row[b], 0);
                yrow[b] = a.win.base ? (const u32x4*)(a.win.base + window_offset(a.win, r)) : nullptr;
                gyrow[b] = (u32x4*)(gy.base + window_offset(gy, r));
                dot[b] = 0.0f;
            }
            for (int u = threadIdx.x; u < units; u += blockDim.x) {
                const u32x4 gv = grow[u];
                u32x4 yv[KBB];
                if (a.win.base) {
#pragma unroll
                    for (int b = 0; b < KBB; ++b)
                        if (row[b] >= 0) yv[b] = __builtin_nontemporal_load(yrow[b] + u);
                }
                float gf[8];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    gf[2 * c] = bf16_lo(gv[c]);
                    gf[2 * c + 1] = bf16_hi(gv[c]);
                }
#pragma unroll
                for (int b = 0; b < KBB; ++b) {
                    if (row[b] < 0) continue;  // wave-uniform
                    u32x4 o;
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        o[c] = pack_bf16(__fmul_rn(w[b], gf[2 * c]), __fmul_rn(w[b], gf[2 * c + 1]));
                    __builtin_nontemporal_store(o, gyrow[b] + u);
                }
                if (a.win.base) {
#pragma unroll
                    for (int b = 0; b < KBB; ++b) {
                        if (row[b] < 0) continue;
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            dot[b] = __fadd_rn(dot[b], __fmul_rn(bf16_lo(yv[b][c]), gf[2 * c]));
                            dot[b] = __fadd_rn(dot[b], __fmul_rn(bf16_hi(yv[b][c]), gf[2 * c + 1]));
                        }
                    }
                }
            }
            if (grad_w) {  // uniform over the workgroup: every thread takes part
#pragma unroll
                for (int b = 0; b < KBB; ++b) {
                    float d = dot[b];
                    for (int off = kWave / 2; off > 0; off >>= 1) d = __fadd_rn(d, __shfl_xor(d, off, kWave));
                    if (lane == 0) part[wave][b] = d;
                }
                __syncthreads();
                if (threadIdx.x < KBB && j0 + (int)threadIdx.x < nk) {
                    const int b = threadIdx.x;
                    grad_w[(int64_t)t * gw_stride + k0 + j0 + b] =
                        __fadd_rn(__fadd_rn(__fadd_rn(part[0][b], part[1][b]), part[2][b]), part[3][b]);
                }
                __syncthreads();
            }
        }
    }
}

}  // namespace

hipError_t launch_combine_backward(const CombineArgs& a, const uint16_t* g, int64_t g_stride, const WindowDesc& gy,
                                   float* grad_w, int64_t gw_stride, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    hipLaunchKernelGGL(combine_backward_kernel, dim3((unsigned)a.T), dim3(256), 0, s, a, g, g_stride, gy, grad_w, gw_stride,
                       a.H / 8);
    return hipGetLastError();
}

// From this many wavefronts of one segment each on, a launch takes two segments per wavefront.
constexpr int64_t kTwoSegmentMinWaves = 16384;
constexpr int kRowSegments = 14;

// Compute units of the current device (0 when it cannot be asked).
static int current_compute_units() {
    static std::atomic<int> cus[64];  // per device, 0 = not asked yet (any thread may fill it in)
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
        cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Rows of exactly kRowSegments segments go whole to one wavefront when the tokens fill the GPU
// in whole rounds of resident wavefronts, or nearly (the whole-row kernel holds two wavefronts
// per SIMD -- its 230 registers -- and a compute unit has four SIMDs): a last round that is half
// empty costs more than the whole-row kernel gains over the segment kernels (T = 2560 on 256
// compute units: 65 us against 59 us; T = 4096: 91 against 94).
void plan_combine(int64_t T, int H, int ranks_per_node, int compute_units, CombinePlan* out) {
    const int units = H / 8;
    const int nseg = (units + kWave - 1) / kWave;
    int64_t nwaves = T * nseg;
    const bool flat = ranks_per_node <= 0;
    const int64_t slots = (int64_t)compute_units * 8;
    bool whole = false;
    if (flat && units == kRowSegments * kWave && slots > 0 && T >= slots) {
        const int64_t rounds = T / slots, rest = T % slots;
        whole = rest == 0 || rounds >= 3 || rest * 8 >= slots * 7;
    }
    const bool two = flat && !whole && nseg % 2 == 0 && nwaves >= kTwoSegmentMinWaves;
    if (whole) nwaves = T;
    if (two) nwaves /= 2;
    out->segments = whole ? kRowSegments : two ? 2 : 1;
    out->whole_row = whole ? 1 : 0;
    out->workgroups = (nwaves + 3) / 4;
}

hipError_t launch_combine(const CombineArgs& a, hipStream_t s) {
    const int units = a.H / 8;
    const int nseg = (units + kWave - 1) / kWave;
    if ((int64_t)a.T * nseg == 0) return hipSuccess;
    CombinePlan p;
    plan_combine(a.T, a.H, a.ranks_per_node, current_compute_units(), &p);
    const int64_t nblk = p.workgroups;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.ranks_per_node > 0)
        hipLaunchKernelGGL(combine_hier_kernel, dim3((unsigned)nblk), dim3(256), 0, s, a, nseg, units);
    else if (p.whole_row)
        hipLaunchKernelGGL(combine_row_kernel<kRowSegments>, dim3((unsigned)nblk), dim3(256), 0, s, a);
    else if (p.segments == 2)
        hipLaunchKernelGGL(combine_kernel<2>, dim3((unsigned)nblk), dim3(256), 0, s, a, nseg, units);
    else
        hipLaunchKernelGGL(combine_kernel<1>, dim3((unsigned)nblk), dim3(256), 0, s, a, nseg, units);
    return hipGetLastError();
}

}  // namespace ep
