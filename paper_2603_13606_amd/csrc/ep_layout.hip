// Routing layout kernels: per-expert / per-destination-rank counts, prefix
// offsets and the stable slot map (Sec. IV-A index algebra; Sec. IV-C "Token
// Count"; the slot rule of Sec. IV-B made deterministic).
//
// The slot of entry i = t*K + k is the number of entries j < i naming the same
// expert: a stable counting sort.  The flattened entry list is cut into
// wave-chunks of 64*passes consecutive entries, one per wavefront:
//   A  each wave builds the histogram of its chunk (bins: E experts, masked,
//      invalid, R destination ranks) using a ballot-based in-wave match;
//   B  a column-wise exclusive scan over the wave-chunks turns the histograms
//      into "entries of this bin before this chunk";
//   C  each wave re-reads its chunk and ranks entries inside the wave with the
//      same ballot match, so slot = chunk prefix + rank of the lane.
// No atomics decide an order anywhere, so the result is a pure function of the
// input.  Small inputs run A, B and C inside one workgroup (one launch).
#include "ep_internal.h"

namespace ep {
namespace {

__device__ __forceinline__ int lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Lanes (among those with valid == true) that hold the same key as this lane.
__device__ __forceinline__ uint64_t match_key(int key, bool valid, int nbits) {
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (key >> b) & 1;
        const uint64_t bal = __ballot(valid && bit);
        peers &= bit ? bal : ~bal;
    }
    return valid ? peers : 0ull;
}

__device__ __forceinline__ int owner_of(const LayoutArgs& a, int e) {
    return a.L_shift >= 0 ? (e >> a.L_shift) : (e / a.L);
}

struct Entry {
    int t, k, e, d;
    bool ok;       // expert id in [0, E)
    bool masked;   // id == -1
    bool invalid;  // any other id
    bool lead;     // first k of its token that names destination rank d
};

__device__ __forceinline__ Entry load_entry(const LayoutArgs& a, int i) {
    Entry en;
    en.t = 0; en.k = 0; en.e = 0; en.d = 0;
    en.ok = en.masked = en.invalid = en.lead = false;
    if (i < a.n) {
        en.t = i / a.K;
        en.k = i - en.t * a.K;
        const int32_t* row = a.topk + (int64_t)en.t * a.topk_stride;
        en.e = row[en.k];
        en.ok = (unsigned)en.e < (unsigned)a.E;
        en.masked = en.e == -1;
        en.invalid = !en.ok && !en.masked;
        if (en.ok) {
            en.d = owner_of(a, en.e);
            en.lead = true;
            for (int k2 = 0; k2 < en.k; ++k2) {
                const int e2 = row[k2];
                if ((unsigned)e2 < (unsigned)a.E && owner_of(a, e2) == en.d) en.lead = false;
            }
        } else {
            en.e = 0;
        }
    }
    return en;
}

// Phase A for one wave-chunk: h[0..W) must be zero on entry.
__device__ void phase_hist(const LayoutArgs& a, int wc, int32_t* h, int lane) {
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int p = 0; p < a.passes; ++p) {
        const int i = (wc * a.passes + p) * kWave + lane;
        const Entry en = load_entry(a, i);
        const uint64_t peers = match_key(en.e, en.ok, a.bits_e);
        if (en.ok && (peers & lt) == 0) h[en.e] += __popcll(peers);
        const uint64_t bm = __ballot(en.masked);
        const uint64_t bi = __ballot(en.invalid);
        if (lane == 0) {
            h[a.E] += __popcll(bm);
            h[a.E + 1] += __popcll(bi);
        }
        const uint64_t peers_r = match_key(en.d, en.lead, a.bits_r);
        if (en.lead && (peers_r & lt) == 0) h[a.E + 2 + en.d] += __popcll(peers_r);
        wave_fence();
    }
}

// Phase C for one wave-chunk: h holds, per bin, the number of entries of that
// bin in earlier chunks; it is advanced as the chunk is walked.
__device__ void phase_slot(const LayoutArgs& a, int wc, int32_t* h, const int32_t* eoff,
                           const int32_t* opre, const int32_t* roff, int lane) {
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int p = 0; p < a.passes; ++p) {
        const int i = (wc * a.passes + p) * kWave + lane;
        const Entry en = load_entry(a, i);
        const uint64_t peers = match_key(en.e, en.ok, a.bits_e);
        const uint64_t peers_r = match_key(en.d, en.lead, a.bits_r);
        const int rank = __popcll(peers & lt);
        const int rank_r = __popcll(peers_r & lt);
        int slot = -1, row = -1, rrow = -1;
        if (en.ok) {
            slot = h[en.e] + rank;
            if (a.padded) row = slot < a.C ? en.e * a.C + slot : -1;
            else row = eoff[en.e] + slot;
            const int pos = opre[en.e] + slot;
            a.sorted_token[pos] = en.t;
            a.sorted_k[pos] = en.k;
            a.sorted_row[pos] = row;
        }
        if (en.lead) rrow = roff[en.d] + h[a.E + 2 + en.d] + rank_r;
        if (i < a.n) {
            a.slot[i] = slot;
            a.dst_row[i] = row;
            a.rank_row[i] = rrow;
        }
        wave_fence();
        if (en.ok && rank == 0) h[en.e] += __popcll(peers);
        if (en.lead && rank_r == 0) h[a.E + 2 + en.d] += __popcll(peers_r);
        wave_fence();
    }
}

// Exclusive scan of in[0..n) into out[0..n], out[n] = total, by the whole block.
// tmp needs blockDim.x / 64 + 1 ints.  Ends with a barrier.
__device__ void block_exclusive_scan(const int32_t* in, int32_t* out, int n, int32_t* tmp) {
    const int tid = threadIdx.x, nth = blockDim.x;
    const int lane = tid & (kWave - 1), w = tid >> 6, nw = (nth + kWave - 1) >> 6;
    const int ipt = (n + nth - 1) / nth;
    const int start = tid * ipt;
    int sum = 0;
    for (int j = 0; j < ipt; ++j) {
        const int idx = start + j;
        if (idx < n) sum += in[idx];
    }
    int inc = sum;
    for (int off = 1; off < kWave; off <<= 1) {
        const int v = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += v;
    }
    if (lane == kWave - 1) tmp[w] = inc;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int j = 0; j < nw; ++j) { const int v = tmp[j]; tmp[j] = run; run += v; }
        tmp[nw] = run;
    }
    __syncthreads();
    int run = tmp[w] + inc - sum;
    for (int j = 0; j < ipt; ++j) {
        const int idx = start + j;
        if (idx < n) { const int v = in[idx]; out[idx] = run; run += v; }
    }
    if (tid == 0) out[n] = tmp[nw];
    __syncthreads();
}

// From the column totals tot[0..W): offsets for phase C (in LDS) and, when
// write_global is set, the per-expert / per-rank arrays and the totals block.
// red: 4 ints of LDS for reductions.  Ends with a barrier.
__device__ void finalize_counts(const LayoutArgs& a, const int32_t* tot, int32_t* eoff,
                                int32_t* opre, int32_t* roff, int32_t* tmp, int32_t* red,
                                bool write_global) {
    const int tid = threadIdx.x, nth = blockDim.x;
    if (tid < 4) red[tid] = 0;
    // own_prefix: exclusive scan of the demand per expert
    block_exclusive_scan(tot, opre, a.E, tmp);
    if (a.padded) {
        for (int e = tid; e <= a.E; e += nth) eoff[e] = e * a.C;
    } else if (a.expert_base) {
        for (int e = tid; e < a.E; e += nth) {
            const int b = a.expert_base[e];
            eoff[e] = b;
            if (tot[e] > 0) atomicMax(&red[2], b + tot[e]);
        }
    } else {
        for (int e = tid; e <= a.E; e += nth) eoff[e] = opre[e];
    }
    // staging windows: one region per destination rank
    if (a.padded) {
        for (int d = tid; d <= a.R; d += nth) roff[d] = d * a.C_rank;
        __syncthreads();
    } else {
        block_exclusive_scan(tot + a.E + 2, roff, a.R, tmp);
    }
    int kept = 0, dropped = 0;
    for (int e = tid; e < a.E; e += nth) {
        const int c = tot[e];
        const int k = a.padded ? min(c, a.C) : c;
        kept += k;
        dropped += c - k;
        if (write_global) {
            a.expert_count[e] = c;
            a.expert_kept[e] = k;
        }
    }
    if (kept) atomicAdd(&red[0], kept);
    if (dropped) atomicAdd(&red[1], dropped);
    __syncthreads();
    if (!a.padded && a.expert_base && tid == 0) eoff[a.E] = red[2];
    __syncthreads();
    if (write_global) {
        for (int e = tid; e <= a.E; e += nth) {
            a.expert_offset[e] = eoff[e];
            a.own_prefix[e] = opre[e];
        }
        for (int d = tid; d < a.R; d += nth) {
            int s = 0;
            for (int l = 0; l < a.L; ++l) s += tot[d * a.L + l];
            a.rank_pair_count[d] = s;
            a.rank_token_count[d] = tot[a.E + 2 + d];
        }
        for (int d = tid; d <= a.R; d += nth) a.rank_offset[d] = roff[d];
        if (tid == 0) {
            int msgs = 0;
            for (int d = 0; d < a.R; ++d) msgs += tot[a.E + 2 + d];
            const int masked = tot[a.E], invalid = tot[a.E + 1];
            a.totals[TOT_KEPT] = red[0];
            a.totals[TOT_DROPPED] = red[1];
            a.totals[TOT_MASKED] = masked;
            a.totals[TOT_INVALID] = invalid;
            a.totals[TOT_SORTED] = opre[a.E];
            a.totals[TOT_MSGS] = msgs;
            a.totals[TOT_STATUS] = (invalid ? STATUS_INVALID_IDS : 0) | (red[1] ? STATUS_CAPACITY_DROP : 0);
            a.totals[TOT_ROWS_END] = eoff[a.E];
        }
    }
    __syncthreads();
}

// ---- one-launch path: everything inside one workgroup of kFusedWaves waves ----
__global__ __launch_bounds__(kFusedWaves* kWave) void layout_fused_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int W = a.W;
    int32_t* hist = lds;                     // [kFusedWaves][W]
    int32_t* tot = hist + kFusedWaves * W;   // [W]
    int32_t* eoff = tot + W;                 // [E+1]
    int32_t* opre = eoff + a.E + 1;          // [E+1]
    int32_t* roff = opre + a.E + 1;          // [R+1]
    int32_t* tmp = roff + a.R + 1;           // [kFusedWaves + 1]
    int32_t* red = tmp + kFusedWaves + 1;    // [4]
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int j = tid; j < kFusedWaves * W; j += blockDim.x) hist[j] = 0;
    __syncthreads();
    if (w < a.nwc) phase_hist(a, w, hist + w * W, lane);
    __syncthreads();
    for (int c = tid; c < W; c += blockDim.x) {
        int run = 0;
        for (int r = 0; r < kFusedWaves; ++r) {
            const int v = hist[r * W + c];
            hist[r * W + c] = run;
            run += v;
        }
        tot[c] = run;
    }
    __syncthreads();
    finalize_counts(a, tot, eoff, opre, roff, tmp, red, true);
    if (w < a.nwc) phase_slot(a, w, hist + w * W, eoff, opre, roff, lane);
}

// ---- three-launch path ---------------------------------------------------------
__global__ void layout_hist_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int W = a.W;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wpb = blockDim.x >> 6;
    const int wc = blockIdx.x * wpb + w;
    int32_t* h = lds + w * W;
    for (int j = lane; j < W; j += kWave) h[j] = 0;
    wave_fence();
    if (wc < a.nwc) {
        phase_hist(a, wc, h, lane);
        int32_t* g = a.hist + (int64_t)wc * W;
        for (int j = lane; j < W; j += kWave) g[j] = h[j];
    }
}

// Column-wise exclusive scan of hist[nwc][W]; one workgroup per 64 columns, the
// rows split into 16 segments (one per wave).
__global__ __launch_bounds__(1024) void layout_colscan_kernel(LayoutArgs a) {
    __shared__ int32_t part[16][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int seg = threadIdx.x >> 6;
    const int col = blockIdx.x * kWave + lane;
    const int rps = (a.nwc + 15) / 16;
    const int r0 = seg * rps, r1 = min(a.nwc, r0 + rps);
    const bool act = col < a.W;
    int sum = 0;
    if (act)
        for (int r = r0; r < r1; ++r) sum += a.hist[(int64_t)r * a.W + col];
    part[seg][lane] = sum;
    __syncthreads();
    int run = 0, total = 0;
    for (int s = 0; s < 16; ++s) {
        const int v = part[s][lane];
        if (s < seg) run += v;
        total += v;
    }
    if (act) {
        for (int r = r0; r < r1; ++r) {
            int32_t* p = a.hist + (int64_t)r * a.W + col;
            const int v = *p;
            *p = run;
            run += v;
        }
        if (seg == 0) a.coltotal[col] = total;
    }
}

__global__ void layout_slot_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int W = a.W;
    const int wpb = blockDim.x >> 6;
    int32_t* hbase = lds;                 // [wpb][W]
    int32_t* tot = hbase + wpb * W;       // [W]
    int32_t* eoff = tot + W;              // [E+1]
    int32_t* opre = eoff + a.E + 1;       // [E+1]
    int32_t* roff = opre + a.E + 1;       // [R+1]
    int32_t* tmp = roff + a.R + 1;        // [wpb + 1]
    int32_t* red = tmp + wpb + 1;         // [4]
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = blockIdx.x * wpb + w;
    for (int c = tid; c < W; c += blockDim.x) tot[c] = a.coltotal[c];
    if (wc < a.nwc) {
        const int32_t* g = a.hist + (int64_t)wc * W;
        int32_t* h = hbase + w * W;
        for (int j = lane; j < W; j += kWave) h[j] = g[j];
    }
    __syncthreads();
    finalize_counts(a, tot, eoff, opre, roff, tmp, red, blockIdx.x == 0);
    if (wc < a.nwc) phase_slot(a, wc, hbase + w * W, eoff, opre, roff, lane);
}

size_t fused_lds_bytes(const LayoutArgs& a) {
    return sizeof(int32_t) * ((size_t)kFusedWaves * a.W + a.W + 2 * (a.E + 1) + (a.R + 1) +
                              kFusedWaves + 1 + 4);
}

size_t slot_lds_bytes(const LayoutArgs& a, int wpb) {
    return sizeof(int32_t) * ((size_t)wpb * a.W + a.W + 2 * (a.E + 1) + (a.R + 1) + wpb + 1 + 4);
}

constexpr size_t kLdsLimit = 64 * 1024;

}  // namespace

// Wave-chunk plan for n entries: small inputs fit one workgroup of kFusedWaves
// waves; larger ones use at most kMaxWaveChunks chunks.
void plan_layout(int n, int* passes, int* nwc) {
    const int max_chunks = n <= kFusedMaxEntries ? kFusedWaves : kMaxWaveChunks;
    int p = (n + kWave * max_chunks - 1) / (kWave * max_chunks);
    if (p < 1) p = 1;
    *passes = p;
    *nwc = (n + kWave * p - 1) / (kWave * p);
}

hipError_t launch_layout(const LayoutArgs& a, hipStream_t s) {
    if (a.n <= kFusedMaxEntries && a.nwc <= kFusedWaves && fused_lds_bytes(a) <= kLdsLimit) {
        hipLaunchKernelGGL(layout_fused_kernel, dim3(1), dim3(kFusedWaves * kWave),
                           fused_lds_bytes(a), s, a);
        return hipGetLastError();
    }
    int wpb = 4;
    while (wpb > 1 && slot_lds_bytes(a, wpb) > kLdsLimit) wpb >>= 1;
    if (slot_lds_bytes(a, wpb) > kLdsLimit) return hipErrorInvalidValue;
    const int nblk = (a.nwc + wpb - 1) / wpb;
    hipLaunchKernelGGL(layout_hist_kernel, dim3(nblk), dim3(wpb * kWave),
                       sizeof(int32_t) * (size_t)wpb * a.W, s, a);
    hipLaunchKernelGGL(layout_colscan_kernel, dim3((a.W + kWave - 1) / kWave), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(layout_slot_kernel, dim3(nblk), dim3(wpb * kWave), slot_lds_bytes(a, wpb), s, a);
    return hipGetLastError();
}

}  // namespace ep
