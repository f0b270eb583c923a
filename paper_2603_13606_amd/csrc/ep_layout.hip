// Routing layout kernels: per-expert / per-destination-rank counts, prefix
// offsets and the stable slot map (Sec. IV-A index algebra; Sec. IV-C "Token
// Count"; the slot rule of Sec. IV-B made deterministic).
//
// The slot of entry i = t*K + k is the number of entries j < i naming the same
// expert: a stable counting sort.  The flattened entry list is cut into chunks,
// one per workgroup, and every chunk into wave-chunks of 64*passes consecutive
// entries, one per wavefront.
//   count kernel  each workgroup histograms its chunk (bins: E experts, masked,
//                 invalid, R destination ranks) with LDS integer atomics --
//                 counts do not depend on the order of the additions;
//   slot kernel   each workgroup sums the histograms of the chunks before it
//                 (its prefix) and of all chunks (the totals, hence the expert
//                 offsets), histograms its own wave-chunks again to split the
//                 prefix per wave, then each wave walks its entries 64 at a
//                 time: slot = prefix of the bin + number of lower lanes with
//                 the same key, found with one ballot per key bit.
// No atomic decides an order anywhere, so the output is a pure function of the
// input.  Inputs of at most 4096 entries run both steps inside one workgroup.
//
// The same kernels serve the receiving side of the once-per-rank dispatch
// (Sec. IV-D): there the entries are the routing vectors found in the headers of
// the staged messages, in window order, filtered to the experts the window's
// rank hosts (Sec. IV-C "Dispatch/recv").
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
    bool ok;       // names an expert that gets a row
    bool masked;   // id == -1
    bool invalid;  // any other id outside [0, E)
    bool lead;     // first k of its token that names destination rank d
};

// Message mode: which destination rank's window holds staging slot m, and is the
// slot in use.  mroff / mcnt are LDS copies of rank_offset / rank_token_count.
__device__ __forceinline__ bool msg_slot_rank(const LayoutArgs& a, int m, const int32_t* mroff,
                                              const int32_t* mcnt, int* d_out) {
    if (m >= a.msg_total_slots) return false;
    if (a.msg_slots_per_rank > 0) {  // fixed-size window per rank
        const int d = m / a.msg_slots_per_rank;
        *d_out = d;
        return (m - d * a.msg_slots_per_rank) < mcnt[d];
    }
    if (m >= mroff[a.R]) return false;  // compact windows: [rank_offset[d], rank_offset[d+1])
    int lo = 0, hi = a.R;               // largest d with rank_offset[d] <= m
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (mroff[mid] <= m) lo = mid; else hi = mid;
    }
    *d_out = lo;
    return true;
}

__device__ __forceinline__ Entry load_entry(const LayoutArgs& a, int i, const int32_t* mroff,
                                            const int32_t* mcnt) {
    Entry en;
    en.t = 0; en.k = 0; en.e = 0; en.d = 0;
    en.ok = en.masked = en.invalid = en.lead = false;
    if (i >= a.n) return en;
    en.t = i / a.K;
    en.k = i - en.t * a.K;
    if (a.msgs) {
        int d = 0;
        if (!msg_slot_rank(a, en.t, mroff, mcnt, &d)) return en;
        const int32_t* hdr = (const int32_t*)(a.msgs + (int64_t)en.t * a.msg_bytes);
        const int e = hdr[1 + en.k];
        en.ok = (unsigned)e < (unsigned)a.E && owner_of(a, e) == d;
        en.e = en.ok ? e : 0;
        en.d = d;
        return en;
    }
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
    return en;
}

// Histogram of one wave-chunk into h[0..W) with LDS atomics (integer adds: the
// result does not depend on their order).
__device__ void wave_hist(const LayoutArgs& a, int wc, int32_t* h, int lane, const int32_t* mroff,
                          const int32_t* mcnt) {
    for (int p = 0; p < a.passes; ++p) {
        const int i = (wc * a.passes + p) * kWave + lane;
        const Entry en = load_entry(a, i, mroff, mcnt);
        if (en.ok) atomicAdd(&h[en.e], 1);
        if (en.masked) atomicAdd(&h[a.E], 1);
        if (en.invalid) atomicAdd(&h[a.E + 1], 1);
        if (en.lead) atomicAdd(&h[a.E + 2 + en.d], 1);
    }
}

// Slot assignment for one wave-chunk: h holds, per bin, the number of entries of
// that bin before this wave-chunk; it is advanced as the chunk is walked.
__device__ void wave_slots(const LayoutArgs& a, int wc, int32_t* h, const int32_t* eoff,
                           const int32_t* opre, const int32_t* roff, int lane, const int32_t* mroff,
                           const int32_t* mcnt) {
    const uint64_t lt = (1ull << lane) - 1ull;
    for (int p = 0; p < a.passes; ++p) {
        const int i = (wc * a.passes + p) * kWave + lane;
        const Entry en = load_entry(a, i, mroff, mcnt);
        const uint64_t peers = match_key(en.e, en.ok, a.bits_e);
        const uint64_t peers_r = a.msgs ? 0ull : match_key(en.d, en.lead, a.bits_r);
        const int rank = __popcll(peers & lt);
        const int rank_r = __popcll(peers_r & lt);
        int slot = -1, row = -1, rrow = -1;
        if (en.ok) {
            slot = h[en.e] + rank;
            if (a.padded) row = slot < a.C ? en.e * a.C + slot : -1;
            else row = eoff[en.e] + slot;
            if (a.sorted_token) {
                const int pos = opre[en.e] + slot;
                a.sorted_token[pos] = en.t;
                a.sorted_k[pos] = en.k;
                a.sorted_row[pos] = row;
            }
        }
        if (en.lead) rrow = roff[en.d] + h[a.E + 2 + en.d] + rank_r;
        if (i < a.n) {
            if (a.slot) a.slot[i] = slot;
            a.dst_row[i] = row;
            if (a.rank_row) a.rank_row[i] = rrow;
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

// From the column totals tot[0..W): offsets for the slot walk (in LDS) and, when
// write_global is set, the per-expert / per-rank arrays and the totals block.
// red: 4 ints of LDS for reductions.  Ends with a barrier.
__device__ void finalize_counts(const LayoutArgs& a, const int32_t* tot, int32_t* eoff,
                                int32_t* opre, int32_t* roff, int32_t* tmp, int32_t* red,
                                bool write_global) {
    const int tid = threadIdx.x, nth = blockDim.x;
    if (tid < 4) red[tid] = 0;
    block_exclusive_scan(tot, opre, a.E, tmp);  // own_prefix: scan of the demand per expert
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
    if (a.padded) {  // staging windows: one region per destination rank
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
        if (a.rank_pair_count) {
            for (int d = tid; d < a.R; d += nth) {
                int s = 0;
                for (int l = 0; l < a.L; ++l) s += tot[d * a.L + l];
                a.rank_pair_count[d] = s;
                a.rank_token_count[d] = tot[a.E + 2 + d];
            }
            for (int d = tid; d <= a.R; d += nth) a.rank_offset[d] = roff[d];
        }
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

// LDS carve-up shared by the kernels: [nw][W] wave histograms, tot[W], eoff[E+1],
// opre[E+1], roff[R+1], mroff[R+1], mcnt[R], tmp[nw+1], red[4].
struct Lds {
    int32_t *wh, *tot, *eoff, *opre, *roff, *mroff, *mcnt, *tmp, *red;
};

__device__ __forceinline__ Lds carve_lds(int32_t* base, const LayoutArgs& a, int nw) {
    Lds l;
    l.wh = base;
    l.tot = l.wh + nw * a.W;
    l.eoff = l.tot + a.W;
    l.opre = l.eoff + a.E + 1;
    l.roff = l.opre + a.E + 1;
    l.mroff = l.roff + a.R + 1;
    l.mcnt = l.mroff + a.R + 1;
    l.tmp = l.mcnt + a.R;
    l.red = l.tmp + nw + 1;
    return l;
}

size_t lds_bytes(const LayoutArgs& a, int nw) {
    return sizeof(int32_t) * ((size_t)nw * a.W + a.W + 2 * (a.E + 1) + 2 * (a.R + 1) + a.R + nw + 1 + 4);
}

__device__ __forceinline__ void stage_msg_tables(const LayoutArgs& a, const Lds& l) {
    if (!a.msgs) return;
    for (int d = threadIdx.x; d <= a.R; d += blockDim.x) l.mroff[d] = a.msg_rank_offset[d];
    for (int d = threadIdx.x; d < a.R; d += blockDim.x) l.mcnt[d] = a.msg_rank_count[d];
}

// ---- one-launch path: everything inside one workgroup of kFusedWaves waves ----
__global__ __launch_bounds__(kFusedWaves* kWave) void layout_fused_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const Lds l = carve_lds(lds, a, kFusedWaves);
    const int W = a.W;
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int j = tid; j < kFusedWaves * W; j += blockDim.x) l.wh[j] = 0;
    stage_msg_tables(a, l);
    __syncthreads();
    if (w < a.nwc) wave_hist(a, w, l.wh + w * W, lane, l.mroff, l.mcnt);
    __syncthreads();
    for (int c = tid; c < W; c += blockDim.x) {
        int run = 0;
        for (int r = 0; r < kFusedWaves; ++r) {
            const int v = l.wh[r * W + c];
            l.wh[r * W + c] = run;
            run += v;
        }
        l.tot[c] = run;
    }
    __syncthreads();
    finalize_counts(a, l.tot, l.eoff, l.opre, l.roff, l.tmp, l.red, true);
    if (w < a.nwc) wave_slots(a, w, l.wh + w * W, l.eoff, l.opre, l.roff, lane, l.mroff, l.mcnt);
}

// ---- two-launch path -------------------------------------------------------------
// Chunk b = wave-chunks [b*wpb, (b+1)*wpb).  Writes hist[b][0..W).
__global__ void layout_count_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int wpb = blockDim.x >> 6;
    const Lds l = carve_lds(lds, a, 1);
    const int W = a.W;
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = blockIdx.x * wpb + w;
    for (int j = tid; j < W; j += blockDim.x) l.wh[j] = 0;
    stage_msg_tables(a, l);
    __syncthreads();
    if (wc < a.nwc) wave_hist(a, wc, l.wh, lane, l.mroff, l.mcnt);
    __syncthreads();
    int32_t* g = a.hist + (int64_t)blockIdx.x * W;
    for (int j = tid; j < W; j += blockDim.x) g[j] = l.wh[j];
}

__global__ void layout_slot_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int wpb = blockDim.x >> 6;
    const Lds l = carve_lds(lds, a, wpb);
    const int W = a.W;
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = blockIdx.x * wpb + w;
    const int nchunks = gridDim.x;
    // Row 0 of wh will hold the chunk prefix (entries of each bin in earlier chunks);
    // rows 1..wpb-1 first receive the histograms of this chunk's waves 0..wpb-2.
    for (int j = tid; j < (wpb - 1) * W; j += blockDim.x) l.wh[W + j] = 0;
    stage_msg_tables(a, l);
    __syncthreads();
    if (w < wpb - 1 && wc < a.nwc) wave_hist(a, wc, l.wh + (w + 1) * W, lane, l.mroff, l.mcnt);
    for (int c = tid; c < W; c += blockDim.x) {
        int before = 0, total = 0;
        const int32_t* col = a.hist + c;
#pragma unroll 8
        for (int r = 0; r < nchunks; ++r) {
            const int v = col[(int64_t)r * W];
            total += v;
            if (r < (int)blockIdx.x) before += v;
        }
        l.tot[c] = total;
        l.wh[c] = before;
    }
    __syncthreads();
    // running sum down the rows: row r = entries of the bin before wave r of this chunk
    for (int c = tid; c < W; c += blockDim.x) {
        int run = l.wh[c];
        for (int r = 1; r < wpb; ++r) {
            const int v = l.wh[r * W + c];
            run += v;
            l.wh[r * W + c] = run;
        }
    }
    __syncthreads();
    finalize_counts(a, l.tot, l.eoff, l.opre, l.roff, l.tmp, l.red, blockIdx.x == 0);
    if (wc < a.nwc) wave_slots(a, wc, l.wh + w * W, l.eoff, l.opre, l.roff, lane, l.mroff, l.mcnt);
}

constexpr size_t kLdsLimit = 64 * 1024;

}  // namespace

// Wave-chunk plan for n entries: small inputs fit one workgroup of kFusedWaves
// waves; larger ones use at most kMaxWaveChunks wave-chunks.
void plan_layout(int n, int* passes, int* nwc) {
    const int max_wc = n <= kFusedMaxEntries ? kFusedWaves : kMaxWaveChunks;
    int p = (n + kWave * max_wc - 1) / (kWave * max_wc);
    if (p < 1) p = 1;
    *passes = p;
    *nwc = (n + kWave * p - 1) / (kWave * p);
}

hipError_t launch_layout(const LayoutArgs& a, hipStream_t s) {
    if (a.n <= kFusedMaxEntries && a.nwc <= kFusedWaves && lds_bytes(a, kFusedWaves) <= kLdsLimit) {
        hipLaunchKernelGGL(layout_fused_kernel, dim3(1), dim3(kFusedWaves * kWave),
                           lds_bytes(a, kFusedWaves), s, a);
        return hipGetLastError();
    }
    int wpb = 4;
    while (wpb > 1 && lds_bytes(a, wpb) > kLdsLimit) wpb >>= 1;
    if (lds_bytes(a, wpb) > kLdsLimit) return hipErrorInvalidValue;
    int nblk = (a.nwc + wpb - 1) / wpb;
    if (nblk < 1) nblk = 1;
    if (nblk > kMaxWaveChunks) return hipErrorInvalidValue;
    hipLaunchKernelGGL(layout_count_kernel, dim3(nblk), dim3(wpb * kWave), lds_bytes(a, 1), s, a);
    hipLaunchKernelGGL(layout_slot_kernel, dim3(nblk), dim3(wpb * kWave), lds_bytes(a, wpb), s, a);
    return hipGetLastError();
}

}  // namespace ep
