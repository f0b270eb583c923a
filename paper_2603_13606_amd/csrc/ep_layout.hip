// Routing layout kernels: per-expert / per-destination-rank counts, prefix
// offsets and the stable slot map (Sec. IV-A index algebra; Sec. IV-C "Token
// Count"; the slot rule of Sec. IV-B made deterministic).
//
// The slot of entry i = t*K + k is the number of entries j < i naming the same
// expert: a stable counting sort.  No atomic decides an order anywhere (atomics
// only add counts or set bits), so the output is a pure function of the input.
//
// Up to 1024 entries (the decode regime): one workgroup, one entry per thread, one
// bitmap per bin; slot = popcount of the bits below the entry (layout_bitmap_kernel).
//
// Larger inputs: the flattened entry list is cut into chunks, one per workgroup of up
// to 16 wavefronts, and every chunk into wave-chunks of 64*passes consecutive entries,
// one per wavefront.
//   count kernel  (only when there is more than one chunk) each workgroup
//                 histograms its chunk -- bins: E experts, masked, invalid, R
//                 destination ranks -- with LDS integer atomics;
//   slot kernel   one thread per bin adds up the histograms of the chunks before
//                 this one (its prefix) and of all chunks (the totals, hence the
//                 expert offsets); the workgroup histograms its own wave-chunks
//                 to split the prefix per wave; every wave builds the offset
//                 tables for itself and then walks its entries 64 at a time:
//                 slot = prefix of the bin + number of lower lanes holding the
//                 same key, found with one ballot per key bit.
// The work is latency bound (a chain of dependent LDS and global round trips per
// wave), so every phase issues all of its global loads before it waits for any of
// them and the workgroup barriers order LDS traffic only.
#include "ep_internal.h"

namespace ep {
namespace {

constexpr int PU = 4;  // passes whose loads are issued together

// Workgroup barrier that orders LDS traffic only: global loads issued before it stay
// in flight across it (a full __syncthreads() would wait for them).
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
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

// Token index of flattened entry i (i / K), with a shift when K is a power of two.
__device__ __forceinline__ int token_of(const LayoutArgs& a, int i) {
    return a.K_shift >= 0 ? (i >> a.K_shift) : (i / a.K);
}

__device__ __forceinline__ int owner_of(const LayoutArgs& a, int e) {
    return a.L_shift >= 0 ? (e >> a.L_shift) : (e / a.L);
}

struct Entry {
    int i;         // flattened index, or -1 beyond the input
    int t, k, e, d;
    bool ok;       // names an expert that gets a row
    bool masked;   // id == -1
    bool invalid;  // any other id outside [0, E)
    bool lead;     // first k of its token that names destination rank d
};

// LDS carve-up shared by the kernels.
struct Lds {
    int32_t *wh;     // [nw][W] per-wave histograms, later per-wave prefixes
    int32_t *tot;    // [W] totals over the whole input
    int32_t *pre;    // [W] entries of each bin in earlier chunks
    int32_t *eoff, *opre, *roff;  // [E+1], [E+1], [R+1]
};

__device__ __forceinline__ Lds carve_lds(int32_t* base, const LayoutArgs& a, int nw) {
    Lds l;
    l.wh = base;
    l.tot = l.wh + nw * a.W;
    l.pre = l.tot + a.W;
    l.eoff = l.pre + a.W;
    l.opre = l.eoff + a.E + 1;
    l.roff = l.opre + a.E + 1;
    return l;
}

size_t lds_bytes(const LayoutArgs& a, int nw) {
    return sizeof(int32_t) * ((size_t)nw * a.W + 2 * a.W + 2 * (a.E + 1) + (a.R + 1));
}

// Marks the entries that are the first of their token to name their destination
// rank.  The entries of a token sit in consecutive lanes, so lane l compares its
// rank with the ranks held by lanes l-1 .. l-k (one cross-lane read each); only
// when a token began before lane 0 are its earlier entries read from memory.
// Must be called by all 64 lanes.
__device__ __forceinline__ void mark_leaders(const LayoutArgs& a, Entry& en, int lane) {
    const int dkey = en.ok ? en.d : -1;
    bool lead = en.ok;
    for (int j = 1; j < a.K; ++j) {
        const int prev = __shfl_up(dkey, j, kWave);
        if (j <= en.k && j <= lane && prev == dkey) lead = false;
    }
    if (en.ok && en.k > lane) {  // entries of this token that precede lane 0 of this pass
        const int32_t* row = a.topk + (int64_t)en.t * a.topk_stride;
        for (int k2 = 0; k2 < en.k - lane; ++k2) {
            const int e2 = row[k2];
            if ((unsigned)e2 < (unsigned)a.E && owner_of(a, e2) == en.d) lead = false;
        }
    }
    en.lead = lead;
}

// Issues the global loads of the ids of passes p0 .. p0+PU-1 of wave-chunk wc
// (nothing waits on them here).
__device__ __forceinline__ void issue_group(const LayoutArgs& a, int wc, int p0, int lane, int (&raw)[PU]) {
#pragma unroll
    for (int j = 0; j < PU; ++j) {
        const int p = p0 + j;
        const int i = (wc * a.passes + p) * kWave + lane;
        raw[j] = 0;
        if (p < a.passes && i < a.n) {
            const int t = token_of(a, i), k = i - t * a.K;
            raw[j] = a.topk[(int64_t)t * a.topk_stride + k];
        }
    }
}

// Classifies the ids loaded by issue_group.  Must be called by all 64 lanes.
__device__ __forceinline__ void classify_group(const LayoutArgs& a, int wc, int p0, int lane,
                                               const int (&raw)[PU], Entry (&en)[PU]) {
#pragma unroll
    for (int j = 0; j < PU; ++j) {
        Entry& x = en[j];
        const int p = p0 + j;
        const int i = (wc * a.passes + p) * kWave + lane;
        const bool in = p < a.passes && i < a.n;
        x.i = in ? i : -1;
        x.t = in ? token_of(a, i) : 0;
        x.k = in ? i - x.t * a.K : 0;
        const int e = raw[j];
        const bool inrange = (unsigned)e < (unsigned)a.E;
        x.d = inrange ? owner_of(a, e) : 0;
        x.ok = in && inrange;
        x.masked = in && e == -1;
        x.invalid = in && !inrange && e != -1;
        if (p < a.passes) mark_leaders(a, x, lane);  // wave-uniform condition
        else x.lead = false;
        x.e = x.ok ? e : 0;
    }
}

__device__ __forceinline__ void load_group(const LayoutArgs& a, int wc, int p0, int lane, Entry (&en)[PU]) {
    int raw[PU];
    issue_group(a, wc, p0, lane, raw);
    classify_group(a, wc, p0, lane, raw, en);
}

// Histogram of a loaded group into h[0..W) with LDS atomics (integer adds: the
// result does not depend on their order).
__device__ __forceinline__ void hist_group(const LayoutArgs& a, const Entry (&en)[PU], int32_t* h) {
#pragma unroll
    for (int j = 0; j < PU; ++j) {
        if (en[j].ok) atomicAdd(&h[en[j].e], 1);
        if (en[j].masked) atomicAdd(&h[a.E], 1);
        if (en[j].invalid) atomicAdd(&h[a.E + 1], 1);
        if (en[j].lead) atomicAdd(&h[a.E + 2 + en[j].d], 1);
    }
}

// Writes what the layout records for one entry, given its slot among the entries of its
// expert and (for a leader) its slot among the tokens of its destination rank.
__device__ __forceinline__ void emit_entry(const LayoutArgs& a, const Entry& x, int slot, int rslot, const Lds& l) {
    int row = -1, rrow = -1;
    if (x.ok) {
        if (a.padded) row = slot < a.C ? x.e * a.C + slot : -1;
        else row = l.eoff[x.e] + slot;
        if (a.sorted_token) {
            const int pos = l.opre[x.e] + slot;
            a.sorted_token[pos] = x.t;
            a.sorted_k[pos] = x.k;
            a.sorted_row[pos] = row;
        }
    }
    if (x.lead) rrow = l.roff[x.d] + rslot;
    if (x.i >= 0) {
        if (a.slot) a.slot[x.i] = slot;
        a.dst_row[x.i] = row;
        if (a.rank_row) a.rank_row[x.i] = rrow;
        if (a.entry_rank) a.entry_rank[x.i] = x.ok ? x.d : -1;
    }
}

// Slot assignment for a loaded group: h holds, per bin, the number of entries of
// that bin before the group; it is advanced as the group is walked.  LDS accesses
// of one wavefront are performed in program order, and the wave barriers keep the
// compiler from moving them across each other.  Must be called by all 64 lanes.
__device__ __forceinline__ void slots_group(const LayoutArgs& a, const Entry (&en)[PU], int p0, int32_t* h,
                                            const Lds& l, int lane) {
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < PU; ++j) {
        if (p0 + j >= a.passes) break;  // wave-uniform
        const Entry& x = en[j];
        const uint64_t peers = match_key(x.e, x.ok, a.bits_e);
        const uint64_t peers_r = match_key(x.d, x.lead, a.bits_r);
        const int rank = __popcll(peers & lt);
        const int rank_r = __popcll(peers_r & lt);
        const int slot = x.ok ? h[x.e] + rank : -1;
        const int rslot = x.lead ? h[a.E + 2 + x.d] + rank_r : -1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        if (x.ok && rank == 0) h[x.e] += __popcll(peers);
        if (x.lead && rank_r == 0) h[a.E + 2 + x.d] += __popcll(peers_r);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        emit_entry(a, x, slot, rslot, l);
    }
}

__device__ __forceinline__ int wave_sum(int v) {
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ int wave_max(int v) {
    for (int off = kWave / 2; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, kWave));
    return v;
}

// From the totals tot[0..W): the offset tables of the slot walk (eoff, opre, roff in
// LDS).  Runs per WAVEFRONT without any workgroup barrier:
// every wave computes the same values and stores them to the same LDS words, and
// afterwards reads only words it has stored itself.  One exclusive scan S over all W
// bins serves both prefix arrays: own_prefix[e] = S[e] and, for compact staging
// windows, rank_offset[d] = S[E+2+d] - S[E+2].  Must be called by all 64 lanes,
// after a barrier that makes tot[] final and pre[] free.
__device__ void wave_offsets(const LayoutArgs& a, const Lds& l, int lane) {
    const int32_t* tot = l.tot;
    const int W = a.W, E = a.E, R = a.R;
    const int ipt = (W + kWave - 1) / kWave;  // bins per lane, consecutive
    const int start = lane * ipt;
    constexpr int TV = 8;  // totals of up to TV own bins are kept in registers
    int tv[TV];
#pragma unroll
    for (int j = 0; j < TV; ++j) tv[j] = (j < ipt && start + j < W) ? tot[start + j] : 0;
    int sum = 0;
#pragma unroll
    for (int j = 0; j < TV; ++j) sum += tv[j];
    for (int j = TV; j < ipt; ++j)
        if (start + j < W) sum += tot[start + j];
    int inc = sum;
    for (int off = 1; off < kWave; off <<= 1) {
        const int v = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += v;
    }
    // S of the first rank bin is held by the lane that owns bin E+2
    const int owner = (E + 2) / ipt, jb = (E + 2) - owner * ipt;
    int my_rbase = inc - sum;
#pragma unroll
    for (int j = 0; j < TV; ++j)
        if (j < jb) my_rbase += tv[j];
    for (int j = TV; j < jb; ++j) my_rbase += tot[start + j];
    const int rbase = __shfl(my_rbase, owner, kWave);
    const int grand = __shfl(inc, kWave - 1, kWave);  // sum over all W bins
    int run = inc - sum;
    int32_t* S = l.pre;
    auto emit = [&](int c, int v) {
        S[c] = run;
        if (c <= E) {  // bin E is "masked": S[E] = number of routed entries
            l.opre[c] = run;
            int eo;
            if (a.padded) eo = c * a.C;
            else if (a.expert_base) eo = c < E ? a.expert_base[c] : 0;  // eoff[E] is only reported
            else eo = run;
            l.eoff[c] = eo;
        }
        if (c >= E + 2) l.roff[c - E - 2] = a.padded ? (c - E - 2) * a.C_rank : run - rbase;
        run += v;
    };
#pragma unroll
    for (int j = 0; j < TV; ++j)
        if (j < ipt && start + j < W) emit(start + j, tv[j]);
    for (int j = TV; j < ipt; ++j)
        if (start + j < W) emit(start + j, tot[start + j]);
    if (lane == 0) l.roff[R] = a.padded ? R * a.C_rank : grand - rbase;  // rank bins are the last R bins
    wave_lds_fence();
}

// The per-expert / per-rank arrays and the totals block in global memory, from the
// tables wave_offsets left in LDS.  One wavefront; must be called by all 64 lanes.
__device__ void wave_write_tables(const LayoutArgs& a, const Lds& l, int lane) {
    const int32_t* tot = l.tot;
    const int32_t* S = l.pre;
    const int E = a.E, R = a.R;
    const int total_e = S[E];
    const int msgs = S[E + 1 + R] + tot[E + 1 + R] - S[E + 2];
    int kept = 0, dropped = 0, rend = 0;
    for (int e = lane; e < E; e += kWave) {
        const int v = tot[e];
        const int k = a.padded ? min(v, a.C) : v;
        kept += k;
        dropped += v - k;
        if (!a.padded && a.expert_base && v > 0) rend = max(rend, l.eoff[e] + v);
        a.expert_count[e] = v;
        a.expert_kept[e] = k;
        a.expert_offset[e] = l.eoff[e];
        a.own_prefix[e] = l.opre[e];
        if (a.run_start) a.run_start[e] = l.opre[e];  // row 0: nothing precedes the first wave-chunk
    }
    kept = wave_sum(kept);
    dropped = wave_sum(dropped);
    rend = wave_max(rend);
    const int rows_end = a.padded ? E * a.C : (a.expert_base ? rend : total_e);
    if (a.rank_pair_count) {
        for (int d = lane; d < R; d += kWave) {
            a.rank_pair_count[d] = S[(d + 1) * a.L] - S[d * a.L];
            a.rank_token_count[d] = tot[E + 2 + d];
        }
        for (int d = lane; d <= R; d += kWave) a.rank_offset[d] = l.roff[d];
    }
    if (lane == 0) {
        const int masked = tot[E], invalid = tot[E + 1];
        a.expert_offset[E] = rows_end;
        a.own_prefix[E] = total_e;
        a.totals[TOT_KEPT] = kept;
        a.totals[TOT_DROPPED] = dropped;
        a.totals[TOT_MASKED] = masked;
        a.totals[TOT_INVALID] = invalid;
        a.totals[TOT_SORTED] = total_e;
        a.totals[TOT_MSGS] = msgs;
        a.totals[TOT_STATUS] = (invalid ? STATUS_INVALID_IDS : 0) | (dropped ? STATUS_CAPACITY_DROP : 0);
        a.totals[TOT_ROWS_END] = rows_end;
    }
}

// Extra workgroups of the slot kernel (blockIdx >= nchunks): read the token rows the caller
// announced, with ordinary cached loads, while the layout workgroups -- a few dozen on a
// part with 256 compute units -- do their latency-bound work.  wb of nwb.
// Rows [r0, r1), 16 bytes per thread and step, the workgroups side by side.
__device__ void warm_tokens(const LayoutArgs& a, int wb, int nwb, int r0, int r1) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int64_t total = (int64_t)(r1 - r0) * a.warm_units;
    const int64_t stride = (int64_t)nwb * blockDim.x;
    uint32_t acc = 0;
    for (int64_t i = (int64_t)wb * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int64_t t = r0 + i / a.warm_units;
        const int col = (int)(i % a.warm_units);
        const u32x4 v = *((const u32x4*)(a.warm_x + t * a.warm_stride) + col);
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (acc == 0x9e3779b9u) a.totals[kTotalsWords - 1] = (int32_t)acc;  // keeps the loads; the word is unused
}

// Chunk b = wave-chunks [b*wpb, (b+1)*wpb).  Writes hist[b][0..W).
__global__ __launch_bounds__(512) void layout_count_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int wpb = blockDim.x >> 6;
    const Lds l = carve_lds(lds, a, 1);
    const int W = a.W;
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = blockIdx.x * wpb + w;
    const bool active = wc < a.nwc;
    int raw[PU];
    if (active) issue_group(a, wc, 0, lane, raw);  // in flight during the LDS set-up
    for (int j = tid; j < W; j += blockDim.x) l.wh[j] = 0;
    lds_barrier();
    if (active) {
        Entry en[PU];
        for (int p0 = 0; p0 < a.passes; p0 += PU) {
            if (p0 > 0) issue_group(a, wc, p0, lane, raw);
            classify_group(a, wc, p0, lane, raw, en);
            hist_group(a, en, l.wh);
        }
    }
    lds_barrier();
    int32_t* g = a.hist + (int64_t)blockIdx.x * W;
    for (int j = tid; j < W; j += blockDim.x) g[j] = l.wh[j];
}

// With one chunk (gridDim.x == 1) this kernel is the whole layout.  MAXT = largest
// workgroup it is launched with; HB = chunk histograms whose words each thread loads
// up front (thread = bin).
template <int MAXT, int HB>
__global__ __launch_bounds__(MAXT) void layout_slot_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    if ((int)blockIdx.x >= a.nchunks) {  // a whole workgroup: no barrier below is reached by part of one
        warm_tokens(a, blockIdx.x - a.nchunks, gridDim.x - a.nchunks, 0, a.warm_rows);
        return;
    }
    const int wpb = blockDim.x >> 6;
    const Lds l = carve_lds(lds, a, wpb);
    const int W = a.W;
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = blockIdx.x * wpb + w;
    const int nchunks = a.nchunks;
    const int b = blockIdx.x;
    const bool active = wc < a.nwc;
    const bool one_group = a.passes <= PU;

    // (1) issue every global load this workgroup needs up front: its own ids and the
    //     other chunks' histograms (consumed in (3)); they stay in flight across the
    //     LDS-only barrier
    int raw[PU];
    if (active) issue_group(a, wc, 0, lane, raw);
    int hv[HB];  // column tid of the first HB chunk histograms
    const int nrows = nchunks > 1 ? nchunks : 0;
#pragma unroll
    for (int r = 0; r < HB; ++r) hv[r] = (r < nrows && tid < W) ? a.hist[(int64_t)r * W + tid] : 0;
    for (int j = tid; j < wpb * W + 2 * W; j += blockDim.x) l.wh[j] = 0;  // wh, tot, pre are contiguous
    lds_barrier();

    // (2) per-wave histograms of this chunk
    Entry en[PU];
    if (active) {
        for (int p0 = 0; p0 < a.passes; p0 += PU) {
            if (p0 > 0) issue_group(a, wc, p0, lane, raw);
            classify_group(a, wc, p0, lane, raw, en);
            hist_group(a, en, l.wh + w * W);
        }
    }
    // (3) totals over all chunks and the prefix of this chunk, per bin (thread = column)
    if (nrows > 0) {
        for (int c = tid; c < W; c += blockDim.x) {
            int before = 0, total = 0;
            if (c == tid) {
#pragma unroll
                for (int r = 0; r < HB; ++r) {
                    total += hv[r];
                    if (r < b) before += hv[r];
                }
            }
            for (int r = (c == tid ? HB : 0); r < nrows; ++r) {
                const int v = a.hist[(int64_t)r * W + c];
                total += v;
                if (r < b) before += v;
            }
            l.tot[c] = total;
            l.pre[c] = before;
        }
    }
    lds_barrier();
    // (4) running sum down the waves: row r becomes "entries of the bin before wave r"
    for (int c = tid; c < W; c += blockDim.x) {
        int run = l.pre[c];
        for (int r = 0; r < wpb; ++r) {
            const int v = l.wh[r * W + c];
            l.wh[r * W + c] = run;
            run += v;
        }
        if (nchunks == 1) l.tot[c] = run;
    }
    lds_barrier();
    // (5) offset tables, per wave
    wave_offsets(a, l, lane);
    // (6) slots
    if (active) {
        for (int p0 = 0; p0 < a.passes; p0 += PU) {
            if (!one_group) load_group(a, wc, p0, lane, en);
            slots_group(a, en, p0, l.wh + w * W, l, lane);
        }
        // the walk has advanced the wave's prefixes past its own entries: they are now the
        // positions at which the next wave-chunk's entries start in the expert-sorted list
        if (a.run_start) {
            wave_lds_fence();
            int32_t* rs = a.run_start + (int64_t)(wc + 1) * a.E;
            const int32_t* h = l.wh + w * W;
            for (int e = lane; e < a.E; e += kWave) rs[e] = l.opre[e] + h[e];
        }
    }
    // (7) one wave publishes the per-expert / per-rank arrays and the totals; it does so
    //     after its own slot walk so that the walk of the chunk is not held up
    if (b == 0 && w == 0) wave_write_tables(a, l, lane);
}

// ---- inputs of at most 1024 entries: one workgroup, one entry per thread, bitmaps ----
//
// Every bin keeps one bit per entry (a 64-bit word per wavefront).  An entry sets its bit;
// its slot is the number of set bits below its own position in the bitmap of its bin --
// a handful of independent LDS reads and popcounts instead of a histogram, a scan across
// waves and a ballot walk.  Bits are set with atomic ORs, whose result does not depend on
// their order.
constexpr int kBitmapWords = 16;   // words per bitmap: one per wavefront of a 1024-thread workgroup
constexpr int kBitmapStride = 17;  // row stride in words: odd, so that the rows start in different LDS banks

size_t bitmap_lds_bytes(const LayoutArgs& a) {
    return 8 * (size_t)(a.E + a.R) * kBitmapStride + sizeof(int32_t) * (2 * (size_t)a.W + 2 * (a.E + 1) + (a.R + 1));
}

// Set bits of a bitmap row below position (w, lane): all 16 words are read at once.
__device__ __forceinline__ int bits_below(const uint64_t* row, int w, uint64_t below_in_word) {
    uint64_t v[kBitmapWords];
#pragma unroll
    for (int j = 0; j < kBitmapWords; ++j) v[j] = row[j];
    int n = 0;
#pragma unroll
    for (int j = 0; j < kBitmapWords; ++j) {
        const uint64_t m = j < w ? ~0ull : (j == w ? below_in_word : 0ull);
        n += __popcll(v[j] & m);
    }
    return n;
}

__global__ __launch_bounds__(1024) void layout_bitmap_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int nbins = a.E + a.R;  // expert bitmaps, then destination-rank bitmaps
    uint64_t* bm = (uint64_t*)lds;
    Lds l;
    l.wh = nullptr;
    l.tot = lds + 2 * nbins * kBitmapStride;
    l.pre = l.tot + a.W;
    l.eoff = l.pre + a.W;
    l.opre = l.eoff + a.E + 1;
    l.roff = l.opre + a.E + 1;
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    int raw[PU];
    issue_group(a, w, 0, lane, raw);  // one pass: the entry of this thread
    for (int j = tid; j < nbins * kBitmapStride; j += blockDim.x) bm[j] = 0ull;
    for (int j = tid; j < a.W; j += blockDim.x) l.tot[j] = 0;
    lds_barrier();
    Entry en[PU];
    classify_group(a, w, 0, lane, raw, en);
    const Entry& x = en[0];
    const uint64_t bit = 1ull << lane;
    if (x.ok) atomicOr((unsigned long long*)&bm[x.e * kBitmapStride + w], (unsigned long long)bit);
    if (x.lead) atomicOr((unsigned long long*)&bm[(a.E + x.d) * kBitmapStride + w], (unsigned long long)bit);
    const uint64_t bmask = __ballot(x.masked), binv = __ballot(x.invalid);
    if (lane == 0) {
        if (bmask) atomicAdd(&l.tot[a.E], __popcll(bmask));
        if (binv) atomicAdd(&l.tot[a.E + 1], __popcll(binv));
    }
    lds_barrier();
    for (int c = tid; c < nbins; c += blockDim.x)  // totals per bin
        l.tot[c < a.E ? c : c + 2] = bits_below(bm + c * kBitmapStride, kBitmapWords, 0ull);
    const int slot = x.ok ? bits_below(bm + x.e * kBitmapStride, w, bit - 1) : -1;
    const int rslot = x.lead ? bits_below(bm + (a.E + x.d) * kBitmapStride, w, bit - 1) : -1;
    lds_barrier();
    wave_offsets(a, l, lane);
    emit_entry(a, x, slot, rslot, l);
    if (w == 0) wave_write_tables(a, l, lane);
}

constexpr size_t kLdsLimit = 64 * 1024;

}  // namespace

// Wave-chunk plan for n entries.  Up to kLayoutOneBlockEntries: one workgroup of 16
// waves, 64*passes entries each (one launch).  Beyond: at least two passes per wave so
// that there are fewer, fuller chunks, and at most kMaxWaveChunks wave-chunks.
void plan_layout(int n, int* passes, int* nwc) {
    int p;
    if (n <= kLayoutOneBlockEntries) {
        p = (n + kWave * kLayoutWavesPerBlock - 1) / (kWave * kLayoutWavesPerBlock);
    } else {
        p = (n + kWave * kMaxWaveChunks - 1) / (kWave * kMaxWaveChunks);
        if (p < 2) p = 2;
    }
    if (p < 1) p = 1;
    *passes = p;
    *nwc = (n + kWave * p - 1) / (kWave * p);
}

static bool use_bitmap(const LayoutArgs& a) {
    return a.passes == 1 && a.nwc >= 1 && a.nwc <= kLayoutWavesPerBlock && bitmap_lds_bytes(a) <= kLdsLimit;
}

bool layout_writes_runs(const LayoutArgs& a) { return a.run_start != nullptr && !use_bitmap(a); }

// The read-ahead rides on the slot kernel of inputs that are laid out by several workgroups.
bool layout_prefetches(const LayoutArgs& a) {
    return a.warm_x != nullptr && a.warm_rows > 0 && a.n >= kRunOrderMinEntries && !use_bitmap(a) &&
           a.nwc > kLayoutWavesPerBlock;
}

constexpr int kWarmBlocks = 2048;  // extra workgroups of the slot kernel that read tokens

hipError_t launch_layout(const LayoutArgs& a_in, hipStream_t s) {
    LayoutArgs a = a_in;
    a.nchunks = 1;
    if (use_bitmap(a)) {
        hipLaunchKernelGGL(layout_bitmap_kernel, dim3(1), dim3(a.nwc * kWave), bitmap_lds_bytes(a), s, a);
        return hipGetLastError();
    }
    // One workgroup of up to 16 waves when the plan has at most 16 wave-chunks and its
    // LDS tables fit; otherwise chunks of at most 8 waves so that the walk is spread
    // over many compute units while one thread per bin can add up the chunk histograms.
    int wpb;
    if (a.nwc <= kLayoutWavesPerBlock && lds_bytes(a, kLayoutWavesPerBlock) <= kLdsLimit) {
        wpb = kLayoutWavesPerBlock;
    } else {
        wpb = kLayoutWavesPerChunk;
        while (wpb > 1 && lds_bytes(a, wpb) > kLdsLimit) wpb >>= 1;
        if (lds_bytes(a, wpb) > kLdsLimit) return hipErrorInvalidValue;
    }
    int nblk = (a.nwc + wpb - 1) / wpb;
    if (nblk < 1) nblk = 1;
    if (nblk > kMaxWaveChunks) return hipErrorInvalidValue;
    const dim3 grid(nblk), block(wpb * kWave);
    const size_t lds = lds_bytes(a, wpb);
    a.nchunks = nblk;
    const bool pf = layout_prefetches(a);
    if (nblk > 1) hipLaunchKernelGGL(layout_count_kernel, grid, block, lds_bytes(a, 1), s, a);
    if (nblk == 1) hipLaunchKernelGGL((layout_slot_kernel<1024, 1>), grid, block, lds, s, a);
    else hipLaunchKernelGGL((layout_slot_kernel<512, 32>), dim3(nblk + (pf ? kWarmBlocks : 0)), block, lds, s, a);
    return hipGetLastError();
}

}  // namespace ep
