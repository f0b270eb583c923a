// Routing layout kernels: per-expert / per-destination-rank counts, prefix
// offsets and the stable slot map (Sec. IV-A index algebra; Sec. IV-C "Token
// Count"; the slot rule of Sec. IV-B made deterministic).
//
// The slot of entry i = t*K + k is the number of entries j < i naming the same
// expert: a stable counting sort.  No atomic decides an order anywhere (atomics
// only add counts or set bits), so the output is a pure function of the input.
//
// The flattened entry list is cut into chunks, one per workgroup of up
// to 16 wavefronts, and every chunk into wave-chunks of 64*passes consecutive entries,
// one per wavefront.  ONE launch (Sec. IV-C "Token Count": the count runs next to the
// send, not as a phase of its own):
//   histogram   every wave histograms its wave-chunk -- bins: E experts, masked,
//               invalid, R destination ranks -- with LDS integer atomics;
//   publish     one thread per bin sums the wave histograms of the chunk and stores
//               the sum, tagged with the number of this launch, to global memory;
//   in-chunk    meanwhile every wave ranks its entries inside the chunk: prefix of the
//   ranks       bin over the earlier waves + number of lower lanes holding the same
//               key, found with one ballot per key bit;
//   look across one thread per bin reads that bin's sums of ALL chunks (it waits, a
//               bounded number of polls, until each carries this launch's tag): entries
//               in earlier chunks (the prefix) and in all chunks (the totals, hence
//               the expert offsets).  Only sums of counts cross between workgroups,
//               so the result does not depend on which chunk is published first;
//   scan        one exclusive scan of the totals over all bins by the whole workgroup;
//   emit        slot = prefix of earlier chunks + in-chunk rank, the destination row
//               and the expert-sorted entry list.
// The chunks wait for each other, so all of them must be resident at the same time:
// there are at most 256 of them (32 with the usual bin counts), no more than the part
// has compute units, they are the lowest workgroup ids of the launch, and every
// wait gives up after a fixed number of polls (status bit, never a hang).
// The work is latency bound (a chain of dependent LDS and global round trips per
// wave), so every phase issues all of its global loads before it waits for any of
// them and the workgroup barriers order LDS traffic only.
#include "ep_internal.h"
#include "ep_fp8.h"

#include <algorithm>

namespace ep {
namespace {

constexpr int PU = 2;  // passes whose loads are issued together and whose entries stay in registers

// Workgroup barrier that orders LDS traffic only: the LDS operations of this wave have
// completed when it arrives (s_waitcnt lgkmcnt(0)), and the compiler moves no memory access
// across it, but global loads and stores issued before it stay in flight (a
// __syncthreads(), or a workgroup-scope fence, would wait for them: a round trip to
// memory at every barrier of a latency-bound kernel).  Global memory written by one wave
// is never read by another wave of the workgroup in these kernels.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Data-parallel-primitive controls of the cross-lane moves below (CDNA ISA, DPP_CTRL).
constexpr int kDppRowShr = 0x110;      // + n: lane i reads lane i-n of its row of 16
constexpr int kDppWaveShr1 = 0x138;    // lane i reads lane i-1 of the wavefront
constexpr int kDppRowBcast15 = 0x142;  // lane 15 of each row to every lane of the next row
constexpr int kDppRowBcast31 = 0x143;  // lane 31 to every lane of rows 2 and 3

// The value of the lane below; lane 0 gets `fill`.
__device__ __forceinline__ int lane_below(int v, int fill) {
    return __builtin_amdgcn_update_dpp(fill, v, kDppWaveShr1, 0xf, 0xf, false);
}

// Inclusive prefix sum over the 64 lanes: within rows of 16 by shifted adds, then the
// row sums are carried into the rows above.  A lane whose source lies outside its row
// (or whose row is masked out) adds 0.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 1, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 2, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 4, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowShr + 8, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowBcast15, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowBcast31, 0xc, 0xf, false);
    return v;
}

__device__ __forceinline__ int wave_sum(int v) {
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ int wave_max(int v) {
    for (int off = kWave / 2; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, kWave));
    return v;
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

// LDS carve-up shared by the kernels.  wh .. flag are contiguous (zeroed in one sweep).
struct Lds {
    int32_t *wh;      // [nw+1][W] per-wave histograms, later "entries of the bin in the earlier waves of the
                      //     chunk"; row nw stands in for the rows a smaller workgroup does not have, so that
                      //     sweeps over kLayoutWavesPerBlock rows need no branch: it reads as 0 and is never used
    int32_t *tot;     // [W] totals over the whole input
    int32_t *S;       // [W] exclusive scan of tot over all bins.  S[e], e <= E, is the first position of expert
                      //     e in the expert-sorted list (S[E] = routed entries), and its first row in the
                      //     concatenated layout unless the caller gave the first rows; the rank bins are the
                      //     last R bins: for compact staging windows rank_offset[d] = S[E+2+d] - S[E+2]
    int32_t *before;  // [W] entries of each bin in earlier chunks
    int32_t *wsum;    // [kLayoutWavesPerBlock] per-wave sums of the scan (0 for waves the workgroup does not have)
    int32_t *flag;    // [1] set when a thread of the workgroup gave up waiting for another chunk
};

__device__ __forceinline__ Lds carve_lds(int32_t* base, const LayoutArgs& a, int nw) {
    Lds l;
    l.wh = base;
    l.tot = l.wh + (nw + 1) * a.W;
    l.S = l.tot + a.W;
    l.before = l.S + a.W;
    l.wsum = l.before + a.W;
    l.flag = l.wsum + kLayoutWavesPerBlock;
    return l;
}

constexpr int lds_ints(int W, int nw) { return (nw + 1) * W + 3 * W + kLayoutWavesPerBlock + 1; }

size_t lds_bytes(const LayoutArgs& a, int nw) { return sizeof(int32_t) * (size_t)lds_ints(a.W, nw); }

// Marks the entries that are the first of their token to name their destination
// rank.  The entries of a token sit in consecutive lanes, so lane l compares its
// rank with the ranks held by lanes l-1 .. l-k (one shift of the wave per step); only
// when a token began before lane 0 are its earlier entries read from memory.
// Must be called by all 64 lanes.
__device__ __forceinline__ void mark_leaders(const LayoutArgs& a, Entry& en, int lane) {
    const int dkey = en.ok ? en.d : -1;
    bool lead = en.ok;
    int prev = dkey;
    for (int j = 1; j < a.K; ++j) {
        prev = lane_below(prev, -2);  // the key of lane l-j; -2 (no key) below lane 0
        if (j <= en.k && prev == dkey) lead = false;
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

// First row of expert e in the receiver's tensor.
__device__ __forceinline__ int first_row(const LayoutArgs& a, const Lds& l, int e) {
    if (a.padded) return e * a.C;
    return a.expert_base ? a.expert_base[e] : l.S[e];
}

// First staging slot of destination rank d (d == R: one past the last).
__device__ __forceinline__ int first_slot(const LayoutArgs& a, const Lds& l, int d) {
    if (a.padded) return d * a.C_rank;
    const int end = d < a.R ? l.S[a.E + 2 + d] : l.S[a.W - 1] + l.tot[a.W - 1];
    return end - l.S[a.E + 2];
}

// Writes what the layout records for one entry, given its rank inside the chunk among the
// entries of its expert and (for a leader) among the tokens of its destination rank; the
// entries of earlier chunks (l.before) turn the ranks into slots.
__device__ __forceinline__ void emit_entry(const LayoutArgs& a, const Entry& x, int slot, int rslot, const Lds& l) {
    int row = -1, rrow = -1;
    if (x.ok) {
        slot += l.before[x.e];
        if (a.padded) row = slot < a.C ? x.e * a.C + slot : -1;
        else row = first_row(a, l, x.e) + slot;
        if (a.sorted_token) {
            const int pos = l.S[x.e] + slot;
            a.sorted_token[pos] = x.t;
            a.sorted_k[pos] = x.k;
            a.sorted_row[pos] = row;
        }
    }
    if (x.lead) rrow = first_slot(a, l, x.d) + l.before[a.E + 2 + x.d] + rslot;
    if (x.i >= 0) {
        if (a.slot) a.slot[x.i] = slot;
        a.dst_row[x.i] = row;
        if (a.rank_row) a.rank_row[x.i] = rrow;
        if (a.entry_rank) a.entry_rank[x.i] = x.ok ? x.d : -1;
    }
}

// Where an entry stands among the entries of its wave that hold the same key, for the expert
// key and (for a leader) the destination-rank key: entries below it and entries in all.
struct InWave {
    int below, all;      // among the lanes naming the same expert
    int below_r, all_r;  // among the leader lanes naming the same destination rank
};

// The in-wave standing of a loaded group: ballots only, no memory.  Must be called by all
// 64 lanes.
__device__ __forceinline__ void rank_group(const LayoutArgs& a, const Entry (&en)[PU], int p0, int lane, InWave (&iw)[PU]) {
    const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < PU; ++j) {
        iw[j] = InWave{0, 0, 0, 0};
        if (p0 + j >= a.passes) continue;  // wave-uniform
        const uint64_t peers = match_key(en[j].e, en[j].ok, a.bits_e);
        const uint64_t peers_r = match_key(en[j].d, en[j].lead, a.bits_r);
        iw[j] = InWave{(int)__popcll(peers & lt), (int)__popcll(peers), (int)__popcll(peers_r & lt), (int)__popcll(peers_r)};
    }
}

// Ranks of a loaded group inside its chunk: h holds, per bin, the number of entries of that
// bin in the earlier waves of the chunk and in the earlier groups of this wave; it is
// advanced as the group is walked.  LDS accesses of one wavefront are performed in program
// order, and the wave barriers keep the compiler from moving them across each other.
// Must be called by all 64 lanes.
__device__ __forceinline__ void place_group(const LayoutArgs& a, const Entry (&en)[PU], const InWave (&iw)[PU], int p0,
                                            int32_t* h, int (&slot)[PU], int (&rslot)[PU]) {
#pragma unroll
    for (int j = 0; j < PU; ++j) {
        slot[j] = -1;
        rslot[j] = -1;
        if (p0 + j >= a.passes) continue;  // wave-uniform
        const Entry& x = en[j];
        if (x.ok) slot[j] = h[x.e] + iw[j].below;
        if (x.lead) rslot[j] = h[a.E + 2 + x.d] + iw[j].below_r;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        if (x.ok && iw[j].below == 0) h[x.e] += iw[j].all;
        if (x.lead && iw[j].below_r == 0) h[a.E + 2 + x.d] += iw[j].all_r;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
    }
}

__device__ __forceinline__ void emit_group(const LayoutArgs& a, const Entry (&en)[PU], int p0, const int (&slot)[PU],
                                           const int (&rslot)[PU], const Lds& l) {
#pragma unroll
    for (int j = 0; j < PU; ++j)
        if (p0 + j < a.passes) emit_entry(a, en[j], slot[j], rslot[j], l);  // wave-uniform condition
}

// Exclusive scan of the totals tot[0..W) over all bins into S, by the whole workgroup
// (thread = bin; with more bins than threads, in rounds).  Starts with a barrier (tot and
// whatever else was written to LDS before become visible) and ends with one (S is final).
// Must be called by every thread of the workgroup.
__device__ void block_scan_totals(const LayoutArgs& a, const Lds& l, int tid, int lane, int w, int nw) {
    int carry = 0;
    lds_barrier();
    for (int c0 = 0; c0 < a.W; c0 += blockDim.x) {
        const int c = c0 + tid;
        const int v = c < a.W ? l.tot[c] : 0;
        const int inc = wave_inclusive_scan(v);
        if (lane == kWave - 1) l.wsum[w] = inc;
        lds_barrier();
        int below = 0, all = 0;
#pragma unroll
        for (int r = 0; r < kLayoutWavesPerBlock; ++r) {  // waves the workgroup does not have left 0
            const int s = l.wsum[r];
            below += r < w ? s : 0;
            all += s;
        }
        if (c < a.W) l.S[c] = carry + below + inc - v;
        carry += all;
        lds_barrier();
    }
}

// The per-expert / per-rank arrays and the totals block (all but the status word) in
// global memory, from tot and S in LDS.  By every thread of one workgroup.  Returns one past
// the highest destination row (in wave 0; other waves get 0).
__device__ int write_tables(const LayoutArgs& a, const Lds& l, int tid, int lane, int w) {
    const int32_t* tot = l.tot;
    const int32_t* S = l.S;
    const int E = a.E, R = a.R;
    for (int e = tid; e < E; e += blockDim.x) {
        const int v = tot[e];
        a.expert_count[e] = v;
        a.expert_kept[e] = a.padded ? min(v, a.C) : v;
        if (a.recv_count) a.recv_count[e] = a.padded ? min(v, a.C) : v;
        a.expert_offset[e] = first_row(a, l, e);
        a.own_prefix[e] = S[e];
        if (a.run_start) a.run_start[e] = S[e];  // row 0: nothing precedes the first wave-chunk
    }
    if (a.rank_pair_count) {
        for (int d = tid; d <= R; d += blockDim.x) {
            if (d < R) {
                a.rank_pair_count[d] = S[(d + 1) * a.L] - S[d * a.L];
                a.rank_token_count[d] = tot[E + 2 + d];
            }
            a.rank_offset[d] = first_slot(a, l, d);
        }
    }
    if (w != 0) return 0;
    // wave 0: the sums over all experts
    int kept = 0, dropped = 0, rend = 0;
    for (int e = lane; e < E; e += kWave) {
        const int v = tot[e];
        const int k = a.padded ? min(v, a.C) : v;
        kept += k;
        dropped += v - k;
        if (!a.padded && a.expert_base && v > 0) rend = max(rend, a.expert_base[e] + v);
    }
    kept = wave_sum(kept);
    dropped = wave_sum(dropped);
    rend = wave_max(rend);
    const int total_e = S[E];
    const int rows_end = a.padded ? E * a.C : (a.expert_base ? rend : total_e);
    if (lane == 0) {
        a.expert_offset[E] = rows_end;
        a.own_prefix[E] = total_e;
        a.totals[TOT_KEPT] = kept;
        a.totals[TOT_DROPPED] = dropped;
        a.totals[TOT_MASKED] = tot[E];
        a.totals[TOT_INVALID] = tot[E + 1];
        a.totals[TOT_SORTED] = total_e;
        a.totals[TOT_MSGS] = S[a.W - 1] + tot[a.W - 1] - S[E + 2];  // the rank bins are the last R bins
        a.totals[TOT_ROWS_END] = rows_end;
        if (a.drop_hint) *a.drop_hint = (int64_t)kept | ((int64_t)dropped << 32);
    }
    return rows_end;
}

// The status word of the totals block.  One wavefront; must be called by all 64 lanes.
__device__ void write_status(const LayoutArgs& a, const Lds& l, int lane, int extra_status) {
    int dropped = 0;
    if (a.padded)
        for (int e = lane; e < a.E; e += kWave) dropped |= l.tot[e] > a.C ? 1 : 0;
    const bool any_dropped = __ballot(dropped != 0) != 0;
    if (lane == 0)
        a.totals[TOT_STATUS] = (l.tot[a.E + 1] ? STATUS_INVALID_IDS : 0) | (any_dropped ? STATUS_CAPACITY_DROP : 0) |
                               extra_status;
}

// Extra workgroups of the layout kernel (blockIdx >= nchunks): read the token rows the
// caller announced, with ordinary cached loads, while the layout workgroups -- a few dozen
// on a part with 256 compute units -- do their latency-bound work.  wb of nwb.  Rows
// [0, warm_rows), 16 bytes per load, four loads of a thread in flight.
constexpr int kWarmUnroll = 4;
__device__ void warm_tokens(const LayoutArgs& a, int wb, int nwb) {
    const uint32_t units = (uint32_t)a.warm_units;
    const uint32_t total = (uint32_t)a.warm_rows * units;  // at most 64 MiB / 16
    const uint32_t stride = (uint32_t)nwb * blockDim.x;
    const bool dense = a.warm_stride == (int64_t)units * 8;  // rows back to back: no division
    uint32_t acc = 0;
    for (uint32_t i0 = (uint32_t)wb * blockDim.x + threadIdx.x; i0 < total; i0 += kWarmUnroll * stride) {
        u32x4 v[kWarmUnroll];
#pragma unroll
        for (int q = 0; q < kWarmUnroll; ++q) {
            const uint32_t i = min(i0 + q * stride, total - 1);  // the tail repeats the last unit
            if (dense) {
                v[q] = *((const u32x4*)a.warm_x + i);
            } else {
                const uint32_t t = i / units;
                v[q] = *((const u32x4*)(a.warm_x + (int64_t)t * a.warm_stride) + (i - t * units));
            }
        }
#pragma unroll
        for (int q = 0; q < kWarmUnroll; ++q) acc ^= v[q][0] ^ v[q][1] ^ v[q][2] ^ v[q][3];
    }
    asm volatile("" ::"v"(acc));  // the loads are the point: keep them
}

constexpr int kLookLimit = 1 << 19;  // rounds of polling after which a thread stops waiting (about a second)
constexpr int HB = 32;               // chunks whose published words a thread loads in one batch (at most 32: bit masks)
constexpr int kTagShift = 24;        // a published word is (tag << 24) | count: a chunk holds fewer than 2^24 entries
constexpr uint32_t kCountMask = (1u << kTagShift) - 1u;
constexpr uint32_t kTags = 255;      // tags 1 .. 255; 0 is what a cleared word holds

// Loads the words chunks r0 .. r0+HB-1 have published for bin c.  Every lane loads from a
// valid address (rows beyond the last chunk repeat it, their words are ignored later):
// no branch, so all HB loads are in flight together.
__device__ __forceinline__ void look_across(const LayoutArgs& a, int c, int r0, uint32_t (&v)[HB]) {
    const int last = a.nchunks - 1;
    const uint32_t* row = a.pub + (int64_t)min(r0, last) * a.W;  // wave-uniform: the row pointer steps in scalar registers
#pragma unroll
    for (int j = 0; j < HB; ++j) {
        v[j] = __hip_atomic_load(row + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        row += r0 + j < last ? a.W : 0;
    }
}

// Chunk b = wave-chunks [b*wpb, (b+1)*wpb); with several chunks workgroup nchunks writes the
// tables; the workgroups after those read tokens ahead.
// With one chunk nothing is published or awaited.
//
// Cross-workgroup state (only with more than one chunk), all in a.pub / a.ctl:
//   pub[r][c]  one word: (tag << 24) | entries of bin c in chunk r, tag = ctl[0] + 1 of the
//              launch that wrote it; written once per launch with one atomic store, so a
//              reader that sees the tag of its own launch also sees the count;
//   ctl[0]     launches completed on this scratch since pub was last cleared (the
//              generation, 0 .. 254); read at the start, advanced by the workgroup that is
//              last to finish looking across, which clears pub when the tags run out;
//   ctl[1]     workgroups of this launch that have finished looking across, in the low 16
//              bits; a workgroup that gave up waiting also adds 1 << 16.  Back to 0 at the end.
// Tags never repeat between two clearings of pub, and the scratch starts out all zero,
// which no launch uses as a tag.
//
// MULTI: more than one chunk.  ONE_GROUP: a wave's entries fit one load group (at most PU
// passes) and stay in registers from the histogram to the emit.
// The same workgroups, for a group that quantises ahead: instead of only reading the token
// rows they quantise them (the FP8 dispatch's format, see ep_fp8.h) into a staging copy, row t
// at quant_out + t * quant_pitch: H bytes of codes, then H/128 float scales.  The quantising
// dispatch that follows copies staged rows in destination order and finds them, like the
// tokens, in the caches.  A lane owns 16 consecutive channels, 8 neighbouring lanes one
// 128-channel group; H is a multiple of 128, so a group never straddles rows and the 8 lanes
// of a group are in or out of range together.  Ordinary cached loads and stores: both the
// tokens and the staged rows are wanted in the cache afterwards.
__device__ void quantize_tokens(const LayoutArgs& a, int wb, int nwb) {
    const uint32_t per_row = (uint32_t)a.warm_units >> 1;   // 32-byte lane items per row (H / 16)
    const uint32_t total = (uint32_t)a.warm_rows * per_row;
    const uint32_t stride = (uint32_t)nwb * blockDim.x;
    const uint32_t H = (uint32_t)a.warm_units * 8;
    for (uint32_t i = (uint32_t)wb * blockDim.x + threadIdx.x; i < total; i += stride) {
        const uint32_t t = i / per_row, u = i - t * per_row;
        const u32x4* src = (const u32x4*)(a.warm_x + (int64_t)t * a.warm_stride) + 2 * u;
        const u32x4 in0 = src[0], in1 = src[1];
        float scale;
        const u32x4 q = quantize16(in0, in1, &scale);
        uint8_t* row = a.quant_out + (int64_t)t * a.quant_pitch;
        *((u32x4*)row + u) = q;
        if ((u & 7u) == 0) *(float*)(row + H + 4 * (u >> 3)) = scale;
    }
}

template <bool MULTI, bool ONE_GROUP>
__device__ __forceinline__ void layout_chunk(const LayoutArgs& a, int32_t* lds, const int b) {
    const int wpb = blockDim.x >> 6;
    const Lds l = carve_lds(lds, a, wpb);
    const int W = a.W;
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wc = b * wpb + w;
    const int nchunks = a.nchunks;
    const bool active = wc < a.nwc;
    constexpr bool one_group = ONE_GROUP, multi = MULTI;

    // (1) the global loads this workgroup can issue at once: its own ids and the generation
    //     (first needed in (3): nothing here waits for it)
    int raw[PU];
    if (active) issue_group(a, wc, 0, lane, raw);
    uint32_t gen = __hip_atomic_load(&a.ctl[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int j = tid; j < lds_ints(W, wpb); j += blockDim.x) l.wh[j] = 0;
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
    lds_barrier();

    // (3) per bin (thread = column): the sum of the chunk, which is published at once, and
    //     the running sum down the waves -- row r becomes "entries of the bin in the waves
    //     before r"
    asm volatile("" : "+v"(gen));  // the generation is first looked at here
    const uint32_t tag = gen + 1u;
    for (int c = tid; c < W; c += blockDim.x) {
        int v[kLayoutWavesPerBlock];
#pragma unroll
        for (int r = 0; r < kLayoutWavesPerBlock; ++r) v[r] = l.wh[min(r, wpb) * W + c];  // rows beyond the last: 0
        int run = 0;
#pragma unroll
        for (int r = 0; r < kLayoutWavesPerBlock; ++r) {
            const int x = v[r];
            v[r] = run;
            run += x;
        }
        if (multi && b < nchunks)  // the workgroup after the last chunk has no entries: it only writes the tables
            __hip_atomic_store(&a.pub[(int64_t)b * W + c], (tag << kTagShift) | (uint32_t)run, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        l.tot[c] = run;
#pragma unroll
        for (int r = 0; r < kLayoutWavesPerBlock; ++r) l.wh[min(r, wpb) * W + c] = v[r];
    }
    // (4) ranks inside the chunk; with one load group they are computed here, while the
    //     other chunks publish, and only then comes the first look across: issued earlier it
    //     finds some of the other chunks' sums not yet there and has to be repeated, a second
    //     round trip (measured: 0.6 us per step later, 1.2 us of the kernel in all)
    InWave iw[PU];
    if (active && one_group) rank_group(a, en, 0, lane, iw);
    lds_barrier();
    int sl[PU], rsl[PU];
    if (active && one_group) place_group(a, en, iw, 0, l.wh + w * W, sl, rsl);
    uint32_t hv[HB];
    if (multi) look_across(a, min(tid, W - 1), 0, hv);

    // (5) per bin: entries in earlier chunks and in all chunks.  A batch of words is polled
    //     as a whole until every word of it carries this launch's tag (rows beyond the last
    //     chunk repeat its words, and the chunk's own word is among them: no exceptions to
    //     test for).  Which words of a batch count, and which belong to earlier chunks, are
    //     wave-uniform bit masks.
    if (multi) {
        int rounds = 0;  // of this thread, over all its batches
        bool gave_up = false;
        bool have = true;  // hv holds the batch (tid, 0)
        for (int c = tid; c < W; c += blockDim.x) {
            int before = 0, total = 0;
            for (int r0 = 0; r0 < nchunks; r0 += HB) {
                for (;;) {
                    if (!have) look_across(a, c, r0, hv);
                    have = false;
                    bool all = true;
#pragma unroll
                    for (int j = 0; j < HB; ++j) all = all && (hv[j] >> kTagShift) == tag;
                    if (all) break;
                    if (++rounds >= kLookLimit) {  // a chunk never published: flag it (the counts are then undefined)
                        gave_up = true;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
                const int nvalid = min(nchunks - r0, HB), nbefore = min(max(b - r0, 0), HB);
                const uint32_t valid = nvalid >= 32 ? ~0u : (1u << nvalid) - 1u;
                const uint32_t earlier = nbefore >= 32 ? ~0u : (1u << nbefore) - 1u;
#pragma unroll
                for (int j = 0; j < HB; ++j) {
                    const uint32_t cnt = hv[j] & kCountMask & (0u - ((valid >> j) & 1u));
                    total += (int)cnt;
                    before += (int)(cnt & (0u - ((earlier >> j) & 1u)));
                }
            }
            l.tot[c] = total;  // the chunk's own sum is one of the words
            l.before[c] = before;
        }
        if (gave_up) atomicOr(l.flag, 1);
    }
    // (6) the scan over the bins (its first barrier also makes tot, before and flag final)
    block_scan_totals(a, l, tid, lane, w, wpb);
    // thread 0 reports for the workgroup: the value it gets back tells wave 0 whether this
    // workgroup is the last to have looked across (then every chunk is done with pub and ctl,
    // and it may advance the generation) and whether any workgroup gave up waiting
    const int any_gave_up = *l.flag;
    uint32_t ticket = 0;
    constexpr uint32_t kGaveUp = 1u << 16;  // low 16 bits count workgroups, the rest flags a time-out
    const uint32_t mine = 1u + (any_gave_up ? kGaveUp : 0u);
    if (multi && tid == 0) ticket = __hip_atomic_fetch_add(&a.ctl[1], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // (7) slots
    if (active) {
        for (int p0 = 0; p0 < a.passes; p0 += PU) {
            if (!one_group) {
                load_group(a, wc, p0, lane, en);
                rank_group(a, en, p0, lane, iw);
                place_group(a, en, iw, p0, l.wh + w * W, sl, rsl);
            }
            emit_group(a, en, p0, sl, rsl, l);
        }
        // the walk has advanced the wave's prefixes past its own entries: they are now the
        // positions at which the next wave-chunk's entries start in the expert-sorted list
        if (a.run_start) {
            wave_lds_fence();
            int32_t* rs = a.run_start + (int64_t)(wc + 1) * a.E;
            const int32_t* h = l.wh + w * W;
            for (int e = lane; e < a.E; e += kWave) rs[e] = l.S[e] + l.before[e] + h[e];
        }
    }
    // (8) the per-expert / per-rank arrays and the totals.  With several chunks they come from a
    //     workgroup of their own, number nchunks, which has no entries: it looks across, scans
    //     and writes the tables while the chunks are still walking theirs (written by a chunk
    //     after its walk they were the last thing the launch waited for).  The status word comes
    //     from one wavefront: with several chunks wave 0 of the workgroup that finished looking
    //     across last, which then also leaves the cross-workgroup words ready for the next launch
    int rows_end = 0;
    if (b == (multi ? nchunks : 0)) rows_end = write_tables(a, l, tid, lane, w);
    if (w != 0) return;
    if (!multi) {  // the caller of a fused launch says how many rows its output takes
        write_status(a, l, lane, (!a.padded && a.rows_cap >= 0 && rows_end > a.rows_cap) ? STATUS_OUTPUT_OVERFLOW : 0);
        return;
    }
    const uint32_t seen = __builtin_amdgcn_readfirstlane(ticket) + mine;  // lane 0 holds the ticket
    if ((int)(seen & (kGaveUp - 1u)) != nchunks + 1) return;  // the chunks and the workgroup of the tables
    write_status(a, l, lane, seen >= kGaveUp ? STATUS_TIMEOUT : 0);
    uint32_t next = gen + 1u;
    if (next >= kTags) {  // the tags have run out: clear every published word and start over
        for (int64_t j = lane; j < (int64_t)kMaxChunks * W; j += kWave) a.pub[j] = 0u;
        next = 0u;
    }
    if (lane == 0) {
        __hip_atomic_store(&a.ctl[1], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&a.ctl[0], next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <bool MULTI, bool ONE_GROUP>
__global__ __launch_bounds__(1024) void layout_kernel(LayoutArgs a) {
    extern __shared__ int32_t lds[];
    const int nlay = a.nchunks + (MULTI ? 1 : 0);  // workgroups that lay out: the chunks and, with several, the one of the tables
    if ((int)blockIdx.x >= nlay) {  // a whole workgroup: no barrier is reached by part of one
        // a short pause first (about 0.4 us): the chunks' loads of their ids then go ahead of the flood of
        // token reads instead of queueing behind it (1.2 us of the kernel at the prefill shape)
        __builtin_amdgcn_s_sleep(16);
        if (a.quant_out) quantize_tokens(a, blockIdx.x - nlay, gridDim.x - nlay);
        else warm_tokens(a, blockIdx.x - nlay, gridDim.x - nlay);
        return;
    }
    layout_chunk<MULTI, ONE_GROUP>(a, lds, blockIdx.x);
}

// ---- layout and direct dispatch of a small input in ONE launch (Sec. IV-C: in the
// low-latency kernels the count runs next to the send) ----
//
// For an input of at most 1024 entries (one per thread of a workgroup).  Workgroup 0 is the
// layout above, single chunk, and writes the handle's arrays, which combine and the queries
// read later.  Every other workgroup copies a share of one token row -- work unit = one
// wavefront x one 1 KiB segment, `spp` segments per workgroup, `parts` workgroups per token
// -- and needs only the destination rows of that token's K entries, which it counts out of
// the ids directly: row of entry (t, k) naming expert e = first row of e + number of entries
// before (t, k) that name e, the first row being the number of entries that name a lower
// expert (or e * C, or the caller's).  Counting = one ballot per wavefront and target over
// the ids its lanes hold, summed over the wavefronts through LDS.  Same ids, same
// arithmetic as the layout: the rows are those workgroup 0 records.  No workgroup waits
// for another.
__global__ __launch_bounds__(1024) void layout_dispatch_kernel(LayoutArgs a, DispatchArgs d, int nseg, int units, int parts,
                                                               int spp) {
    extern __shared__ int32_t lds[];
    if (blockIdx.x == 0) {
        layout_chunk<false, true>(a, lds, 0);
        return;
    }
    const int tid = threadIdx.x;
    const int lane = lane_id();
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = blockDim.x >> 6;
    const int wg = blockIdx.x - 1;
    const int t = wg / parts;
    const int seg = (wg - t * parts) * spp + w;
    const bool copies = w < spp && seg < nseg;
    const int unit = seg * kWave + lane;
    const bool active = copies && unit < units;
    // the loads this wave needs, all issued before any is waited for: its piece of the
    // token, the id of the entry this thread stands for, the token's K ids and gate weights
    u32x4 v = {0u, 0u, 0u, 0u};
    if (active) v = __builtin_nontemporal_load((const u32x4*)(d.x + (int64_t)t * d.x_stride) + unit);
    int id = -1;
    if (tid < a.n) {
        const int ti = token_of(a, tid);
        id = a.topk[(int64_t)ti * a.topk_stride + (tid - ti * a.K)];
    }
    const int my_e = lane < a.K ? a.topk[(int64_t)t * a.topk_stride + lane] : -1;
    float my_w = 1.0f;
    if (copies && seg == 0 && d.w && lane < a.K) my_w = d.w[(int64_t)t * d.w_stride + lane];
    int my_base = 0;
    if (!a.padded && a.expert_base && lane < a.K && (unsigned)my_e < (unsigned)a.E) my_base = a.expert_base[my_e];
    // per target k (lane k keeps its counts): entries of this wave that name the same expert
    // and come before (t, k), and entries of this wave that name a lower expert
    int same_before = 0, lower = 0;
    const int first = t * a.K;
    for (int k = 0; k < a.K; ++k) {
        const int e = __builtin_amdgcn_readlane(my_e, k);
        const uint64_t m_same = __ballot(id == e && tid < first + k);
        const uint64_t m_lower = __ballot((unsigned)id < (unsigned)e);  // ids that are not routed compare high
        if (lane == k) {
            same_before = __popcll(m_same);
            lower = __popcll(m_lower);
        }
    }
    int32_t* part_same = lds;                    // [nw][64]
    int32_t* part_lower = lds + nw * kWave;      // [nw][64]
    part_same[w * kWave + lane] = same_before;
    part_lower[w * kWave + lane] = lower;
    lds_barrier();
    if (!copies) return;
    int slot = 0, start = 0;
    for (int r = 0; r < nw; ++r) {
        slot += part_same[r * kWave + lane];
        start += part_lower[r * kWave + lane];
    }
    int my_row = -1;
    if (lane < a.K && (unsigned)my_e < (unsigned)a.E) {
        if (a.padded) my_row = slot < a.C ? my_e * a.C + slot : -1;
        else my_row = (a.expert_base ? my_base : start) + slot;
    }
    for (int k = 0; k < a.K; ++k) {
        const int row = __builtin_amdgcn_readlane(my_row, k);
        if (row < 0 || row >= d.win.rows_cap) continue;  // rows beyond the output are flagged by workgroup 0
        uint16_t* dst = d.win.base + window_offset(d.win, row);
        if (active) __builtin_nontemporal_store(v, (u32x4*)dst + unit);
        if (seg == 0 && lane == 0) {
            if (d.recv_w) d.recv_w[row] = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(my_w), k));
            if (d.recv_src) d.recv_src[row] = t;
        }
    }
}

constexpr size_t kLdsLimit = 64 * 1024;

}  // namespace

// Wave-chunk plan for n entries: 64*passes consecutive entries per wavefront.  Up to
// kLayoutOneBlockEntries: one workgroup of 16 waves (one launch, nothing crosses between
// workgroups).  Beyond: as many wave-chunks as there are passes of 64 entries, up to
// kMaxWaveChunks, so that every wave has as short a chain of dependent steps as possible.
void plan_layout(int n, int* passes, int* nwc) {
    int p;
    if (n <= kLayoutOneBlockEntries) p = (n + kWave * kLayoutWavesPerBlock - 1) / (kWave * kLayoutWavesPerBlock);
    else p = (n + kWave * kMaxWaveChunks - 1) / (kWave * kMaxWaveChunks);
    if (p < 1) p = 1;
    *passes = p;
    *nwc = (n + kWave * p - 1) / (kWave * p);
}

bool layout_writes_runs(const LayoutArgs& a) { return a.run_start != nullptr; }

// The read-ahead rides on the layout kernel of inputs that are laid out by several workgroups.
bool layout_prefetches(const LayoutArgs& a) {
    return a.warm_x != nullptr && a.warm_rows > 0 && a.n >= kRunOrderMinEntries && a.nwc > kLayoutWavesPerBlock;
}

constexpr int kFusedMaxEntries = kLayoutWavesPerBlock * kWave;  // one entry per thread of a workgroup

// The one-launch path takes inputs of at most 1024 entries, copied by the plain token-ordered
// walk (bf16 rows, the K entries of a token held by the lanes of one wave).
bool layout_dispatch_fusable(const LayoutArgs& a, const DispatchArgs& d) {
    return a.n >= 1 && a.n <= kFusedMaxEntries && a.passes == 1 && a.K <= kWave && d.H >= 8 &&
           lds_bytes(a, kLayoutWavesPerBlock) <= kLdsLimit;
}

hipError_t launch_layout_dispatch(const LayoutArgs& a_in, const DispatchArgs& d, hipStream_t s) {
    LayoutArgs a = a_in;
    a.nchunks = 1;
    if (!layout_dispatch_fusable(a, d)) return hipErrorInvalidValue;
    a.rows_cap = d.win.rows_cap;
    a.recv_count = d.recv_count;
    const int units = d.H / 8;
    const int nseg = (units + kWave - 1) / kWave;
    // workgroups per token: enough of them to put every compute unit to work, at most 16 segments each
    int parts = (nseg + kLayoutWavesPerBlock - 1) / kLayoutWavesPerBlock;
    while (parts < nseg && (int64_t)a.T * parts < 256) ++parts;
    const int spp = (nseg + parts - 1) / parts;
    parts = (nseg + spp - 1) / spp;
    const int64_t nblk = 1 + (int64_t)a.T * parts;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    // a thread per entry, a wave per segment, and the 16 waves the layout workgroup is laid out for
    const size_t lds = std::max(lds_bytes(a, kLayoutWavesPerBlock), sizeof(int32_t) * 2 * kLayoutWavesPerBlock * kWave);
    hipLaunchKernelGGL(layout_dispatch_kernel, dim3((unsigned)nblk), dim3(kLayoutWavesPerBlock * kWave), lds, s, a, d, nseg,
                       units, parts, spp);
    return hipGetLastError();
}

// Extra workgroups of the layout kernel that read tokens.  All of them should be running from the
// start: a compute unit of this part holds two workgroups of 1024 threads, the part has 256 units,
// and the layout workgroups take their places first; workgroups that find no place start when the
// others are done and then read their share alone, as a tail.
constexpr int kWarmBlocks = 448;
constexpr int kResidentBlocks = 2 * 256;

hipError_t launch_layout(const LayoutArgs& a_in, hipStream_t s) {
    LayoutArgs a = a_in;
    a.nchunks = 1;
    // Workgroups of 16 waves, fewer when the bin tables would not fit the LDS otherwise.
    int wpb = kLayoutWavesPerBlock;
    while (wpb > 1 && lds_bytes(a, wpb) > kLdsLimit) wpb >>= 1;
    if (lds_bytes(a, wpb) > kLdsLimit) return hipErrorInvalidValue;
    int nblk = (a.nwc + wpb - 1) / wpb;
    if (nblk < 1) nblk = 1;
    if (nblk > kMaxChunks) return hipErrorInvalidValue;
    if ((int64_t)wpb * kWave * a.passes > (int64_t)kCountMask) return hipErrorInvalidValue;  // a chunk's count must fit its word
    a.nchunks = nblk;
    const bool pf = layout_prefetches(a);
    const int nlay = nblk + (nblk > 1 ? 1 : 0);
    const int nwarm = pf ? std::max(64, std::min(kWarmBlocks, kResidentBlocks - nlay - 16)) : 0;
    const dim3 grid(nlay + nwarm), block(wpb * kWave);
    const size_t lds = lds_bytes(a, wpb);
    const bool one_group = a.passes <= PU;
    if (nblk > 1 && one_group) hipLaunchKernelGGL((layout_kernel<true, true>), grid, block, lds, s, a);
    else if (nblk > 1) hipLaunchKernelGGL((layout_kernel<true, false>), grid, block, lds, s, a);
    else if (one_group) hipLaunchKernelGGL((layout_kernel<false, true>), grid, block, lds, s, a);
    else hipLaunchKernelGGL((layout_kernel<false, false>), grid, block, lds, s, a);
    return hipGetLastError();
}

}  // namespace ep
