// Footprint-optimised dispatch (Sec. IV-D): a token is sent ONCE per destination
// rank into that rank's staging window, with the source token index, the routing
// vector and the gate weights in the message header; the receiving side expands
// each message to the local experts its header names (Sec. IV-C "Dispatch/recv").
//
// Message = { int32 src_token; int32 route[K]; float w[K]; zero padding to a
// multiple of 16 bytes; 2H bytes of token data }.  Slots are msg_stride bytes apart
// (a multiple of 256) and a message starts msg_lead bytes into its slot, so that its
// token data starts on a 256-byte boundary: every 1 KiB wave access to the data covers
// whole memory lines, and the short header sits in the line before.
//
//   send kernel    work unit = one wavefront x one 1 KiB segment of one token's data,
//                  loaded once and stored to every destination rank's slot; the wave
//                  of segment 0 also builds and stores the header.
//   rank kernel    the receiving side: one workgroup per staging window ranks the
//                  header entries that name one of the window's local experts among
//                  the entries of the same expert, in slot order (a stable counting
//                  sort over L bins), which gives every entry its expert row.
//   fan-out kernel work unit = one wavefront x one 1 KiB payload segment of one
//                  staged message: loaded once, stored to each local expert row.
// Pure data movement: HBM bound.  On one GPU this path moves about 2.6x the bytes
// of the direct path; what it saves is staging footprint, O(R*B*P) instead of
// O(E*B*P).
#include "ep_internal.h"

namespace ep {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void dedup_send_kernel(DedupSendArgs a, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (u >= (int64_t)a.T * nseg) return;
    const int t = (int)(u / nseg);
    const int seg = (int)(u - (int64_t)t * nseg);
    const int unit = seg * kWave + lane;  // 16-byte unit inside the token data
    const bool active = unit < units;
    u32x4 v = {0u, 0u, 0u, 0u}, hv = {0u, 0u, 0u, 0u};
    if (active) v = __builtin_nontemporal_load((const u32x4*)(a.x + (int64_t)t * a.x_stride) + unit);
    const bool header = seg == 0 && lane < a.hdr_units;  // this lane holds 16 bytes of the header
    if (header) {
        const int32_t* route = a.topk + (int64_t)t * a.topk_stride;
        const float* wt = a.w ? a.w + (int64_t)t * a.w_stride : nullptr;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = lane * 4 + c;  // header word index
            uint32_t word = 0u;
            if (j == 0) word = (uint32_t)t;
            else if (j <= a.K) word = (uint32_t)route[j - 1];
            else if (j <= 2 * a.K) word = wt ? __float_as_uint(wt[j - 1 - a.K]) : __float_as_uint(1.0f);
            hv[c] = word;
        }
    }
    const int my_slot = lane < a.K ? a.rank_row[(int64_t)t * a.K + lane] : -1;
    for (int k = 0; k < a.K; ++k) {
        const int m = __builtin_amdgcn_readlane(my_slot, k);
        if (m < 0) continue;
        if (m >= a.staging_slots) {
            if (seg == 0 && lane == 0) atomicOr(&a.totals[TOT_STATUS], STATUS_OUTPUT_OVERFLOW);
            continue;
        }
        u32x4* msg = (u32x4*)(a.staging + (int64_t)m * a.msg_stride + a.msg_lead);
        if (header) msg[lane] = hv;
        if (active) __builtin_nontemporal_store(v, msg + a.hdr_units + unit);
    }
}

__global__ __launch_bounds__(256) void dedup_fanout_kernel(DedupFanoutArgs a, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (blockIdx.x == 0 && a.recv_count) {
        for (int e = threadIdx.x; e < a.E; e += blockDim.x) a.recv_count[e] = a.recv_kept[e];
    }
    if (u >= (int64_t)a.staging_slots * nseg) return;
    const int m = (int)(u / nseg);
    const int seg = (int)(u - (int64_t)m * nseg);
    // is slot m in use?
    if (a.slots_per_rank > 0) {
        const int d = m / a.slots_per_rank;
        if (m - d * a.slots_per_rank >= a.rank_count[d]) return;
    } else if (m >= a.rank_offset[a.R]) {
        return;
    }
    const int unit = seg * kWave + lane;  // 16-byte unit inside the payload
    const bool active = unit < units;
    const uint8_t* msg = a.staging + (int64_t)m * a.msg_stride + a.msg_lead;
    const int32_t* hdr = (const int32_t*)msg;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (active) v = __builtin_nontemporal_load((const u32x4*)(msg + a.hdr_bytes) + unit);
    const int my_row = lane < a.K ? a.recv_dst_row[(int64_t)m * a.K + lane] : -1;
    for (int k = 0; k < a.K; ++k) {
        const int row = __builtin_amdgcn_readlane(my_row, k);
        if (row < 0) continue;
        if (row >= a.win.rows_cap) {
            if (seg == 0 && lane == 0) atomicOr(&a.totals[TOT_STATUS], STATUS_OUTPUT_OVERFLOW);
            continue;
        }
        uint16_t* dst = a.win.base + window_offset(a.win, row);
        if (active) __builtin_nontemporal_store(v, (u32x4*)dst + unit);
        if (seg == 0 && lane == 0) {
            if (a.recv_w) a.recv_w[row] = __uint_as_float((uint32_t)hdr[1 + a.K + k]);
            if (a.recv_src) a.recv_src[row] = hdr[0];
        }
    }
}

// ---- receiver-side ranking (Sec. IV-C "Dispatch/recv": the receiver places each arriving
// token in the region of every local expert its header names) ----
//
// Window d holds the messages for rank d in slot order; entry (m, k) counts when route[k]
// of message m is one of rank d's L experts.  The row of an entry is
//   concat: expert_offset[e] + (number of earlier entries of the window naming e)
//   padded: e * C + the same number, or none when that number reaches C
// where "earlier" is the order of (slot, k).  The per-expert offsets of the concatenated
// layout are the ones fixed when the handle was made (the per-expert counts are exchanged
// at that point, Sec. III-C).  No atomic decides an order: LDS atomics only add counts.
// The flattened entries of a window are cut into one contiguous range per wavefront;
// histogram per range, running sum down the ranges, then every wave walks its range 64
// entries at a time and ranks equal keys with one ballot per key bit.
constexpr int kRankWaves = 16;
constexpr int kRankCached = 12;  // passes of a wave whose ids stay in registers

__device__ __forceinline__ uint64_t match_bits(int key, bool valid, int nbits) {
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (key >> b) & 1;
        const uint64_t bal = __ballot(valid && bit);
        peers &= bit ? bal : ~bal;
    }
    return valid ? peers : 0ull;
}

__global__ __launch_bounds__(kRankWaves * kWave) void dedup_rank_kernel(DedupRankArgs a, int nw) {
    extern __shared__ int32_t lds[];  // [nw][L] per-wave counts, then per-wave prefixes; [L] first rows
    const int d = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int L = a.L;
    int m0, nmsg;
    if (a.slots_per_rank > 0) {
        m0 = d * a.slots_per_rank;
        nmsg = min(a.rank_count[d], a.slots_per_rank);
    } else {
        m0 = a.rank_offset[d];
        nmsg = a.rank_offset[d + 1] - m0;
    }
    nmsg = max(0, min(nmsg, (int)a.staging_slots - m0));
    const int n = nmsg * a.K;                                       // entries of the window
    const int per = ((n + nw - 1) / nw + kWave - 1) / kWave * kWave;  // entries per wave, whole passes
    const int i0 = w * per, i1 = min(n, i0 + per);
    for (int j = threadIdx.x; j < nw * L; j += blockDim.x) lds[j] = 0;
    int32_t* first_row = lds + nw * L;
    for (int c = threadIdx.x; c < L; c += blockDim.x)
        first_row[c] = a.padded ? (d * L + c) * a.C : a.expert_offset[d * L + c];
    int32_t* h = lds + w * L;
    auto load_id = [&](int i) -> int {  // expert id named by entry i of the window
        const int mi = a.K_shift >= 0 ? (i >> a.K_shift) : (i / a.K);
        const int k = i - mi * a.K;
        return ((const int32_t*)(a.staging + (int64_t)(m0 + mi) * a.msg_stride + a.msg_lead))[1 + k];
    };
    auto local = [&](int e, int* le) -> bool {  // is e one of this window's experts, and which
        if ((unsigned)e >= (unsigned)a.E) return false;
        const int owner = a.L_shift >= 0 ? (e >> a.L_shift) : (e / L);
        *le = e - owner * L;
        return owner == d;
    };
    // the ids of the first kRankCached passes of the wave's range are loaded once, all at
    // the same time, and kept in registers for both sweeps; later passes load again
    int ev[kRankCached];
#pragma unroll
    for (int j = 0; j < kRankCached; ++j) {
        const int i = i0 + j * kWave + lane;
        ev[j] = (w < nw && i < i1) ? load_id(i) : -1;
    }
    __syncthreads();
    if (w < nw) {
#pragma unroll
        for (int j = 0; j < kRankCached; ++j) {
            int le = 0;
            if (local(ev[j], &le)) atomicAdd(&h[le], 1);
        }
        for (int i = i0 + kRankCached * kWave + lane; i < i1; i += kWave) {
            int le = 0;
            if (local(load_id(i), &le)) atomicAdd(&h[le], 1);
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < L; c += blockDim.x) {  // thread = local expert: sums down the waves
        int run = 0;
        for (int r = 0; r < nw; ++r) {
            const int v = lds[r * L + c];
            lds[r * L + c] = run;
            run += v;
        }
        const int e = d * L + c;
        a.recv_count[e] = run;
        a.recv_kept[e] = a.padded ? min(run, a.C) : run;
    }
    __syncthreads();
    if (w >= nw) return;
    const uint64_t lt = (1ull << lane) - 1ull;
    auto place = [&](int i, int e) {  // all 64 lanes take part
        int le = 0;
        const bool ok = i < i1 && local(e, &le);
        const uint64_t peers = match_bits(le, ok, a.bits_l);
        const int rank = __popcll(peers & lt);
        const int slot = ok ? h[le] + rank : -1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        if (ok && rank == 0) h[le] += __popcll(peers);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        if (i < i1) {
            int row = -1;
            if (ok && (!a.padded || slot < a.C)) row = first_row[le] + slot;
            const int mi = a.K_shift >= 0 ? (i >> a.K_shift) : (i / a.K);
            a.recv_dst_row[(int64_t)(m0 + mi) * a.K + (i - mi * a.K)] = row;
        }
    };
#pragma unroll
    for (int j = 0; j < kRankCached; ++j) {
        if (i0 + j * kWave >= i1) break;  // wave-uniform
        place(i0 + j * kWave + lane, ev[j]);
    }
    for (int ib = i0 + kRankCached * kWave; ib < i1; ib += kWave) {
        const int i = ib + lane;
        place(i, i < i1 ? load_id(i) : -1);
    }
}

}  // namespace

hipError_t launch_dedup_rank(const DedupRankArgs& a, hipStream_t s) {
    // as many waves as the per-wave count tables leave room for in 48 KiB of LDS
    int nw = kRankWaves;
    while (nw > 1 && (size_t)(nw + 1) * a.L * sizeof(int32_t) > 48 * 1024) nw >>= 1;
    const size_t lds = (size_t)(nw + 1) * a.L * sizeof(int32_t);
    if (lds > 48 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dedup_rank_kernel, dim3((unsigned)a.R), dim3(kRankWaves * kWave), lds, s, a, nw);
    return hipGetLastError();
}

hipError_t launch_dedup_send(const DedupSendArgs& a, hipStream_t s) {
    const int units = a.H / 8;
    const int nseg = (units + kWave - 1) / kWave;
    const int64_t nwaves = (int64_t)a.T * nseg;
    if (nwaves == 0) return hipSuccess;
    if (a.hdr_units > kWave) return hipErrorInvalidValue;  // the header is built by one wavefront
    const int64_t nblk = (nwaves + 3) / 4;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dedup_send_kernel, dim3((unsigned)nblk), dim3(256), 0, s, a, nseg, units);
    return hipGetLastError();
}

hipError_t launch_dedup_fanout(const DedupFanoutArgs& a, hipStream_t s) {
    const int units = a.H / 8;
    const int nseg = (units + kWave - 1) / kWave;
    const int64_t nwaves = (int64_t)a.staging_slots * nseg;
    int64_t nblk = (nwaves + 3) / 4;
    if (nblk < 1) nblk = 1;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dedup_fanout_kernel, dim3((unsigned)nblk), dim3(256), 0, s, a, nseg, units);
    return hipGetLastError();
}

}  // namespace ep
