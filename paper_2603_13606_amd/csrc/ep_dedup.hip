// Footprint-optimised dispatch (Sec. IV-D): a token is sent ONCE per destination
// rank into that rank's staging window, with the source token index, the routing
// vector and the gate weights in the message header; the receiving side expands
// each message to the local experts its header names (Sec. IV-C "Dispatch/recv").
//
// Message slot = { int32 src_token; int32 route[K]; float w[K]; zero padding to a
// multiple of 16 bytes; 2H bytes of token data }.
//
//   send kernel    work unit = one wavefront x one 1 KiB segment of one token's
//                  message: a lane builds its 16 bytes once (header words or row
//                  data) and stores them to every destination rank's slot.
//   (layout)       the receiving side ranks the header entries of all windows with
//                  the layout kernels in message mode.
//   fan-out kernel work unit = one wavefront x one 1 KiB payload segment of one
//                  staged message: loaded once, stored to each local expert row.
// Pure data movement: HBM bound.  On one GPU this path moves about 2.6x the bytes
// of the direct path; what it saves is staging footprint, O(R*B*P) instead of
// O(E*B*P).
#include "ep_internal.h"

namespace ep {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int64_t window_offset(const WindowDesc& w, int row) {
    if (w.padded) {
        const int e = row / w.C;
        const int s = row - e * w.C;
        return (int64_t)e * w.stride0 + (int64_t)s * w.stride1;
    }
    return (int64_t)row * w.stride0;
}

__global__ __launch_bounds__(256) void dedup_send_kernel(DedupSendArgs a, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (u >= (int64_t)a.T * nseg) return;
    const int t = (int)(u / nseg);
    const int seg = (int)(u - (int64_t)t * nseg);
    const int unit = seg * kWave + lane;  // 16-byte unit inside the message
    const bool active = unit < units;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (active) {
        if (unit < a.hdr_units) {
            const int32_t* route = a.topk + (int64_t)t * a.topk_stride;
            const float* wt = a.w ? a.w + (int64_t)t * a.w_stride : nullptr;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int j = unit * 4 + c;  // header word index
                uint32_t word = 0u;
                if (j == 0) word = (uint32_t)t;
                else if (j <= a.K) word = (uint32_t)route[j - 1];
                else if (j <= 2 * a.K) word = wt ? __float_as_uint(wt[j - 1 - a.K]) : __float_as_uint(1.0f);
                v[c] = word;
            }
        } else {
            v = __builtin_nontemporal_load((const u32x4*)(a.x + (int64_t)t * a.x_stride) + (unit - a.hdr_units));
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
        if (active) __builtin_nontemporal_store(v, (u32x4*)(a.staging + (int64_t)m * a.msg_bytes) + unit);
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
    const uint8_t* msg = a.staging + (int64_t)m * a.msg_bytes;
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

}  // namespace

hipError_t launch_dedup_send(const DedupSendArgs& a, hipStream_t s) {
    const int units = a.hdr_units + a.H / 8;
    const int nseg = (units + kWave - 1) / kWave;
    const int64_t nwaves = (int64_t)a.T * nseg;
    if (nwaves == 0) return hipSuccess;
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
