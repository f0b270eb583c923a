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

__global__ __launch_bounds__(256) void dispatch_direct_kernel(DispatchArgs a, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    if (blockIdx.x == 0 && a.recv_count) {
        for (int e = threadIdx.x; e < a.E; e += blockDim.x) a.recv_count[e] = a.expert_kept[e];
    }
    if (u >= (int64_t)a.T * nseg) return;
    const int t = (int)(u / nseg);
    const int seg = (int)(u - (int64_t)t * nseg);
    const int unit = seg * kWave + lane;
    const bool active = unit < units;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (active) v = __builtin_nontemporal_load((const u32x4*)(a.x + (int64_t)t * a.x_stride) + unit);
    const int32_t* rows = a.dst_row + (int64_t)t * a.K;
    for (int k = 0; k < a.K; ++k) {
        const int row = __builtin_amdgcn_readfirstlane(rows[k]);
        if (row < 0) continue;
        if (row >= a.win.rows_cap) {
            if (seg == 0 && lane == 0) atomicOr(&a.totals[TOT_STATUS], STATUS_OUTPUT_OVERFLOW);
            continue;
        }
        uint16_t* dst = a.win.base + window_offset(a.win, row);
        if (active) __builtin_nontemporal_store(v, (u32x4*)dst + unit);
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

}  // namespace

hipError_t launch_calibration_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const int64_t n16 = (int64_t)(bytes / 16);
    if (n16 == 0) return hipSuccess;
    int64_t nblk = (n16 + 255) / 256;
    if (nblk > 256 * 64) nblk = 256 * 64;
    hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)nblk), dim3(256), 0, s, (u32x4*)dst,
                       (const u32x4*)src, n16);
    return hipGetLastError();
}

hipError_t launch_dispatch(const DispatchArgs& a, hipStream_t s) {
    const int units = a.H / 8;  // 16-byte units per row
    const int nseg = (units + kWave - 1) / kWave;
    const int64_t nwaves = (int64_t)a.T * nseg;
    int64_t nblk = (nwaves + 3) / 4;
    if (nblk < 1) nblk = 1;  // block 0 also copies the per-expert counts
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(dispatch_direct_kernel, dim3((unsigned)nblk), dim3(256), 0, s, a, nseg, units);
    return hipGetLastError();
}

}  // namespace ep
