// Staged execution (Sec. III-B "send_only", Sec. III-F decode pattern) and the
// coordination counters of Sec. IV-B / IV-D.
//
// A staged call runs only the send phase and then performs the "update-and-flush":
// for dispatch the counter of every (expert, this source) pair is set to m + 1, m =
// rows sent for that pair (Sec. IV-B: the +1 makes the update visible when m = 0); on
// the once-per-rank path the counters are per destination rank and carry the number of
// messages + 1; for combine every counter is set to 1.  ep_complete is the receive
// phase: it waits until every counter of the pending call is non-zero, learns the
// counts from them, clears them for the next use, and finishes the call (per-expert
// counts, receiver-side ranking and fan-out, or the reduction).
//
// Counters are published with release stores and read with acquire loads at agent
// scope, so the two phases may run on different streams.  The wait is bounded: after
// spin_limit polls a thread gives up, flags STATUS_TIMEOUT and reports a count of 0, so
// every wave exits whatever the sender does.
#include "ep_internal.h"

namespace ep {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void publish_counts_kernel(int32_t* sig, const int32_t* counts, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const int v = counts ? counts[i] + 1 : 1;
        __hip_atomic_store(&sig[i], v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// One workgroup.  count_out[i] = sig[i] - 1 (0 on time-out); offset_out (optional,
// n + 1 entries) = exclusive prefix sum of the counts; sig[i] is cleared.
__global__ __launch_bounds__(1024) void await_counts_kernel(int32_t* sig, int n, int spin_limit,
                                                             int32_t* count_out, int32_t* offset_out,
                                                             int32_t* totals) {
    __shared__ int32_t cnt[kMaxExperts + 1];
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        int v = 0;
        for (int spins = 0; spins <= spin_limit; ++spins) {
            v = __hip_atomic_load(&sig[i], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
            if (v != 0) break;
            __builtin_amdgcn_s_sleep(8);
        }
        if (v == 0) atomicOr(&totals[TOT_STATUS], STATUS_TIMEOUT);
        const int c = v > 0 ? v - 1 : 0;
        cnt[i] = c;
        if (count_out) count_out[i] = c;
        __hip_atomic_store(&sig[i], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (offset_out && threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < n; ++i) { offset_out[i] = run; run += cnt[i]; }
        offset_out[n] = run;
    }
}

__global__ __launch_bounds__(256) void clear_counts_kernel(int32_t* sig, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x)
        __hip_atomic_store(&sig[i], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Send phase of a staged combine (Sec. IV-D): the expert side packs its outputs into
// the source's staging at slot t*K + k -- no wasted slots, O(B*K*P).  Work unit = one
// wavefront x one 1 KiB segment of one (t, k) entry.
__global__ __launch_bounds__(256) void combine_pack_kernel(CombineArgs a, uint16_t* stage, int nseg, int units) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t u = (int64_t)blockIdx.x * 4 + wave;
    const int64_t entries = (int64_t)a.T * a.K;
    if (u >= entries * nseg) return;
    const int64_t i = u / nseg;
    const int seg = (int)(u - i * nseg);
    const int row = __builtin_amdgcn_readfirstlane(a.dst_row[i]);
    if (row < 0 || row >= a.win.rows_cap) return;
    const int unit = seg * kWave + lane;
    if (unit < units) {
        const u32x4 v = __builtin_nontemporal_load((const u32x4*)(a.win.base + window_offset(a.win, row)) + unit);
        __builtin_nontemporal_store(v, (u32x4*)(stage + i * a.H) + unit);
    }
}

}  // namespace

hipError_t launch_publish_counts(int32_t* sig, const int32_t* counts, int n, hipStream_t s) {
    hipLaunchKernelGGL(publish_counts_kernel, dim3((n + 255) / 256), dim3(256), 0, s, sig, counts, n);
    return hipGetLastError();
}

hipError_t launch_await_counts(int32_t* sig, int n, int spin_limit, int32_t* count_out, int32_t* offset_out,
                               int32_t* totals, hipStream_t s) {
    if (n > kMaxExperts) return hipErrorInvalidValue;
    hipLaunchKernelGGL(await_counts_kernel, dim3(1), dim3(n <= 256 ? 256 : 1024), 0, s, sig, n, spin_limit,
                       count_out, offset_out, totals);
    return hipGetLastError();
}

hipError_t launch_clear_counts(int32_t* sig, int n, hipStream_t s) {
    hipLaunchKernelGGL(clear_counts_kernel, dim3((n + 255) / 256), dim3(256), 0, s, sig, n);
    return hipGetLastError();
}

hipError_t launch_combine_pack(const CombineArgs& a, uint16_t* stage, hipStream_t s) {
    const int units = a.H / 8;
    const int nseg = (units + kWave - 1) / kWave;
    const int64_t nwaves = (int64_t)a.T * a.K * nseg;
    if (nwaves == 0) return hipSuccess;
    const int64_t nblk = (nwaves + 3) / 4;
    if (nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(combine_pack_kernel, dim3((unsigned)nblk), dim3(256), 0, s, a, stage, nseg, units);
    return hipGetLastError();
}

}  // namespace ep
