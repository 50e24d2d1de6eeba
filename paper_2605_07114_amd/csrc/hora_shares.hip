// Allocation statistics per Phase-A outcome (Sec. 4, "Allocation dynamics" and the figure that
// goes with it: which share of the prompts has c_i = k, and which share of the Phase-B budget
// those prompts received).  One pass over c and delta: per-workgroup tallies in LDS (integer
// atomics, one wavefront ballot per class instead of one atomic per prompt), then one 64-bit
// atomic per class and workgroup on the outputs, which a small kernel zeroes first.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"

namespace hora {

constexpr int kShareClasses = HORA_CLASS_MAX_G0 + 1;
constexpr int kShareBlocks = 512;       // workgroups, at most

__global__ void k_shares_zero(long long* __restrict__ class_count, long long* __restrict__ class_budget, int nc) {
    const int t = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (t < nc) { class_count[t] = 0; class_budget[t] = 0; }
}

__global__ __launch_bounds__(kThreads) void k_shares(long long n, int g0, const int32_t* __restrict__ c,
                                                     const int32_t* __restrict__ delta,
                                                     long long* __restrict__ class_count,
                                                     long long* __restrict__ class_budget, int32_t* dev_status) {
    __shared__ unsigned long long s_cnt[kShareClasses], s_sum[kShareClasses];
    if (threadIdx.x < kShareClasses) { s_cnt[threadIdx.x] = 0ull; s_sum[threadIdx.x] = 0ull; }
    __syncthreads();
    const int nc = g0 + 1;
    const int lane = lane_id();
    unsigned long long my_cnt = 0, my_sum = 0;     // lane k of every wavefront gathers class k
    bool bad = false;
    const long long stride = (long long)gridDim.x * kThreads;
    // whole wavefronts run every round, so that the ballots below see all lanes
    for (long long i0 = (long long)blockIdx.x * kThreads; i0 < n; i0 += stride) {
        const long long i = i0 + threadIdx.x;
        int x = -1, d = 0;
        if (i < n) {
            x = c[i];
            d = delta[i];
            if (x < 0 || x > g0 || d < 0) { bad = true; x = -1; }
        }
        for (int k = 0; k < nc; ++k) {
            const bool mine = x == k;
            const unsigned long long m = __ballot(mine);
            if (m == 0ull) continue;               // uniform
            const long long units = wave_sum<long long>(mine ? (long long)d : 0ll);
            if (lane == k) { my_cnt += (unsigned long long)__popcll(m); my_sum += (unsigned long long)units; }
        }
    }
    if (lane < nc && my_cnt) { atomicAdd(&s_cnt[lane], my_cnt); atomicAdd(&s_sum[lane], my_sum); }
    __syncthreads();
    if (threadIdx.x < (unsigned)nc && s_cnt[threadIdx.x]) {
        atomicAdd((unsigned long long*)&class_count[threadIdx.x], s_cnt[threadIdx.x]);
        atomicAdd((unsigned long long*)&class_budget[threadIdx.x], s_sum[threadIdx.x]);
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

}  // namespace hora

using namespace hora;

extern "C" int hora_allocation_shares(int64_t n, int32_t g0, const int32_t* c, const int32_t* delta,
                                      int64_t* class_count, int64_t* class_budget, int32_t* dev_status,
                                      void* stream) {
    if (n < 0 || g0 < 0 || !dev_status || !class_count || !class_budget) return HORA_ERR_INVALID_ARG;
    if (g0 > HORA_CLASS_MAX_G0) return HORA_ERR_UNSUPPORTED;
    if (n > 0 && (!c || !delta)) return HORA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(c) & 3) || (reinterpret_cast<uintptr_t>(delta) & 3) ||
        (reinterpret_cast<uintptr_t>(class_count) & 7) || (reinterpret_cast<uintptr_t>(class_budget) & 7) ||
        (reinterpret_cast<uintptr_t>(dev_status) & 3))
        return HORA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_shares_zero, dim3(1), dim3(kShareClasses), 0, s, (long long*)class_count,
                       (long long*)class_budget, (int)g0 + 1);
    if (n > 0) {
        long long blocks = (n + kThreads - 1) / kThreads;
        if (blocks > kShareBlocks) blocks = kShareBlocks;
        hipLaunchKernelGGL(k_shares, dim3((unsigned)blocks), dim3(kThreads), 0, s, (long long)n, (int)g0, c, delta,
                           (long long*)class_count, (long long*)class_budget, dev_status);
    }
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}
