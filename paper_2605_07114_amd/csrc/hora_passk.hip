// Unbiased Pass@K estimator (Sec. 4, Eq. 6): for every problem with N samples of which c
// are correct, 1 - C(N - c, K) / C(N, K); the benchmark value is the mean over the
// problems.  The ratio of the two binomial coefficients is evaluated as a product of
// min(c, K) quotients,
//   C(N-c, K) / C(N, K) = prod_{j<c} (N-K-j)/(N-j) = prod_{j<K} (N-c-j)/(N-j),
// in binary64, which stays within a few ulp per factor of the exact value and never
// forms the (huge) coefficients themselves.  Means are two-stage sums: per workgroup, then
// one workgroup per K over the partial sums, in a fixed order.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"

namespace hora {

constexpr int kMaxK = 64;           // values of K per call
constexpr int kPassBlocks = 256;    // workgroups (partial sums) per K, at most

struct KList { int k[kMaxK]; };

__device__ __forceinline__ double pass_at_k_one(int n, int c, int k) {
    if (n - c < k) return 1.0;                 // every K-subset holds a correct sample
    const int terms = c < k ? c : k;
    const int other = c < k ? k : c;           // the product runs over the smaller of the two
    double ratio = 1.0;
    for (int j = 0; j < terms; ++j) ratio = ratio * ((double)(n - other - j) / (double)(n - j));
    return 1.0 - ratio;
}

__global__ __launch_bounds__(kThreads) void k_pass_at_k(long long n_problems, const int32_t* __restrict__ n_samples,
                                                        const int32_t* __restrict__ correct, KList ks,
                                                        double* __restrict__ per_problem,
                                                        double* __restrict__ partial, int32_t* dev_status) {
    __shared__ double s_red[kWaves];
    const int k = ks.k[blockIdx.y];
    double sum = 0.0;
    bool bad = false;
    const long long stride = (long long)gridDim.x * kThreads;
    for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < n_problems; i += stride) {
        const int n = n_samples[i], c = correct[i];
        double v = 0.0;
        if (n < 1 || c < 0 || c > n || k < 1 || k > n) bad = true;
        else v = pass_at_k_one(n, c, k);
        if (per_problem) per_problem[(long long)blockIdx.y * n_problems + i] = v;
        sum += v;
    }
    sum = block_sum<double>(sum, s_red);
    if (threadIdx.x == 0) partial[(long long)blockIdx.y * gridDim.x + blockIdx.x] = sum;
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

__global__ __launch_bounds__(kWave) void k_pass_mean(long long n_problems, int blocks, const double* __restrict__ partial,
                                                     double* __restrict__ mean) {
    double sum = 0.0;
    for (int b = (int)threadIdx.x; b < blocks; b += kWave) sum += partial[(long long)blockIdx.x * blocks + b];
    sum = wave_sum<double>(sum);
    if (threadIdx.x == 0) mean[blockIdx.x] = n_problems > 0 ? sum / (double)n_problems : 0.0;
}

static int pass_blocks(int64_t n_problems) {
    long long b = (n_problems + kThreads - 1) / kThreads;
    if (b < 1) b = 1;
    return (int)(b > kPassBlocks ? kPassBlocks : b);
}

}  // namespace hora

using namespace hora;

extern "C" size_t hora_pass_at_k_workspace_bytes(int64_t n_problems, int32_t n_k) {
    if (n_problems < 0 || n_k < 0 || n_k > kMaxK) return 0;
    return (((size_t)(n_k > 0 ? n_k : 1) * pass_blocks(n_problems) * sizeof(double)) + 255) & ~(size_t)255;
}

extern "C" int hora_pass_at_k(int64_t n_problems, const int32_t* n_samples, const int32_t* correct, int32_t n_k,
                              const int32_t* ks, double* per_problem, double* mean, int32_t* dev_status,
                              void* workspace, size_t workspace_bytes, void* stream) {
    if (n_problems < 0 || n_k < 0 || !dev_status) return HORA_ERR_INVALID_ARG;
    if (n_k > kMaxK) return HORA_ERR_UNSUPPORTED;
    if (n_k == 0) return HORA_OK;
    if (!ks || !mean) return HORA_ERR_INVALID_ARG;
    if (n_problems > 0 && (!n_samples || !correct)) return HORA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(n_samples) & 3) || (reinterpret_cast<uintptr_t>(correct) & 3) ||
        (reinterpret_cast<uintptr_t>(per_problem) & 7) || (reinterpret_cast<uintptr_t>(mean) & 7))
        return HORA_ERR_INVALID_ARG;
    KList list;
    for (int i = 0; i < kMaxK; ++i) list.k[i] = i < n_k ? ks[i] : 1;
    for (int i = 0; i < n_k; ++i)
        if (ks[i] < 1) return HORA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 7)) return HORA_ERR_WORKSPACE;
    if (workspace_bytes < hora_pass_at_k_workspace_bytes(n_problems, n_k)) return HORA_ERR_WORKSPACE;
    const int blocks = pass_blocks(n_problems);
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(k_pass_at_k, dim3((unsigned)blocks, (unsigned)n_k), dim3(kThreads), 0, s,
                       (long long)n_problems, n_samples, correct, list, per_problem, (double*)workspace, dev_status);
    hipLaunchKernelGGL(k_pass_mean, dim3((unsigned)n_k), dim3(kWave), 0, s, (long long)n_problems, blocks,
                       (const double*)workspace, mean);
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}
