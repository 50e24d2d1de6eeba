// Pieces shared by the allocation kernels: posterior sources, the per-prompt monotone
// search, and the constants of the threshold search.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hora.h"
#include "hora_device.h"

namespace hora {

constexpr int kBins = 256;        // intervals per narrowing pass of the threshold search
constexpr int kSelectPasses = 9;  // every pass cuts the bracket at least 128-fold: enough for 63 bits

// ----------------------------------------------------------------------------------
// Posterior sources (Sec. 3.2 Eq. 2; App. D for the per-prompt form).
// ----------------------------------------------------------------------------------
struct CountsSource {
    static constexpr bool kHasClasses = true;    // the posterior depends on c[i] only
    const int32_t* c;
    int g0;
    double alpha0, beta0;
    __device__ __forceinline__ bool load(long long i, double& a, double& b) const {
        int x = c[i];
        bool ok = (x >= 0) && (x <= g0);
        x = x < 0 ? 0 : (x > g0 ? g0 : x);
        a = alpha0 + (double)x;
        b = beta0 + (double)(g0 - x);
        return ok;
    }
};

struct PosteriorSource {
    static constexpr bool kHasClasses = false;
    const double* alpha;
    const double* beta;
    __device__ __forceinline__ bool load(long long i, double& a, double& b) const {
        a = alpha[i];
        b = beta[i];
        bool ok = (a > 0.0) && (b > 0.0) && (a < INFINITY) && (b < INFINITY);
        if (!ok) { a = 1.0; b = 1.0; }
        return ok;
    }
};

__device__ __forceinline__ unsigned long long read_lane_u64(unsigned long long v, int src) {
    unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v & 0xffffffffull), src);
    unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), src);
    return ((unsigned long long)hi << 32) | lo;
}

// Number of gains of one prompt that exceed tau, at most `limit`; also leaves the next
// gain (the first one <= tau) in `g`, l as a double in `lf` and, if asked, the survival
// product E(k) in `e`.
template <bool kSurvival>
__device__ __forceinline__ long long walk_above(double a, double b, unsigned long long tau_bits, long long limit,
                                                double& g, double& lf, double& e) {
    const double s = a + b;
    g = gain_first(a, s);
    lf = 0.0;
    e = 1.0;
    long long k = 0;
    while (k < limit && gain_bits(g) > tau_bits) {
        if (kSurvival) e = surv_next(e, b, s, lf);
        g = gain_next(g, b, s, lf);
        lf += 1.0;
        k += 1;
    }
    return k;
}

// A batch small enough for one workgroup, solved in a single launch (defined with the
// sharded kernels, whose workgroup-per-shard code it reuses).
int allocate_small_counts(const CountsSource& src, int64_t n, int32_t g0, int64_t budget, int32_t delta_max,
                          int32_t* delta, double* util, void* group_off, int32_t off_t, hora_alloc_summary* summary,
                          int32_t* dev_status, hipStream_t stream);
int allocate_small_posterior(const PosteriorSource& src, int64_t n, int32_t g0, int64_t budget, int32_t delta_max,
                             int32_t* delta, double* util, void* group_off, int32_t off_t,
                             hora_alloc_summary* summary, int32_t* dev_status, hipStream_t stream);

}  // namespace hora
