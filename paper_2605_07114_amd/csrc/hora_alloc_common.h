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

// ----------------------------------------------------------------------------------
// Tallies of one pass of the threshold search.  The bracket (lo, hi] of tau's bit pattern is
// cut into at most kBins intervals of 2^shift patterns; per interval the number of gains that
// fall inside, and the largest and smallest pattern seen there, are kept.
// ----------------------------------------------------------------------------------
struct TallyBins {
    unsigned long long cnt[kBins];       // pairs whose gain falls into the interval
    unsigned long long vmax[kBins];      // largest gain pattern seen in the interval
    unsigned long long vmin_inv[kBins];  // ~(smallest gain pattern seen in the interval)
};

// log2 of the interval width for the bracket (lo, hi]: ((v - lo - 1) >> shift) < kBins for lo < v <= hi.
__device__ __forceinline__ int bracket_shift(unsigned long long lo, unsigned long long hi) {
    const unsigned long long width = hi - lo;                  // >= 1
    const int bitlen = width > 1 ? 64 - __clzll((long long)(width - 1)) : 0;   // bits of width - 1
    // The bracket is the same in every lane.  The shift amount is handed on in a scalar register:
    // a 64-bit shift that takes its amount from the last vector register of the wavefront's
    // allocation shifts by a wrong amount on gfx950, and nothing in the source decides which
    // register the compiler picks.
    return __builtin_amdgcn_readfirstlane(bitlen > 8 ? bitlen - 8 : 0);
}

// Every lane of a wavefront offers one gain pattern (`inside` says whether it lies in the
// bracket); all of them are tallied into `bins` (LDS).  Lanes that hold the same gain (the
// rule under a shared prior) tally once, through a leader: up to 8 distinct gains per call
// that way, the rest lane by lane.  A wavefront whose first pending gain does not repeat
// (per-prompt posteriors never repeat) skips the merging, which is scalar-heavy.
// Must be called by whole wavefronts.
__device__ __forceinline__ void tally_gains(TallyBins& bins, bool inside, unsigned long long gb,
                                            unsigned long long lo, int shift) {
    const int lane = lane_id();
    shift = __builtin_amdgcn_readfirstlane(shift);   // uniform; see bracket_shift
    bool todo = inside;                              // this lane's gain has not been tallied yet
    unsigned long long pending = __ballot(todo);
    for (int round = 0; round < 8 && pending; ++round) {
        const int leader = __ffsll((long long)pending) - 1;
        const unsigned long long v = read_lane_u64(gb, leader);
        const bool match = todo && gb == v;
        const unsigned long long same = __ballot(match);
        if (round == 0 && same == (1ull << leader)) break;
        if (lane == leader) {
            const int j = (int)((v - lo - 1ull) >> shift);
            // no result is used: the three updates are issued without a wait
            atomicAdd(&bins.cnt[j], (unsigned long long)__popcll(same));
            atomicMax(&bins.vmax[j], v);
            atomicMax(&bins.vmin_inv[j], ~v);
        }
        todo = todo && !match;
        pending &= ~same;
    }
    if (todo) {
        const int j = (int)((gb - lo - 1ull) >> shift);
        atomicAdd(&bins.cnt[j], 1ull);
        atomicMax(&bins.vmax[j], gb);
        atomicMax(&bins.vmin_inv[j], ~gb);
    }
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
