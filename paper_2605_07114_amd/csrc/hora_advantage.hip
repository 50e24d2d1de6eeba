// Group-relative advantages over variable-size groups (Sec. 3.1 GRPO; Sec. 4 / App. E RLOO),
// and the per-response loss weights of the objective with variable-size groups (Sec. 3.2).
//
// A sub-group of L lanes (L a power of two, chosen from the mean group size) owns one
// group.  Every lane takes runs of 16 bytes of the group's rewards (four floats, two doubles),
// one load or store per run, so that the lanes of a group cover whole cache lines; the lanes
// combine their partial sums with a butterfly.  A group of up to 8 L (or 16 L) responses,
// 1.75 times the mean or more, is read once and kept in registers: two dependent memory round
// trips per wavefront, offsets then rewards.  What is computed once per group (mean, standard
// deviation, reciprocals) is repeated by its L lanes.
// All sums are binary64; a float output is rounded once at the store.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"

namespace hora {

// Cross-lane steps inside a sub-group of L lanes.  Inside a row of 16 lanes they are DPP
// operand modifiers (register moves: quad permutations, the mirror of 8 and of 16 lanes); only
// what crosses rows takes the LDS-routed shuffle.  A double moves as two halves.
template <int kCtrl>
__device__ __forceinline__ int dpp_take(int v) {
    return __builtin_amdgcn_update_dpp(0, v, kCtrl, 0xf, 0xf, true);
}
template <int kCtrl>
__device__ __forceinline__ double dpp_take(double v) {
    const long long bits = __double_as_longlong(v);
    const int lo = dpp_take<kCtrl>((int)(unsigned)((unsigned long long)bits & 0xffffffffull));
    const int hi = dpp_take<kCtrl>((int)(unsigned)((unsigned long long)bits >> 32));
    return __longlong_as_double((long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo));
}
constexpr int kQuadXor1 = 0xb1, kQuadXor2 = 0x4e;       // quad_perm [1,0,3,2], [2,3,0,1]
constexpr int kHalfMirror = 0x141, kRowMirror = 0x140;  // lane i <-> 7 - i, 15 - i inside its row

template <int L>
__device__ __forceinline__ double sub_sum(double v) {
    // quads first, then the other quad of the 8 (any of its lanes holds its sum), then the other 8
    if (L >= 2) v += dpp_take<kQuadXor1>(v);
    if (L >= 4) v += dpp_take<kQuadXor2>(v);
    if (L >= 8) v += dpp_take<kHalfMirror>(v);
    if (L >= 16) v += dpp_take<kRowMirror>(v);
#pragma unroll
    for (int d = 16; d < L; d <<= 1) v += __shfl_xor(v, d, L);
    return v;
}

// 1 / d for d > 0: the hardware's approximation, two Newton steps and a residual step (the
// division's own sequence without its scaling and special cases): the rounded quotient
// where d and 1 / d are normal numbers (beyond that it ends in 0 or infinity like the
// quotient does), at a quarter of the instructions of a division; every lane of a group
// repeats it.
__device__ __forceinline__ double reciprocal(double d) {
    double r = __builtin_amdgcn_rcp(d);
    r = __builtin_fma(__builtin_fma(-d, r, 1.0), r, r);
    r = __builtin_fma(__builtin_fma(-d, r, 1.0), r, r);
    return __builtin_fma(__builtin_fma(-d, r, 1.0), r, r);   // (the division's own last step: the residual of the quotient)
}

template <int L>
__device__ __forceinline__ int sub_and(int v) {
    if (L >= 2) v &= dpp_take<kQuadXor1>(v);
    if (L >= 4) v &= dpp_take<kQuadXor2>(v);
    if (L >= 8) v &= dpp_take<kHalfMirror>(v);
    if (L >= 16) v &= dpp_take<kRowMirror>(v);
#pragma unroll
    for (int d = 16; d < L; d <<= 1) v &= __shfl_xor(v, d, L);
    return v;
}

// The value of the sub-group's first lane, in all of its lanes.
template <int L>
__device__ __forceinline__ double sub_first(double v) {
    if (L == 1) return v;
    if (L == 2) return dpp_take<0xa0>(v);   // quad_perm [0,0,2,2]
    if (L == 4) return dpp_take<0x00>(v);   // quad_perm [0,0,0,0]
    return __shfl(v, 0, L);
}

// Rewards a lane keeps in registers: a group of up to L * kKeep responses is read from
// memory once; what lies beyond is read again in every pass.  A lane's rewards are runs of
// 16 bytes (four floats, two doubles), moved by one load or store each: the four lanes of a
// group then cover whole 64-byte lines, where single elements per lane would make every
// instruction touch a quarter of each line it visits (the address path, not the memory,
// bounded that form at 0.4 of the peak).

template <typename F> struct Run;
template <> struct Run<float> { static constexpr int kPer = 4; typedef float V __attribute__((ext_vector_type(4), aligned(4))); };
template <> struct Run<double> { static constexpr int kPer = 2; typedef double V __attribute__((ext_vector_type(2), aligned(8))); };

template <typename F, typename I, int L, int kKeep>
__global__ __launch_bounds__(kThreads) void k_group_adv(long long n_groups, const I* __restrict__ off,
                                                        long long n_resp, const F* __restrict__ reward,
                                                        F* __restrict__ adv, int mode, double eps, int ddof,
                                                        int32_t* dev_status) {
    constexpr int kPer = Run<F>::kPer;        // responses per run
    constexpr int kRuns = kKeep / kPer;       // runs per lane
    typedef typename Run<F>::V V;
    const int sub = (int)(threadIdx.x % L);
    const long long g = ((long long)blockIdx.x * kThreads + threadIdx.x) / L;
    const bool live = g < n_groups;
    long long lo = 0, hi = 0;
    if (live) {
        lo = (long long)off[g];
        hi = (long long)off[g + 1];
        bool bad = lo < 0 || hi < lo || hi > n_resp;
        if (g == 0 && lo != 0) bad = true;
        if (g == n_groups - 1 && hi != n_resp) bad = true;
        if (bad) {
            if (sub == 0) report(dev_status, HORA_ERR_RANGE);
            lo = lo < 0 ? 0 : (lo > n_resp ? n_resp : lo);
            hi = hi < lo ? lo : (hi > n_resp ? n_resp : hi);
        }
    }
    const long long size = hi - lo;
    // run r of this lane holds the responses lo + kPer * (sub + L * r) + i, i < kPer
    const long long rest = lo + (long long)kKeep * L + sub;    // this lane's first response beyond the registers (stride L)

    // one round of loads: whole runs where the array allows it (what lies beyond the group
    // but inside the array is loaded and not used)
    double x[kKeep];
    bool in[kKeep];
    const F* const src0 = reward + lo + kPer * sub;    // this lane's first run
    F* const dst0 = adv + lo + kPer * sub;
    // responses of the group from this lane's first run on (as far as the registers reach)
    int ahead = (int)(size - kPer * sub < (long long)kKeep * L ? (size - kPer * sub > 0 ? size - kPer * sub : 0)
                                                              : (long long)kKeep * L);
    // (the compiler is kept from folding the 32-bit count back into 64-bit comparisons with the group's size)
    asm volatile("" : "+v"(ahead));
#pragma unroll
    for (int r = 0; r < kRuns; ++r) {
        const int at = kPer * L * r;                   // from this lane's first run
        const F* src = src0 + at;
        const int have = ahead - at;                   // responses of the group from this run on (may be <= 0)
        F raw[kPer];
        if (have > 0 && lo + kPer * sub + at + kPer <= n_resp) {
            const V v = *reinterpret_cast<const V*>(src);
#pragma unroll
            for (int i = 0; i < kPer; ++i) raw[i] = v[i];
        } else {
#pragma unroll
            for (int i = 0; i < kPer; ++i) raw[i] = i < have ? src[i] : (F)0;
        }
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            in[r * kPer + i] = i < have;
            x[r * kPer + i] = (double)(in[r * kPer + i] ? raw[i] : (F)0);
        }
    }
    const double first = sub_first<L>(x[0]);   // reward[lo] (0 for an empty group)
    double sum = 0.0;
    int equal = 1;
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
        sum += x[k];
        equal &= (!in[k] || x[k] == first) ? 1 : 0;
    }
    for (long long j = rest; j < hi; j += L) {
        const double y = (double)reward[j];
        sum += y;
        equal &= (y == first) ? 1 : 0;
    }
    sum = sub_sum<L>(sum);
    equal = sub_and<L>(equal);

    // the kept responses go back run by run: one store where the whole run is the group's
    auto put = [&](const double (&y)[kKeep]) {
#pragma unroll
        for (int r = 0; r < kRuns; ++r) {
            F* dst = dst0 + kPer * L * r;
            if (in[r * kPer + kPer - 1]) {
                V v;
#pragma unroll
                for (int i = 0; i < kPer; ++i) v[i] = (F)y[r * kPer + i];
                *reinterpret_cast<V*>(dst) = v;
            } else {
#pragma unroll
                for (int i = 0; i < kPer; ++i)
                    if (in[r * kPer + i]) dst[i] = (F)y[r * kPer + i];
            }
        }
    };
    double y[kKeep];

    // Every quotient whose divisor belongs to the group is formed as a product with the
    // divisor's reciprocal (`reciprocal`: once per lane instead of a division per response):
    // a few units in the last place away from the quotient itself, against a tolerance of 1e-12.
    if (mode == HORA_ADV_RLOO) {
        // (a group of one, or of equal rewards, gets exact zeros: both factors vanish)
        const bool none = size <= 1 || equal;
        const double inv = none ? 0.0 : reciprocal((double)(size - 1));
        const double own = none ? 0.0 : 1.0;
        // (product and difference rounded separately, as the definition's quotient and difference
        // are: a response that equals the mean of the others gets an exact zero where it does there)
#pragma unroll
        for (int k = 0; k < kKeep; ++k) y[k] = own * x[k] - (sum - x[k]) * inv;
        put(y);
        for (long long j = rest; j < hi; j += L) {
            const double z = (double)reward[j];
            adv[j] = (F)(own * z - (sum - z) * inv);
        }
        return;
    }

    const double mean = size > 0 ? sum * reciprocal((double)size) : 0.0;
    if (mode == HORA_ADV_CENTER) {
#pragma unroll
        for (int k = 0; k < kKeep; ++k) y[k] = equal ? 0.0 : x[k] - mean;
        put(y);
        for (long long j = rest; j < hi; j += L) {
            const double z = (double)reward[j];
            adv[j] = (F)(equal ? 0.0 : z - mean);
        }
        return;
    }
    const bool zero = equal || (size - ddof <= 0);
    double ss = 0.0;
    if (!zero) {
#pragma unroll
        for (int k = 0; k < kKeep; ++k) {
            const double d = x[k] - mean;
            ss += in[k] ? d * d : 0.0;
        }
        for (long long j = rest; j < hi; j += L) {
            const double d = (double)reward[j] - mean;
            ss += d * d;
        }
    }
    ss = sub_sum<L>(ss);
    const double inv = zero ? 0.0 : reciprocal(sqrt(ss * reciprocal((double)(size - ddof))) + eps);
    // (inv = 0 for a group without variance: the sum with +0 makes every product a +0)
#pragma unroll
    for (int k = 0; k < kKeep; ++k) y[k] = __builtin_fma(x[k] - mean, inv, 0.0);
    put(y);
    for (long long j = rest; j < hi; j += L) {
        const double z = (double)reward[j];
        adv[j] = (F)__builtin_fma(z - mean, inv, 0.0);
    }
}

template <typename F, typename I, int kKeep>
static int launch_adv_keep(int64_t n_groups, const void* off, int64_t n_resp, const void* reward, void* adv,
                           int mode, double eps, int ddof, int32_t* dev_status, hipStream_t stream) {
    // lanes per group: the fewest whose registers hold a group of 1.75 times the mean size
    const long long roomy = n_groups > 0 ? (7 * n_resp + 4 * n_groups - 1) / (4 * n_groups) : 0;
    int lanes = 1;
    while (lanes < kWave && (long long)lanes * kKeep < roomy) lanes *= 2;
#define HORA_LAUNCH_ADV(LL)                                                                                   \
    do {                                                                                                      \
        const long long blocks = (n_groups * LL + kThreads - 1) / kThreads;                                   \
        if (blocks > INT_MAX) return HORA_ERR_UNSUPPORTED;                                                    \
        hipLaunchKernelGGL((k_group_adv<F, I, LL, kKeep>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, \
                           (long long)n_groups, (const I*)off, (long long)n_resp, (const F*)reward, (F*)adv,  \
                           mode, eps, ddof, dev_status);                                                      \
    } while (0)
    switch (lanes) {
        case 1: HORA_LAUNCH_ADV(1); break;
        case 2: HORA_LAUNCH_ADV(2); break;
        case 4: HORA_LAUNCH_ADV(4); break;
        case 8: HORA_LAUNCH_ADV(8); break;
        case 16: HORA_LAUNCH_ADV(16); break;
        case 32: HORA_LAUNCH_ADV(32); break;
        default: HORA_LAUNCH_ADV(64); break;
    }
#undef HORA_LAUNCH_ADV
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

// Responses a lane keeps: eight, or sixteen where the work per group is large next to the
// work per response (float rewards with the standard deviation: two divisions and a square
// root per group and lane): twice the responses per lane halve the lanes that repeat it.
template <typename F, typename I>
static int launch_adv(int64_t n_groups, const void* off, int64_t n_resp, const void* reward, void* adv, int mode,
                      double eps, int ddof, int32_t* dev_status, hipStream_t stream) {
    if (sizeof(F) == 4 && mode == HORA_ADV_GRPO)
        return launch_adv_keep<F, I, 16>(n_groups, off, n_resp, reward, adv, mode, eps, ddof, dev_status, stream);
    return launch_adv_keep<F, I, 8>(n_groups, off, n_resp, reward, adv, mode, eps, ddof, dev_status, stream);
}

// Loss weight of the tokens of every response: 1 / (G_i * |o_j|), or 1 / (G_i * L) with a
// constant L in place of the response length; 0 for a response without tokens.  kLanes
// lanes stride over the responses of one group.
constexpr int kWeightLanes = 8;

template <typename F, typename IG, typename IT>
__global__ __launch_bounds__(kThreads) void k_response_weights(long long n_groups, const IG* __restrict__ group_off,
                                                               long long n_resp, const IT* __restrict__ tok_off,
                                                               double length_const, F* __restrict__ weight,
                                                               int32_t* dev_status) {
    const int sub = (int)(threadIdx.x % kWeightLanes);
    const long long g = ((long long)blockIdx.x * kThreads + threadIdx.x) / kWeightLanes;
    if (g >= n_groups) return;
    long long lo = (long long)group_off[g], hi = (long long)group_off[g + 1];
    bool bad = lo < 0 || hi < lo || hi > n_resp || (g == 0 && lo != 0) || (g == n_groups - 1 && hi != n_resp);
    if (bad) {
        lo = lo < 0 ? 0 : (lo > n_resp ? n_resp : lo);
        hi = hi < lo ? lo : (hi > n_resp ? n_resp : hi);
    }
    const double size = (double)(hi - lo);
    for (long long j = lo + sub; j < hi; j += kWeightLanes) {
        const long long len = (long long)tok_off[j + 1] - (long long)tok_off[j];
        bad |= len < 0;
        const double norm = length_const > 0.0 ? length_const : (double)len;
        weight[j] = (F)(len <= 0 ? 0.0 : 1.0 / (size * norm));
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

template <typename F, typename IG, typename IT>
static int launch_weights(int64_t n_groups, const void* group_off, int64_t n_resp, const void* tok_off,
                          double length_const, void* weight, int32_t* dev_status, hipStream_t stream) {
    const long long blocks = (n_groups * kWeightLanes + kThreads - 1) / kThreads;
    if (blocks > INT_MAX) return HORA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_response_weights<F, IG, IT>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                       (long long)n_groups, (const IG*)group_off, (long long)n_resp, (const IT*)tok_off,
                       length_const, (F*)weight, dev_status);
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

}  // namespace hora

using namespace hora;

extern "C" int hora_group_advantage(int64_t n_groups, const void* group_off, int32_t off_t, int64_t n_resp,
                                    const void* reward, void* adv, int32_t ft, int32_t mode, double eps,
                                    int32_t ddof, int32_t* dev_status, void* stream) {
    if (n_groups < 0 || n_resp < 0 || !dev_status) return HORA_ERR_INVALID_ARG;
    if (off_t != HORA_I32 && off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (ft != HORA_F32 && ft != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (mode != HORA_ADV_GRPO && mode != HORA_ADV_RLOO && mode != HORA_ADV_CENTER) return HORA_ERR_INVALID_ARG;
    if (!(eps >= 0.0) || (ddof != 0 && ddof != 1)) return HORA_ERR_INVALID_ARG;
    if (n_groups == 0) return n_resp == 0 ? HORA_OK : HORA_ERR_INVALID_ARG;
    if (!group_off) return HORA_ERR_INVALID_ARG;
    if (n_resp > 0 && (!reward || !adv)) return HORA_ERR_INVALID_ARG;
    if (off_t == HORA_I32 && n_resp >= (1ll << 31)) return HORA_ERR_INVALID_ARG;
    const uintptr_t fmask = ft == HORA_F32 ? 3 : 7, imask = off_t == HORA_I32 ? 3 : 7;
    if ((reinterpret_cast<uintptr_t>(reward) & fmask) || (reinterpret_cast<uintptr_t>(adv) & fmask) ||
        (reinterpret_cast<uintptr_t>(group_off) & imask))
        return HORA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (ft == HORA_F32) {
        if (off_t == HORA_I32)
            return launch_adv<float, int32_t>(n_groups, group_off, n_resp, reward, adv, mode, eps, ddof, dev_status, s);
        return launch_adv<float, long long>(n_groups, group_off, n_resp, reward, adv, mode, eps, ddof, dev_status, s);
    }
    if (off_t == HORA_I32)
        return launch_adv<double, int32_t>(n_groups, group_off, n_resp, reward, adv, mode, eps, ddof, dev_status, s);
    return launch_adv<double, long long>(n_groups, group_off, n_resp, reward, adv, mode, eps, ddof, dev_status, s);
}

extern "C" int hora_response_weights(int64_t n_groups, const void* group_off, int32_t group_off_t, int64_t n_resp,
                                     const void* tok_off, int32_t tok_off_t, double length_const, void* weight,
                                     int32_t ft, int32_t* dev_status, void* stream) {
    if (n_groups < 0 || n_resp < 0 || !dev_status) return HORA_ERR_INVALID_ARG;
    if (group_off_t != HORA_I32 && group_off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (tok_off_t != HORA_I32 && tok_off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (ft != HORA_F32 && ft != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (!(length_const == length_const) || length_const == INFINITY) return HORA_ERR_INVALID_ARG;
    if (n_groups == 0) return n_resp == 0 ? HORA_OK : HORA_ERR_INVALID_ARG;
    if (!group_off) return HORA_ERR_INVALID_ARG;
    if (n_resp > 0 && (!tok_off || !weight)) return HORA_ERR_INVALID_ARG;
    if (group_off_t == HORA_I32 && n_resp >= (1ll << 31)) return HORA_ERR_INVALID_ARG;
    const uintptr_t fmask = ft == HORA_F32 ? 3 : 7, gmask = group_off_t == HORA_I32 ? 3 : 7,
                    tmask = tok_off_t == HORA_I32 ? 3 : 7;
    if ((reinterpret_cast<uintptr_t>(weight) & fmask) || (reinterpret_cast<uintptr_t>(group_off) & gmask) ||
        (reinterpret_cast<uintptr_t>(tok_off) & tmask))
        return HORA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
#define HORA_WEIGHTS(F)                                                                                          \
    (group_off_t == HORA_I32                                                                                     \
         ? (tok_off_t == HORA_I32 ? launch_weights<F, int32_t, int32_t>(n_groups, group_off, n_resp, tok_off,    \
                                                                        length_const, weight, dev_status, s)     \
                                  : launch_weights<F, int32_t, long long>(n_groups, group_off, n_resp, tok_off,  \
                                                                          length_const, weight, dev_status, s))  \
         : (tok_off_t == HORA_I32 ? launch_weights<F, long long, int32_t>(n_groups, group_off, n_resp, tok_off,  \
                                                                          length_const, weight, dev_status, s)   \
                                  : launch_weights<F, long long, long long>(n_groups, group_off, n_resp, tok_off, \
                                                                            length_const, weight, dev_status, s)))
    if (ft == HORA_F32) return HORA_WEIGHTS(float);
    return HORA_WEIGHTS(double);
#undef HORA_WEIGHTS
}
