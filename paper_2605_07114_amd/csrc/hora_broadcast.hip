// Per-token advantage broadcast (Sec. 3.1: the advantage of a response is the same
// for all of its tokens).
//
// The output is cut into rows of 4 KiB (one 16-byte store per thread of a workgroup)
// and into super-tiles of kGroup * kRows rows (1 MiB).  The kGroup workgroups of a
// super-tile interleave their rows (workgroup g writes rows g, g + kGroup, ...), so
// the workgroups that run at the same time write one compact window of memory: on this
// part that sustains clearly more HBM write bandwidth than giving every workgroup its
// own contiguous 64 KiB.  Work is balanced by tokens, not by responses, and every store
// is a 16-byte store to a 16-byte-aligned address whatever the response boundaries are.
//
// Per workgroup: a 256-ary search over the packed offsets finds the response that holds
// the super-tile's first token; the ends and advantages of the responses that intersect
// the super-tile are staged in LDS; 2 * kRows threads bracket the staged responses of
// each of the workgroup's rows; each lane then finds the response of its vector by a
// short binary search inside its row's bracket.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"

namespace hora {

constexpr int kRows = 16;        // rows (16-byte vectors per thread) per workgroup and super-tile
constexpr int kGroup = 16;       // workgroups that share a super-tile
constexpr int kSegCap = 2048;    // response ends staged in LDS per gather round

template <typename O> struct VecOf;
template <> struct VecOf<float> { typedef v4f type; static constexpr int n = 4; };
template <> struct VecOf<double> { typedef v2d type; static constexpr int n = 2; };

// first staged response in [a, b] whose end lies beyond position r (ends are non-decreasing)
__device__ __forceinline__ int first_end_beyond(const int* s_end, int a, int b, int r) {
    while (a < b) {
        const int mid = (a + b) >> 1;
        if (s_end[mid] > r) b = mid; else a = mid + 1;
    }
    return a;
}

template <typename A, typename O, typename I>
__global__ __launch_bounds__(kThreads) void k_token_broadcast(long long n_resp, const A* __restrict__ adv,
                                                              const I* __restrict__ tok_off, O* __restrict__ out,
                                                              long long n_tokens, int skew, int32_t* dev_status) {
    typedef typename VecOf<O>::type Vec;
    constexpr int kVec = VecOf<O>::n;
    constexpr int kRowElems = kThreads * kVec;                  // 4 KiB
    constexpr int kSuperElems = kRowElems * kRows * kGroup;     // 1 MiB
    __shared__ int s_end[kSegCap];
    __shared__ O s_val[kSegCap];
    __shared__ int s_row_lo[kRows], s_row_hi[kRows];

    // packed offsets must start at 0, not decrease, and end at n_tokens
    {
        const long long stride = (long long)gridDim.x * kThreads;
        bool bad = false;
        for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < n_resp; j += stride) {
            const long long a = (long long)tok_off[j], b = (long long)tok_off[j + 1];
            bad |= b < a;
            if (j == 0) bad |= a != 0;
            if (j == n_resp - 1) bad |= b != n_tokens;
        }
        if (bad) report(dev_status, HORA_ERR_RANGE);
    }

    // super-tile in token coordinates; p0 may be negative in the first one of a skewed buffer
    const long long super = blockIdx.x / kGroup;
    const int member = (int)(blockIdx.x % kGroup);
    const long long p0 = super * kSuperElems - skew;
    const long long p_lo = p0 < 0 ? 0 : p0;
    const long long p_hi = p0 + kSuperElems < n_tokens ? p0 + kSuperElems : n_tokens;
    if (p_lo >= p_hi) return;
    if (p0 + (long long)member * kRowElems >= p_hi) return;   // none of this workgroup's rows exists

    // response holding token p_lo: the largest j with tok_off[j] <= p_lo
    long long lo = 0, hi = n_resp;
    while (hi - lo > 1) {
        const long long width = hi - lo;
        const long long sample = lo + 1 + ((width - 1) * (long long)threadIdx.x) / kThreads;
        const bool below = (long long)tok_off[sample] <= p_lo;
        const int cnt = __syncthreads_count(below ? 1 : 0);
        const long long new_lo = cnt > 0 ? lo + 1 + ((width - 1) * (long long)(cnt - 1)) / kThreads : lo;
        const long long new_hi = cnt < kThreads ? lo + 1 + ((width - 1) * (long long)cnt) / kThreads : hi;
        lo = new_lo;
        hi = new_hi;
    }
    long long seg = lo;      // first response not yet fully written
    long long cur = p_lo;    // first token not yet written

    while (cur < p_hi) {
        // stage the ends (relative to p0) and advantages of the next responses
        int nseg = 0;
        bool last_found = false;
        for (int base = 0; base < kSegCap && !last_found; base += kThreads) {
            const long long idx = seg + base + threadIdx.x;
            long long e = idx < n_resp ? (long long)tok_off[idx + 1] : LLONG_MAX;
            const bool inside = e < p_hi;   // this response ends inside the super-tile: more follow
            e = e < cur ? cur : (e > p_hi ? p_hi : e);
            s_end[base + threadIdx.x] = (int)(e - p0);
            s_val[base + threadIdx.x] = idx < n_resp ? (O)adv[idx] : (O)0;
            const int cnt = __syncthreads_count(inside ? 1 : 0);
            if (cnt < kThreads) {
                nseg = base + cnt + 1;
                last_found = true;
            } else {
                nseg = base + kThreads;
            }
        }
        const long long cover = last_found ? p_hi : p0 + s_end[nseg - 1];
        const int lo_rel = (int)(cur - p0);
        const int hi_rel = (int)((cover > cur ? cover : cur) - p0);

        // bracket of staged responses for each of this workgroup's rows
        if (threadIdx.x < 2 * kRows) {
            const int k = (int)threadIdx.x >> 1;
            const int row_first = (member + k * kGroup) * kRowElems;
            if (threadIdx.x & 1) s_row_hi[k] = first_end_beyond(s_end, 0, nseg - 1, row_first + kRowElems - 1);
            else s_row_lo[k] = first_end_beyond(s_end, 0, nseg - 1, row_first);
        }
        __syncthreads();

        if (hi_rel > lo_rel) {
#pragma unroll 4
            for (int k = 0; k < kRows; ++k) {
                const int r0 = (member + k * kGroup) * kRowElems + (int)threadIdx.x * kVec;
                if (r0 + kVec <= lo_rel || r0 >= hi_rel) continue;
                int a = first_end_beyond(s_end, s_row_lo[k], s_row_hi[k], r0);
                O vals[kVec];
                if (s_end[a] >= r0 + kVec) {
                    const O v = s_val[a];
#pragma unroll
                    for (int i = 0; i < kVec; ++i) vals[i] = v;
                } else {
#pragma unroll
                    for (int i = 0; i < kVec; ++i) {
                        while (a < nseg - 1 && s_end[a] <= r0 + i) ++a;
                        vals[i] = s_val[a];
                    }
                }
                O* dst = out + (p0 + r0);
                if (r0 >= lo_rel && r0 + kVec <= hi_rel) {
                    Vec v;
#pragma unroll
                    for (int i = 0; i < kVec; ++i) v[i] = vals[i];
                    *reinterpret_cast<Vec*>(dst) = v;
                } else {
#pragma unroll
                    for (int i = 0; i < kVec; ++i)
                        if (r0 + i >= lo_rel && r0 + i < hi_rel) dst[i] = vals[i];
                }
            }
        }
        __syncthreads();   // LDS is rewritten by the next round
        if (last_found) break;
        cur = cover > cur ? cover : cur;
        seg += nseg;
    }
}

template <typename A, typename O, typename I>
static int launch_broadcast(int64_t n_resp, const void* adv, const void* tok_off, void* out, int64_t n_tokens,
                            int32_t* dev_status, hipStream_t stream) {
    constexpr int kVec = VecOf<O>::n;
    constexpr long long kSuperElems = (long long)kThreads * kVec * kRows * kGroup;
    const int skew = (int)((reinterpret_cast<uintptr_t>(out) & 15) / sizeof(O));
    long long supers = (n_tokens + skew + kSuperElems - 1) / kSuperElems;
    if (supers < 1) supers = 1;
    if (supers * kGroup > INT_MAX) return HORA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_token_broadcast<A, O, I>), dim3((unsigned)(supers * kGroup)), dim3(kThreads), 0, stream,
                       (long long)n_resp, (const A*)adv, (const I*)tok_off, (O*)out, (long long)n_tokens, skew,
                       dev_status);
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

}  // namespace hora

using namespace hora;

extern "C" int hora_token_broadcast(int64_t n_resp, const void* adv, int32_t adv_t, const void* tok_off,
                                    int32_t off_t, void* tok_adv, int32_t out_t, int64_t n_tokens,
                                    int32_t* dev_status, void* stream) {
    if (n_resp < 0 || n_tokens < 0 || !dev_status) return HORA_ERR_INVALID_ARG;
    if (adv_t != HORA_F32 && adv_t != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (out_t != HORA_F32 && out_t != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (off_t != HORA_I32 && off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (adv_t == HORA_F32 && out_t == HORA_F64) return HORA_ERR_INVALID_ARG;  // never widen
    if (n_resp == 0) return n_tokens == 0 ? HORA_OK : HORA_ERR_INVALID_ARG;
    if (!adv || !tok_off) return HORA_ERR_INVALID_ARG;
    if (n_tokens > 0 && !tok_adv) return HORA_ERR_INVALID_ARG;
    if (off_t == HORA_I32 && n_tokens >= (1ll << 31)) return HORA_ERR_INVALID_ARG;
    const uintptr_t amask = adv_t == HORA_F32 ? 3 : 7, omask = out_t == HORA_F32 ? 3 : 7,
                    imask = off_t == HORA_I32 ? 3 : 7;
    if ((reinterpret_cast<uintptr_t>(adv) & amask) || (reinterpret_cast<uintptr_t>(tok_adv) & omask) ||
        (reinterpret_cast<uintptr_t>(tok_off) & imask))
        return HORA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
#define HORA_BCAST(A, O)                                                                                       \
    (off_t == HORA_I32 ? launch_broadcast<A, O, int32_t>(n_resp, adv, tok_off, tok_adv, n_tokens, dev_status, s) \
                       : launch_broadcast<A, O, long long>(n_resp, adv, tok_off, tok_adv, n_tokens, dev_status, s))
    if (adv_t == HORA_F32) return HORA_BCAST(float, float);
    if (out_t == HORA_F32) return HORA_BCAST(double, float);
    return HORA_BCAST(double, double);
#undef HORA_BCAST
}
