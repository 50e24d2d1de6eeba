// Per-token advantage broadcast (Sec. 3.1: the advantage of a response is the same
// for all of its tokens).
//
// The output is cut into rows of 4 KiB (one 16-byte store per thread of a workgroup),
// aligned to 16 bytes whatever the caller's pointer is.  Work is balanced by tokens,
// not by responses, and every store is a 16-byte store to a 16-byte-aligned address
// whatever the response boundaries are.
//
// Pass 1 (k_row_index, one thread per response): checks the packed offsets and writes,
// for every row, the index of the response that holds the row's first token.  It runs
// while the memory system is idle, so that pass 2 needs no search under write load.
//
// Pass 2 (k_token_fill): the kGroup workgroups of a super-tile (kGroup * kRows rows,
// 1 MiB) interleave their rows (workgroup g writes rows g, g + kGroup, ...), so the
// workgroups that run at the same time write one compact window of memory: on this part
// that sustains clearly more HBM write bandwidth than giving every workgroup its own
// contiguous 64 KiB.  A workgroup reads the row index of its rows, stages the ends and
// advantages of the few responses that intersect them in LDS (two dependent loads in
// all), and each lane finds the response of its vector by a short binary search in LDS.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"

namespace hora {

constexpr int kBcastThreads = 256;   // threads per workgroup of the fill kernel
constexpr int kRows = 16;            // rows (16-byte vectors per thread) per workgroup and super-tile
constexpr int kGroup = 16;           // workgroups that share a super-tile
constexpr int kSegCap = 2048;        // response ends staged in LDS per workgroup

template <typename O> struct VecOf;
template <> struct VecOf<float> { typedef v4f type; static constexpr int n = 4; };
template <> struct VecOf<double> { typedef v2d type; static constexpr int n = 2; };

// ----------------------------------------------------------------------------------
// Pass 1.  Row r holds the elements q in [r*row_elems, (r+1)*row_elems) of the aligned
// index space q = token + skew.  row_seg[r] = response of the first token of row r;
// row_seg[n_rows] = n_resp - 1.  Also the data checks: offsets start at 0, do not
// decrease, and end at n_tokens.
// ----------------------------------------------------------------------------------
template <typename I>
__global__ __launch_bounds__(kThreads) void k_row_index(long long n_resp, const I* __restrict__ tok_off,
                                                        long long n_tokens, int skew, int row_elems,
                                                        long long n_rows, int32_t* __restrict__ row_seg,
                                                        int32_t* dev_status) {
    const long long stride = (long long)gridDim.x * kThreads;
    bool bad = false;
    for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < n_resp; j += stride) {
        long long a = (long long)tok_off[j], b = (long long)tok_off[j + 1];
        bad |= b < a || a < 0 || b > n_tokens;
        if (j == 0) bad |= a != 0;
        if (j == n_resp - 1) {
            bad |= b != n_tokens;
            row_seg[n_rows] = (int32_t)j;
        }
        a = a < 0 ? 0 : (a > n_tokens ? n_tokens : a);
        b = b < 0 ? 0 : (b > n_tokens ? n_tokens : b);
        if (b <= a) continue;
        long long r_min = a == 0 ? 0 : (a + skew + row_elems - 1) / row_elems;
        long long r_max = (b - 1 + skew) / row_elems;
        if (r_max > n_rows - 1) r_max = n_rows - 1;
        for (long long r = r_min; r <= r_max; ++r) row_seg[r] = (int32_t)j;
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

// first staged entry in [a, b] whose end lies beyond position r (ends are non-decreasing)
__device__ __forceinline__ int first_end_beyond(const int* s_end, int a, int b, int r) {
    while (a < b) {
        const int mid = (a + b) >> 1;
        if (s_end[mid] > r) b = mid; else a = mid + 1;
    }
    return a;
}

// ----------------------------------------------------------------------------------
// Pass 2.
// ----------------------------------------------------------------------------------
template <typename A, typename O, typename I>
__global__ __launch_bounds__(kBcastThreads) void k_token_fill(long long n_resp, const A* __restrict__ adv,
                                                              const I* __restrict__ tok_off, O* __restrict__ out,
                                                              long long n_tokens, int skew, long long n_rows,
                                                              const int32_t* __restrict__ row_seg) {
    typedef typename VecOf<O>::type Vec;
    constexpr int kVec = VecOf<O>::n;
    constexpr int kRowElems = kBcastThreads * kVec;                  // 4 KiB
    __shared__ int s_end[kSegCap];     // staged response ends, relative to the start of their row
    __shared__ O s_val[kSegCap];       // staged advantages
    __shared__ int s_lo[kRows];        // first response of row k
    __shared__ int s_cnt[kRows];       // responses that may intersect row k (0: the row does not exist)
    __shared__ int s_base[kRows + 1];  // where row k's entries start in the staging arrays

    const long long super = blockIdx.x / kGroup;
    const int member = (int)(blockIdx.x % kGroup);
    const long long row0 = super * (long long)(kGroup * kRows) + member;   // row of k = 0; row k = row0 + k * kGroup
    if (row0 >= n_rows) return;

    // responses of this workgroup's rows: row_seg[row] .. row_seg[row + 1]
    if (threadIdx.x < kRows) {
        const int k = (int)threadIdx.x;
        const long long row = row0 + (long long)k * kGroup;
        int lo = 0, cnt = 0;
        if (row < n_rows) {
            lo = row_seg[row];
            int hi = row_seg[row + 1];
            const int last = (int)(n_resp - 1);
            lo = lo < 0 ? 0 : (lo > last ? last : lo);
            hi = hi < lo ? lo : (hi > last ? last : hi);
            cnt = hi - lo + 1;
        }
        s_lo[k] = lo;
        s_cnt[k] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
#pragma unroll
        for (int k = 0; k < kRows; ++k) { s_base[k] = acc; acc += s_cnt[k]; }
        s_base[kRows] = acc;
    }
    __syncthreads();
    const int total = s_base[kRows];
    const bool staged = total <= kSegCap;
    if (staged) {
        for (int e = (int)threadIdx.x; e < total; e += kBcastThreads) {
            int k = 0;
#pragma unroll
            for (int step = kRows / 2; step > 0; step >>= 1)
                if (s_base[k + step] <= e) k += step;          // row of entry e
            const long long j = (long long)s_lo[k] + (e - s_base[k]);
            const long long row_first = (row0 + (long long)k * kGroup) * kRowElems - skew;   // token of element 0
            long long rel = (long long)tok_off[j + 1] - row_first;
            rel = rel < 0 ? 0 : (rel > kRowElems ? kRowElems : rel);
            s_end[e] = (int)rel;
            s_val[e] = (O)adv[j];
        }
        __syncthreads();
    }

#pragma unroll 4
    for (int k = 0; k < kRows; ++k) {
        const int cnt = s_cnt[k];
        if (cnt == 0) continue;
        const long long row_first = (row0 + (long long)k * kGroup) * kRowElems - skew;
        const int r0 = (int)threadIdx.x * kVec;
        // elements of the row that are tokens: [rel_lo, rel_hi)
        const int rel_lo = row_first < 0 ? (int)(-row_first) : 0;
        const int rel_hi = n_tokens - row_first < kRowElems ? (int)(n_tokens - row_first) : kRowElems;
        O* dst = out + (row_first + r0);
        O vals[kVec];
        if (staged) {
            const int base = s_base[k];
            if (cnt == 1) {
                const O v1 = s_val[base];
#pragma unroll
                for (int i = 0; i < kVec; ++i) vals[i] = v1;
            } else {
                const int last = base + cnt - 1;
                int a = first_end_beyond(s_end, base, last, r0);
                if (s_end[a] >= r0 + kVec) {
                    const O v1 = s_val[a];
#pragma unroll
                    for (int i = 0; i < kVec; ++i) vals[i] = v1;
                } else {
#pragma unroll
                    for (int i = 0; i < kVec; ++i) {
                        while (a < last && s_end[a] <= r0 + i) ++a;
                        vals[i] = s_val[a];
                    }
                }
            }
        } else {
            // too many responses for the staging arrays (runs of very short or empty
            // responses): search the packed offsets in global memory instead
            long long a = s_lo[k], b = a + cnt - 1;
            const long long p = row_first + r0;
            while (a < b) {   // first response in [a, b] whose end lies beyond p
                const long long mid = (a + b) >> 1;
                if ((long long)tok_off[mid + 1] > p) b = mid; else a = mid + 1;
            }
            const long long last = (long long)s_lo[k] + cnt - 1;
#pragma unroll
            for (int i = 0; i < kVec; ++i) {
                while (a < last && (long long)tok_off[a + 1] <= p + i) ++a;
                vals[i] = (O)adv[a];
            }
        }
        if (r0 >= rel_lo && r0 + kVec <= rel_hi) {
            Vec v;
#pragma unroll
            for (int i = 0; i < kVec; ++i) v[i] = vals[i];
            *reinterpret_cast<Vec*>(dst) = v;
        } else {
#pragma unroll
            for (int i = 0; i < kVec; ++i)
                if (r0 + i >= rel_lo && r0 + i < rel_hi) dst[i] = vals[i];
        }
    }
}

template <typename O>
static long long rows_for(int64_t n_tokens, int skew) {
    const long long row_elems = (long long)kBcastThreads * VecOf<O>::n;
    return (n_tokens + skew + row_elems - 1) / row_elems;
}

template <typename A, typename O, typename I>
static int launch_broadcast(int64_t n_resp, const void* adv, const void* tok_off, void* out, int64_t n_tokens,
                            int32_t* dev_status, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    const int row_elems = kBcastThreads * VecOf<O>::n;
    const int skew = (int)((reinterpret_cast<uintptr_t>(out) & 15) / sizeof(O));
    const long long n_rows = rows_for<O>(n_tokens, skew);
    if ((size_t)(n_rows + 1) * sizeof(int32_t) > workspace_bytes) return HORA_ERR_WORKSPACE;
    int32_t* row_seg = (int32_t*)workspace;
    long long blocks1 = (n_resp + kThreads - 1) / kThreads;
    if (blocks1 > 65536) blocks1 = 65536;
    hipLaunchKernelGGL((k_row_index<I>), dim3((unsigned)blocks1), dim3(kThreads), 0, stream, (long long)n_resp,
                       (const I*)tok_off, (long long)n_tokens, skew, row_elems, n_rows, row_seg, dev_status);
    if (n_rows > 0) {
        const long long supers = (n_rows + kGroup * kRows - 1) / (kGroup * kRows);
        if (supers * kGroup > INT_MAX) return HORA_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((k_token_fill<A, O, I>), dim3((unsigned)(supers * kGroup)), dim3(kBcastThreads), 0,
                           stream, (long long)n_resp, (const A*)adv, (const I*)tok_off, (O*)out,
                           (long long)n_tokens, skew, n_rows, row_seg);
    }
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

}  // namespace hora

using namespace hora;

extern "C" size_t hora_token_broadcast_workspace_bytes(int64_t n_tokens, int32_t out_t) {
    if (n_tokens < 0 || (out_t != HORA_F32 && out_t != HORA_F64)) return 0;
    const long long n_rows = out_t == HORA_F32 ? rows_for<float>(n_tokens, 3) : rows_for<double>(n_tokens, 1);
    return (((size_t)(n_rows + 1) * sizeof(int32_t)) + 255) & ~(size_t)255;
}

extern "C" int hora_token_broadcast(int64_t n_resp, const void* adv, int32_t adv_t, const void* tok_off,
                                    int32_t off_t, void* tok_adv, int32_t out_t, int64_t n_tokens,
                                    int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream) {
    if (n_resp < 0 || n_tokens < 0 || !dev_status) return HORA_ERR_INVALID_ARG;
    if (adv_t != HORA_F32 && adv_t != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (out_t != HORA_F32 && out_t != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (off_t != HORA_I32 && off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (adv_t == HORA_F32 && out_t == HORA_F64) return HORA_ERR_INVALID_ARG;  // never widen
    if (n_resp == 0) return n_tokens == 0 ? HORA_OK : HORA_ERR_INVALID_ARG;
    if (n_resp >= (1ll << 31)) return HORA_ERR_UNSUPPORTED;
    if (!adv || !tok_off) return HORA_ERR_INVALID_ARG;
    if (n_tokens > 0 && !tok_adv) return HORA_ERR_INVALID_ARG;
    if (off_t == HORA_I32 && n_tokens >= (1ll << 31)) return HORA_ERR_INVALID_ARG;
    const uintptr_t amask = adv_t == HORA_F32 ? 3 : 7, omask = out_t == HORA_F32 ? 3 : 7,
                    imask = off_t == HORA_I32 ? 3 : 7;
    if ((reinterpret_cast<uintptr_t>(adv) & amask) || (reinterpret_cast<uintptr_t>(tok_adv) & omask) ||
        (reinterpret_cast<uintptr_t>(tok_off) & imask))
        return HORA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 3)) return HORA_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
#define HORA_BCAST(A, O)                                                                                      \
    (off_t == HORA_I32 ? launch_broadcast<A, O, int32_t>(n_resp, adv, tok_off, tok_adv, n_tokens, dev_status, \
                                                         workspace, workspace_bytes, s)                       \
                       : launch_broadcast<A, O, long long>(n_resp, adv, tok_off, tok_adv, n_tokens,           \
                                                           dev_status, workspace, workspace_bytes, s))
    if (adv_t == HORA_F32) return HORA_BCAST(float, float);
    if (out_t == HORA_F32) return HORA_BCAST(double, float);
    return HORA_BCAST(double, double);
#undef HORA_BCAST
}
