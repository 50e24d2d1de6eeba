// Per-token advantage broadcast (Sec. 3.1: the advantage of a response is the same
// for all of its tokens).
//
// The output is cut into rows of 4 KiB (one 16-byte store per thread of a workgroup),
// aligned to 16 bytes whatever the caller's pointer is.  Work is balanced by tokens,
// not by responses, and every store is a 16-byte store to a 16-byte-aligned address
// whatever the response boundaries are.
//
// Pass 1 (k_row_desc, one thread per response): checks the packed offsets and writes one
// descriptor per row: the ends (relative to the row) of the first four responses that
// intersect the row and the advantages of the first five, already converted to the
// output type.  It runs while the memory system is idle, so that pass 2 needs neither a
// search nor a second dependent load under write load.
//
// Pass 2 (k_token_fill): a workgroup owns kRows rows; the kGroup workgroups of a
// super-tile interleave their rows (workgroup g writes rows g, g + kGroup, ...), so the
// workgroups that run at the same time write one compact window of memory.  Every
// wavefront reads the descriptors of its rows with scalar loads (issued together, one
// wait), then each lane picks the response of its vector by comparing its position with
// the four ends; a wavefront whose 1 KiB lies inside one response takes a splat path
// decided by scalar compares.  No LDS, no barrier, and no vector load in the streaming
// part: loads and stores share one memory counter on this part, and a load in the loop
// body would make every store wait for the one before it.  Rows that intersect more
// than five responses (runs of very short or empty responses) are flagged by pass 1 and
// handled afterwards by a search of the packed offsets in global memory.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"

namespace hora {

constexpr int kBcastThreads = 256;   // threads per workgroup of the fill kernel
constexpr int kRows = 2;             // rows (16-byte vectors per thread) per workgroup
constexpr int kGroupShift = 4;       // log2 of the workgroups that share a super-tile
constexpr int kGroup = 1 << kGroupShift;
constexpr int kEnds = 4;             // response ends held by a row descriptor
constexpr int kVals = kEnds + 1;     // advantages held by a row descriptor
constexpr unsigned kOverflowBit = 0x80000000u;

typedef unsigned v4u __attribute__((ext_vector_type(4)));

template <typename O> struct VecOf;
template <> struct VecOf<float> { typedef v4f type; static constexpr int n = 4; };
template <> struct VecOf<double> { typedef v2d type; static constexpr int n = 2; };

// Row descriptor, an array of 32-bit words (little endian):
//   words [0, kEnds/2)          ends[k], 16 bits each: end of the k-th response that
//                               intersects the row, as an element index relative to the
//                               row, clamped to [0, row length]; unused entries hold the
//                               row length
//   then kVals values of type O vals[k]: advantage of that response
//   then one word               first: index of the response that holds the row's first
//                               token; bit 31 is set when more than kVals responses
//                               intersect the row
// padded to a power of two (32 bytes for float, 64 for double output with kEnds = 4).
template <typename O> struct DescLayout {
    static constexpr int kValWords = (int)(sizeof(O) / 4);
    static constexpr int kValBase = kEnds / 2;
    static constexpr int kFirstWord = kValBase + kVals * kValWords;
    static constexpr int kUsed = kFirstWord + 1;
    static constexpr int kWords = kUsed <= 8 ? 8 : kUsed <= 16 ? 16 : kUsed <= 32 ? 32 : 64;
    static constexpr int kBytes = kWords * 4;
};
static_assert(kEnds % 4 == 0, "values of a double descriptor must be 8-byte aligned");
template <typename O> struct alignas(DescLayout<O>::kBytes) RowDesc { unsigned u[DescLayout<O>::kWords]; };

__device__ __forceinline__ unsigned val_word(float v, int) { return __float_as_uint(v); }
__device__ __forceinline__ unsigned val_word(double v, int half) {
    return (unsigned)(half ? __double2hiint(v) : __double2loint(v));
}

template <typename O>
__device__ __forceinline__ RowDesc<O> load_row_desc(const RowDesc<O>* __restrict__ desc, long long row) {
    RowDesc<O> x;
    const v4u* src = reinterpret_cast<const v4u*>(desc + row);
#pragma unroll
    for (int i = 0; i < DescLayout<O>::kWords / 4; ++i) {
        const v4u q = src[i];
        x.u[4 * i] = q.x; x.u[4 * i + 1] = q.y; x.u[4 * i + 2] = q.z; x.u[4 * i + 3] = q.w;
    }
    return x;
}
template <typename O>
__device__ __forceinline__ int desc_end(const RowDesc<O>& x, int k) {
    const unsigned pair = x.u[k >> 1];
    return (int)((k & 1) ? pair >> 16 : pair & 0xffffu);
}
__device__ __forceinline__ float desc_val(const RowDesc<float>& x, int k) {
    return __uint_as_float(x.u[DescLayout<float>::kValBase + k]);
}
__device__ __forceinline__ double desc_val(const RowDesc<double>& x, int k) {
    return __hiloint2double((int)x.u[DescLayout<double>::kValBase + 2 * k + 1],
                            (int)x.u[DescLayout<double>::kValBase + 2 * k]);
}
template <typename O>
__device__ __forceinline__ unsigned desc_first(const RowDesc<O>& x) { return x.u[DescLayout<O>::kFirstWord]; }

// ----------------------------------------------------------------------------------
// Pass 1.  Row r holds the elements q in [r*row_elems, (r+1)*row_elems) of the aligned
// index space q = token + skew.  The response that holds a row's first token writes the
// row's descriptor.  Also the data checks: offsets start at 0, do not decrease, and end
// at n_tokens.  Offsets are clamped to [0, n_tokens] before use, so that bad data cannot
// move any access outside the buffers.
// ----------------------------------------------------------------------------------
template <typename A, typename O, typename I>
__global__ __launch_bounds__(kThreads) void k_row_desc(long long n_resp, const A* __restrict__ adv,
                                                       const I* __restrict__ tok_off, long long n_tokens, int skew,
                                                       long long n_rows, RowDesc<O>* __restrict__ desc,
                                                       int32_t* dev_status) {
    constexpr int kRowElems = kBcastThreads * VecOf<O>::n;
    const long long stride = (long long)gridDim.x * kThreads;
    bool bad = false;
    for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < n_resp; j += stride) {
        // every load of this response up front (one round trip): its start, the ends of
        // the kVals responses from it on, and their advantages
        long long a = (long long)tok_off[j];
        long long e[kVals];
        O v[kVals];
#pragma unroll
        for (int k = 0; k < kVals; ++k) {
            e[k] = j + k < n_resp ? (long long)tok_off[j + 1 + k] : n_tokens;
            v[k] = j + k < n_resp ? (O)adv[j + k] : (O)0;
        }
        long long b = e[0];
        bad |= b < a || a < 0 || b > n_tokens;
        if (j == 0) bad |= a != 0;
        if (j == n_resp - 1) bad |= b != n_tokens;
        a = a < 0 ? 0 : (a > n_tokens ? n_tokens : a);
#pragma unroll
        for (int k = 0; k < kVals; ++k) e[k] = e[k] < 0 ? 0 : (e[k] > n_tokens ? n_tokens : e[k]);
        b = e[0];
        if (b <= a) continue;
        const long long r_min = a == 0 ? 0 : (a + skew + kRowElems - 1) / kRowElems;
        long long r_max = (b - 1 + skew) / kRowElems;
        if (r_max > n_rows - 1) r_max = n_rows - 1;
        for (long long r = r_min; r <= r_max; ++r) {
            const long long row_first = r * kRowElems - skew;   // token of the row's element 0
            RowDesc<O> d;
#pragma unroll
            for (int i = 0; i < DescLayout<O>::kWords; ++i) d.u[i] = 0u;
#pragma unroll
            for (int k = 0; k < kEnds; ++k) {
                long long rel = e[k] - row_first;
                rel = rel < 0 ? 0 : (rel > kRowElems ? kRowElems : rel);
                d.u[k >> 1] |= (unsigned)rel << (16 * (k & 1));
            }
#pragma unroll
            for (int k = 0; k < kVals; ++k)
#pragma unroll
                for (int h = 0; h < DescLayout<O>::kValWords; ++h)
                    d.u[DescLayout<O>::kValBase + k * DescLayout<O>::kValWords + h] = val_word(v[k], h);
            long long row_end = row_first + kRowElems;
            if (row_end > n_tokens) row_end = n_tokens;
            d.u[DescLayout<O>::kFirstWord] = (unsigned)j | (e[kVals - 1] < row_end ? kOverflowBit : 0u);
            v4u* dst = reinterpret_cast<v4u*>(desc + r);
#pragma unroll
            for (int i = 0; i < DescLayout<O>::kWords / 4; ++i) {
                v4u q = {d.u[4 * i], d.u[4 * i + 1], d.u[4 * i + 2], d.u[4 * i + 3]};
                dst[i] = q;
            }
        }
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

// ----------------------------------------------------------------------------------
// Pass 2.
// ----------------------------------------------------------------------------------
// Stores one thread's vector of a row: whole where every element is a token, element by
// element in the first and the last row of the output.
template <typename O>
__device__ __forceinline__ void store_vec(O* __restrict__ out, long long row, long long n_rows, long long row_first,
                                          long long n_tokens, int r0, const O (&vals)[VecOf<O>::n]) {
    typedef typename VecOf<O>::type Vec;
    constexpr int kVec = VecOf<O>::n;
    constexpr int kRowElems = kBcastThreads * kVec;
    O* dst = out + (row_first + r0);
    if (row > 0 && row < n_rows - 1) {
        Vec v;
#pragma unroll
        for (int i = 0; i < kVec; ++i) v[i] = vals[i];
        *reinterpret_cast<Vec*>(dst) = v;
    } else {
        // elements of the row that are tokens: [rel_lo, rel_hi)
        const int rel_lo = row_first < 0 ? (int)(-row_first) : 0;
        const int rel_hi = n_tokens - row_first < kRowElems ? (int)(n_tokens - row_first) : kRowElems;
#pragma unroll
        for (int i = 0; i < kVec; ++i)
            if (r0 + i >= rel_lo && r0 + i < rel_hi) dst[i] = vals[i];
    }
}

template <typename O>
__device__ __forceinline__ void fill_row(const RowDesc<O>& d, O* __restrict__ out, long long row, long long n_rows,
                                         long long n_tokens, int skew) {
    constexpr int kVec = VecOf<O>::n;
    constexpr int kRowElems = kBcastThreads * kVec;
    constexpr int kWaveElems = kWave * kVec;
    const long long row_first = row * kRowElems - skew;
    const int r0 = (int)threadIdx.x * kVec;
    int e[kEnds];
    O v[kVals];
#pragma unroll
    for (int k = 0; k < kEnds; ++k) e[k] = desc_end(d, k);
#pragma unroll
    for (int k = 0; k < kVals; ++k) v[k] = desc_val(d, k);
    // the wavefront's elements [w0, w1) of the row: when the first and the last of them
    // belong to the same response, all of them do
    const int w0 = __builtin_amdgcn_readfirstlane(r0) & ~(kWaveElems - 1);
    const int w1 = w0 + kWaveElems;
    int s_first = 0, s_last = 0;
#pragma unroll
    for (int k = 0; k < kEnds; ++k) {
        s_first += (int)(e[k] <= w0);
        s_last += (int)(e[k] < w1);
    }
    O vals[kVec];
    if (s_first == s_last) {
        O x = v[0];
#pragma unroll
        for (int k = 1; k < kVals; ++k) x = s_first >= k ? v[k] : x;
#pragma unroll
        for (int i = 0; i < kVec; ++i) vals[i] = x;
    } else {
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
            const int p = r0 + i;
            O x = v[0];
#pragma unroll
            for (int k = 0; k < kEnds; ++k) x = p >= e[k] ? v[k + 1] : x;
            vals[i] = x;
        }
    }
    store_vec<O>(out, row, n_rows, row_first, n_tokens, r0, vals);
}

// A row that more than kVals responses intersect: every lane searches the packed offsets
// for the response of its first element, starting from the response of the row's first
// token.  Kept out of line: its loads must not sit between the stores of the fast rows.
template <typename A, typename O, typename I>
__device__ __noinline__ void fill_row_by_search(unsigned first, long long n_resp, const A* __restrict__ adv,
                                                const I* __restrict__ tok_off, O* __restrict__ out, long long row,
                                                long long n_rows, long long n_tokens, int skew) {
    constexpr int kVec = VecOf<O>::n;
    constexpr int kRowElems = kBcastThreads * kVec;
    const long long row_first = row * kRowElems - skew;
    const int r0 = (int)threadIdx.x * kVec;
    const long long last = n_resp - 1;
    long long a = (long long)(first & ~kOverflowBit);
    a = a > last ? last : a;
    long long b = last;
    const long long p = row_first + r0;
    while (a < b) {   // first response in [a, b] whose end lies beyond p
        const long long mid = (a + b) >> 1;
        if ((long long)tok_off[mid + 1] > p) b = mid; else a = mid + 1;
    }
    O vals[kVec];
#pragma unroll
    for (int i = 0; i < kVec; ++i) {
        while (a < last && (long long)tok_off[a + 1] <= p + i) ++a;
        vals[i] = (O)adv[a];
    }
    store_vec<O>(out, row, n_rows, row_first, n_tokens, r0, vals);
}

template <typename A, typename O, typename I>
__global__ __launch_bounds__(kBcastThreads) void k_token_fill(long long n_resp, const A* __restrict__ adv,
                                                              const I* __restrict__ tok_off, O* __restrict__ out,
                                                              long long n_tokens, int skew, long long n_rows,
                                                              const RowDesc<O>* __restrict__ desc) {
    const long long super = blockIdx.x >> kGroupShift;
    const long long member = blockIdx.x & (kGroup - 1);
    const long long row0 = ((super * kRows) << kGroupShift) + member;   // row k of this workgroup = row0 + k * kGroup
    RowDesc<O> d[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) {   // all descriptor loads first: one wait for the lot
        const long long row = row0 + ((long long)k << kGroupShift);
        d[k] = load_row_desc<O>(desc, row < n_rows ? row : n_rows - 1);
    }
    bool any_search = false;
#pragma unroll
    for (int k = 0; k < kRows; ++k) {
        const long long row = row0 + ((long long)k << kGroupShift);
        if (row < n_rows) {
            if (desc_first(d[k]) & kOverflowBit) any_search = true;
            else fill_row<O>(d[k], out, row, n_rows, n_tokens, skew);
        }
    }
    if (any_search) {
        for (int k = 0; k < kRows; ++k) {
            const long long row = row0 + ((long long)k << kGroupShift);
            if (row < n_rows && (desc_first(d[k]) & kOverflowBit))
                fill_row_by_search<A, O, I>(desc_first(d[k]), n_resp, adv, tok_off, out, row, n_rows, n_tokens, skew);
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
    const int skew = (int)((reinterpret_cast<uintptr_t>(out) & 15) / sizeof(O));
    const long long n_rows = rows_for<O>(n_tokens, skew);
    if ((size_t)(n_rows + 1) * sizeof(RowDesc<O>) > workspace_bytes) return HORA_ERR_WORKSPACE;
    RowDesc<O>* desc = (RowDesc<O>*)workspace;
    long long blocks1 = (n_resp + kThreads - 1) / kThreads;
    if (blocks1 > 65536) blocks1 = 65536;
    hipLaunchKernelGGL((k_row_desc<A, O, I>), dim3((unsigned)blocks1), dim3(kThreads), 0, stream,
                       (long long)n_resp, (const A*)adv, (const I*)tok_off, (long long)n_tokens, skew, n_rows, desc,
                       dev_status);
    if (n_rows > 0) {
        const long long supers = (n_rows + kGroup * kRows - 1) / (kGroup * kRows);
        if (supers * kGroup > INT_MAX) return HORA_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((k_token_fill<A, O, I>), dim3((unsigned)(supers * kGroup)), dim3(kBcastThreads), 0,
                           stream, (long long)n_resp, (const A*)adv, (const I*)tok_off, (O*)out,
                           (long long)n_tokens, skew, n_rows, desc);
    }
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

}  // namespace hora

using namespace hora;

extern "C" size_t hora_token_broadcast_workspace_bytes(int64_t n_tokens, int32_t out_t) {
    if (n_tokens < 0 || (out_t != HORA_F32 && out_t != HORA_F64)) return 0;
    const size_t bytes = out_t == HORA_F32 ? (size_t)(rows_for<float>(n_tokens, 3) + 1) * sizeof(RowDesc<float>)
                                           : (size_t)(rows_for<double>(n_tokens, 1) + 1) * sizeof(RowDesc<double>);
    return (bytes + 255) & ~(size_t)255;
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
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 63)) return HORA_ERR_WORKSPACE;
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
