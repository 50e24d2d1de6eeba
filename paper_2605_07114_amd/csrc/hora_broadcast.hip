// Per-token advantage broadcast (Sec. 3.1: the advantage of a response is the same
// for all of its tokens).
//
// The output is cut into rows of 8 KiB, aligned to 16 bytes whatever the caller's pointer
// is; a workgroup writes one row, every lane 32 consecutive bytes as two 16-byte stores.
// Work is balanced by tokens, not by responses, and every store is a 16-byte store to a
// 16-byte-aligned address whatever the response boundaries are.
//
// Pass 1 (k_row_desc, one thread per response): checks the packed offsets and writes one
// short descriptor per row: the ends (relative to the row) of the first four responses
// that intersect the row and the advantages of the first five, already converted to the
// output type.  A row that more responses intersect gets a flag there and a wide
// descriptor (eight ends, nine advantages) in a second array.  It runs while the memory
// system is idle, so that pass 2 needs neither a search nor, for most rows, a second
// dependent load under write load.
//
// Pass 2 (k_token_fill): every wavefront reads the short descriptor of its row with one
// scalar load, then each lane picks the response of each of its elements by comparing
// its position with the ends; a wavefront whose 2 KiB lie inside one response takes a
// splat path decided by scalar compares.  No LDS, no barrier, and no vector load in the
// streaming part: loads and stores share one memory counter on this part, and a load
// between the stores would make every store wait for the one before it.  What limits the
// kernel besides the stores is the number of cache lines of descriptors fetched under
// write load, so the short descriptors of workgroups that run on the same die (workgroup
// index modulo 8) share cache lines.  Flagged rows take a slower path: through the wide
// descriptor, or, when more than nine responses intersect the row (runs of very short or
// empty responses), by a search of the packed offsets.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"

namespace hora {

constexpr int kBcastThreads = 256;   // threads per workgroup of the fill kernel
constexpr int kLaneVecs = 2;         // consecutive 16-byte vectors a lane stores
constexpr int kEnds = 8;             // response ends held by a wide row descriptor
constexpr int kVals = kEnds + 1;     // advantages held by a wide row descriptor
constexpr int kShortEnds = 4;        // the same for a short descriptor
constexpr int kShortVals = kShortEnds + 1;
constexpr int kDies = 8;             // workgroup w runs on die w % kDies
constexpr int kDieBlock = 64;        // workgroups whose short descriptors are regrouped by die
constexpr unsigned kOverflowBit = 0x80000000u;

typedef unsigned v4u __attribute__((ext_vector_type(4)));

template <typename O> struct VecOf;
template <> struct VecOf<float> { typedef v4f type; static constexpr int n = 4; };
template <> struct VecOf<double> { typedef v2d type; static constexpr int n = 2; };

template <typename O> struct RowOf {
    static constexpr int kLaneElems = kLaneVecs * VecOf<O>::n;        // elements a lane writes
    static constexpr int kWaveElems = kWave * kLaneElems;             // elements a wavefront writes
    static constexpr int kRowElems = kBcastThreads * kLaneElems;      // elements of a row
};
static_assert(RowOf<float>::kRowElems < (1 << 15), "an end and the flag share 16 bits");

// Row descriptor with E ends, an array of 32-bit words (little endian):
//   words [0, E/2)              ends[k], 16 bits each: end of the k-th response that
//                               intersects the row, as an element index relative to the
//                               row, clamped to [0, row length]; unused entries hold the
//                               row length
//   then E+1 values of type O   vals[k]: advantage of that response
//   wide descriptors (E = kEnds) then hold one word `first`: index of the response that
//   holds the row's first token, bit 31 set when more than E+1 responses intersect the
//   row; short ones (E = kShortEnds) carry their flag in bit 31 of word 0 instead (the
//   top bit of ends[1], which needs 12 of its 16 bits).
// Padded to a power of two: short 32 / 64 bytes, wide 64 / 128 bytes (float / double).
template <typename O, int E> struct DescLayout {
    static constexpr bool kWide = E == kEnds;
    static constexpr int kValWords = (int)(sizeof(O) / 4);
    static constexpr int kEndWords = E / 2;
    static constexpr int kValBase = kValWords == 2 ? (kEndWords + 1) / 2 * 2 : kEndWords;   // doubles on even words
    static constexpr int kFirstWord = kValBase + (E + 1) * kValWords;
    static constexpr int kUsed = kFirstWord + (kWide ? 1 : 0);
    static constexpr int kWords = kUsed <= 4 ? 4 : kUsed <= 8 ? 8 : kUsed <= 16 ? 16 : kUsed <= 32 ? 32 : 64;
    static constexpr int kBytes = kWords * 4;
};
static_assert(kEnds % 2 == 0 && kShortEnds % 2 == 0 && kShortEnds < kEnds, "two ends per word");
static_assert(DescLayout<float, kShortEnds>::kBytes == 32 && DescLayout<double, kShortEnds>::kBytes == 64, "short");
static_assert(DescLayout<float, kEnds>::kBytes == 64 && DescLayout<double, kEnds>::kBytes == 128, "wide");
template <typename O, int E> struct alignas(DescLayout<O, E>::kBytes) Desc { unsigned u[DescLayout<O, E>::kWords]; };
template <typename O> using WideDesc = Desc<O, kEnds>;
template <typename O> using ShortDesc = Desc<O, kShortEnds>;

__device__ __forceinline__ unsigned val_word(float v, int) { return __float_as_uint(v); }
__device__ __forceinline__ unsigned val_word(double v, int half) {
    return (unsigned)(half ? __double2hiint(v) : __double2loint(v));
}

// One descriptor, fetched with 16-byte loads (scalar loads when the address is uniform).
template <typename O, int E>
__device__ __forceinline__ Desc<O, E> load_desc(const Desc<O, E>* __restrict__ src) {
    Desc<O, E> x;
    const v4u* q = reinterpret_cast<const v4u*>(src);
#pragma unroll
    for (int i = 0; i < DescLayout<O, E>::kWords / 4; ++i) {
        const v4u w = q[i];
        x.u[4 * i] = w.x; x.u[4 * i + 1] = w.y; x.u[4 * i + 2] = w.z; x.u[4 * i + 3] = w.w;
    }
    return x;
}
template <typename O, int E>
__device__ __forceinline__ void store_desc(Desc<O, E>* __restrict__ dst, const Desc<O, E>& d) {
    v4u* q = reinterpret_cast<v4u*>(dst);
#pragma unroll
    for (int i = 0; i < DescLayout<O, E>::kWords / 4; ++i) {
        const v4u w = {d.u[4 * i], d.u[4 * i + 1], d.u[4 * i + 2], d.u[4 * i + 3]};
        q[i] = w;
    }
}
template <typename O, int E>
__device__ __forceinline__ int desc_end(const Desc<O, E>& x, int k) {
    const unsigned pair = x.u[k >> 1];
    return (int)((k & 1) ? (pair >> 16) & 0x7fffu : pair & 0xffffu);
}
template <int E>
__device__ __forceinline__ float desc_val(const Desc<float, E>& x, int k) {
    return __uint_as_float(x.u[DescLayout<float, E>::kValBase + k]);
}
template <int E>
__device__ __forceinline__ double desc_val(const Desc<double, E>& x, int k) {
    return __hiloint2double((int)x.u[DescLayout<double, E>::kValBase + 2 * k + 1],
                            (int)x.u[DescLayout<double, E>::kValBase + 2 * k]);
}
template <typename O>
__device__ __forceinline__ unsigned desc_first(const WideDesc<O>& x) { return x.u[DescLayout<O, kEnds>::kFirstWord]; }
template <typename O>
__device__ __forceinline__ bool desc_flagged(const ShortDesc<O>& x) { return (x.u[0] & kOverflowBit) != 0; }

// Fills the ends and values of a descriptor from the ends e[] (tokens, clamped) and the
// advantages v[] of consecutive responses, for the row whose element 0 is token row_first.
template <typename O, int E, int N>
__device__ __forceinline__ void set_desc(Desc<O, E>& d, const long long (&e)[N], const O (&v)[N], long long row_first) {
    static_assert(N >= E + 1, "enough responses loaded");
    constexpr int kRowElems = RowOf<O>::kRowElems;
#pragma unroll
    for (int i = 0; i < DescLayout<O, E>::kWords; ++i) d.u[i] = 0u;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        long long rel = e[k] - row_first;
        rel = rel < 0 ? 0 : (rel > kRowElems ? kRowElems : rel);
        d.u[k >> 1] |= (unsigned)rel << (16 * (k & 1));
    }
#pragma unroll
    for (int k = 0; k < E + 1; ++k)
#pragma unroll
        for (int h = 0; h < DescLayout<O, E>::kValWords; ++h)
            d.u[DescLayout<O, E>::kValBase + k * DescLayout<O, E>::kValWords + h] = val_word(v[k], h);
}

// Where the short descriptor of row r (written by workgroup r) is kept: inside every
// block of kDieBlock rows those with the same r % kDies lie together.
__host__ __device__ __forceinline__ long long short_slot(long long row) {
    const long long block = row & ~(long long)(kDieBlock - 1);
    const int within = (int)(row & (kDieBlock - 1));
    return block + (within % kDies) * (kDieBlock / kDies) + within / kDies;
}
// Short-descriptor slots that n_rows rows take up (whole blocks).
__host__ __device__ __forceinline__ long long short_slots(long long n_rows) {
    return (n_rows + kDieBlock - 1) / kDieBlock * kDieBlock;
}

// ----------------------------------------------------------------------------------
// Pass 1.  Row r holds the elements q in [r*row_elems, (r+1)*row_elems) of the aligned
// index space q = token + skew.  The response that holds a row's first token writes the
// row's descriptors.  Also the data checks: offsets start at 0, do not decrease, and end
// at n_tokens.  Offsets are clamped to [0, n_tokens] before use, so that bad data cannot
// move any access outside the buffers.
// ----------------------------------------------------------------------------------
template <typename A, typename O, typename I>
__global__ __launch_bounds__(kThreads) void k_row_desc(long long n_resp, const A* __restrict__ adv,
                                                       const I* __restrict__ tok_off, long long n_tokens, int skew,
                                                       long long n_rows, ShortDesc<O>* __restrict__ short_desc,
                                                       WideDesc<O>* __restrict__ wide_desc, int32_t* dev_status) {
    constexpr int kRowElems = RowOf<O>::kRowElems;
    const long long stride = (long long)gridDim.x * kThreads;
    bool bad = false;
    for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < n_resp; j += stride) {
        // the loads a short descriptor needs up front (one round trip): the start of the
        // response, the ends of the kShortVals responses from it on, and their advantages
        long long a = (long long)tok_off[j];
        long long e[kVals];
        O v[kVals];
#pragma unroll
        for (int k = 0; k < kShortVals; ++k) {
            e[k] = j + k < n_resp ? (long long)tok_off[j + 1 + k] : n_tokens;
            v[k] = j + k < n_resp ? (O)adv[j + k] : (O)0;
        }
        long long b = e[0];
        bad |= b < a || a < 0 || b > n_tokens;
        if (j == 0) bad |= a != 0;
        if (j == n_resp - 1) bad |= b != n_tokens;
        a = a < 0 ? 0 : (a > n_tokens ? n_tokens : a);
#pragma unroll
        for (int k = 0; k < kShortVals; ++k) e[k] = e[k] < 0 ? 0 : (e[k] > n_tokens ? n_tokens : e[k]);
        b = e[0];
        if (b <= a) continue;
        const long long r_min = a == 0 ? 0 : (a + skew + kRowElems - 1) / kRowElems;
        long long r_max = (b - 1 + skew) / kRowElems;
        if (r_max > n_rows - 1) r_max = n_rows - 1;
        bool have_rest = false;
        for (long long r = r_min; r <= r_max; ++r) {
            const long long row_first = r * kRowElems - skew;   // token of the row's element 0
            long long row_end = row_first + kRowElems;
            if (row_end > n_tokens) row_end = n_tokens;
            const bool wide = e[kShortVals - 1] < row_end;      // more than kShortVals responses
            ShortDesc<O> d;
            set_desc<O, kShortEnds, kVals>(d, e, v, row_first);
            if (wide) d.u[0] |= kOverflowBit;
            store_desc<O, kShortEnds>(short_desc + short_slot(r), d);
            if (wide) {
                if (!have_rest) {   // a second round of loads, for the few rows that need it
#pragma unroll
                    for (int k = kShortVals; k < kVals; ++k) {
                        long long x = j + k < n_resp ? (long long)tok_off[j + 1 + k] : n_tokens;
                        e[k] = x < 0 ? 0 : (x > n_tokens ? n_tokens : x);
                        v[k] = j + k < n_resp ? (O)adv[j + k] : (O)0;
                    }
                    have_rest = true;
                }
                WideDesc<O> x;
                set_desc<O, kEnds, kVals>(x, e, v, row_first);
                x.u[DescLayout<O, kEnds>::kFirstWord] = (unsigned)j | (e[kVals - 1] < row_end ? kOverflowBit : 0u);
                store_desc<O, kEnds>(wide_desc + r, x);
            }
        }
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

// ----------------------------------------------------------------------------------
// Pass 2.
// ----------------------------------------------------------------------------------
// A 16-byte store with the workgroup-scope bit (sc0) set.  It changes nothing in what
// other workgroups may observe; for this pure write stream it measured about 1.5 % faster
// than the default (wavefront-scope) store, while the device- and system-scope bits and
// the non-temporal bit each cost a factor of three or more.
template <typename Vec>
__device__ __forceinline__ void store16(Vec* p, const Vec& v) {
    static_assert(sizeof(Vec) == 16, "one 16-byte vector");
    // The data registers of a store wider than 8 bytes must not be written again in the two
    // wait states after it; the compiler keeps that distance for its own stores but cannot
    // see into this one, hence the s_nop (four wait states, twice what is required).
    asm volatile("global_store_dwordx4 %0, %1, off sc0\n\ts_nop 3" : : "v"(p), "v"(v) : "memory");
}

// Stores one lane's elements of a row: whole vectors where every element of the row is a
// token, element by element in the first and the last row of the output.
template <typename O>
__device__ __forceinline__ void store_lane(O* __restrict__ out, long long row, long long n_rows, long long row_first,
                                           long long n_tokens, int r0, const O (&vals)[RowOf<O>::kLaneElems]) {
    typedef typename VecOf<O>::type Vec;
    constexpr int kVec = VecOf<O>::n;
    constexpr int kRowElems = RowOf<O>::kRowElems;
    O* dst = out + (row_first + r0);
    if (row > 0 && row < n_rows - 1) {
#pragma unroll
        for (int q = 0; q < kLaneVecs; ++q) {
            Vec v;
#pragma unroll
            for (int i = 0; i < kVec; ++i) v[i] = vals[q * kVec + i];
            store16(reinterpret_cast<Vec*>(dst) + q, v);
        }
    } else {
        // elements of the row that are tokens: [rel_lo, rel_hi)
        const int rel_lo = row_first < 0 ? (int)(-row_first) : 0;
        const int rel_hi = n_tokens - row_first < kRowElems ? (int)(n_tokens - row_first) : kRowElems;
#pragma unroll
        for (int i = 0; i < RowOf<O>::kLaneElems; ++i)
            if (r0 + i >= rel_lo && r0 + i < rel_hi) dst[i] = vals[i];
    }
}

template <typename O, int E>
__device__ __forceinline__ void fill_row(const Desc<O, E>& d, O* __restrict__ out, long long row, long long n_rows,
                                         long long n_tokens, int skew) {
    constexpr int kLaneElems = RowOf<O>::kLaneElems;
    constexpr int kWaveElems = RowOf<O>::kWaveElems;
    const long long row_first = row * RowOf<O>::kRowElems - skew;
    const int r0 = (int)threadIdx.x * kLaneElems;
    int e[E];
    O v[E + 1];
#pragma unroll
    for (int k = 0; k < E; ++k) e[k] = desc_end(d, k);
#pragma unroll
    for (int k = 0; k < E + 1; ++k) v[k] = desc_val(d, k);
    // the wavefront's elements [w0, w1) of the row: when the first and the last of them
    // belong to the same response, all of them do
    const int w0 = __builtin_amdgcn_readfirstlane(r0) & ~(kWaveElems - 1);
    const int w1 = w0 + kWaveElems;
    int s_first = 0, s_last = 0;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        s_first += (int)(e[k] <= w0);
        s_last += (int)(e[k] < w1);
    }
    O vals[kLaneElems];
    if (s_first == s_last) {
        O x = v[0];
#pragma unroll
        for (int k = 1; k < E + 1; ++k) x = s_first >= k ? v[k] : x;
#pragma unroll
        for (int i = 0; i < kLaneElems; ++i) vals[i] = x;
    } else {
#pragma unroll
        for (int i = 0; i < kLaneElems; ++i) {
            const int p = r0 + i;
            O x = v[0];
#pragma unroll
            for (int k = 0; k < E; ++k) x = p >= e[k] ? v[k + 1] : x;
            vals[i] = x;
        }
    }
    store_lane<O>(out, row, n_rows, row_first, n_tokens, r0, vals);
}

// A row that more than kVals responses intersect: every lane searches the packed offsets
// for the response of its first element, starting from the response of the row's first
// token.
template <typename A, typename O, typename I>
__device__ __forceinline__ void fill_row_by_search(unsigned first, long long n_resp, const A* __restrict__ adv,
                                                   const I* __restrict__ tok_off, O* __restrict__ out, long long row,
                                                   long long n_rows, long long n_tokens, int skew) {
    constexpr int kLaneElems = RowOf<O>::kLaneElems;
    const long long row_first = row * RowOf<O>::kRowElems - skew;
    const int r0 = (int)threadIdx.x * kLaneElems;
    const long long last = n_resp - 1;
    long long a = (long long)(first & ~kOverflowBit);
    a = a > last ? last : a;
    long long b = last;
    const long long p = row_first + r0;
    while (a < b) {   // first response in [a, b] whose end lies beyond p
        const long long mid = (a + b) >> 1;
        if ((long long)tok_off[mid + 1] > p) b = mid; else a = mid + 1;
    }
    O vals[kLaneElems];
#pragma unroll
    for (int i = 0; i < kLaneElems; ++i) {
        while (a < last && (long long)tok_off[a + 1] <= p + i) ++a;
        vals[i] = (O)adv[a];
    }
    store_lane<O>(out, row, n_rows, row_first, n_tokens, r0, vals);
}

// A row whose short descriptor is flagged: through its wide descriptor, or by the search.
template <typename A, typename O, typename I>
__device__ __forceinline__ void fill_flagged_row(const WideDesc<O>* __restrict__ wide_desc, long long n_resp,
                                              const A* __restrict__ adv, const I* __restrict__ tok_off,
                                              O* __restrict__ out, long long row, long long n_rows,
                                              long long n_tokens, int skew) {
    const WideDesc<O> x = load_desc<O, kEnds>(wide_desc + row);
    const unsigned first = desc_first(x);
    if (first & kOverflowBit) fill_row_by_search<A, O, I>(first, n_resp, adv, tok_off, out, row, n_rows, n_tokens, skew);
    else fill_row<O, kEnds>(x, out, row, n_rows, n_tokens, skew);
}

// (eight wavefronts per SIMD: the bytes in flight per compute unit are what hides the
// latency of the stores, so the register count is held to what full occupancy allows)
template <typename A, typename O, typename I>
__global__ __launch_bounds__(kBcastThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_token_fill(
    // what every row needs comes first: the leading kernel arguments arrive in registers
    const ShortDesc<O>* __restrict__ short_desc, O* __restrict__ out, long long n_tokens, long long n_rows, int skew,
    const WideDesc<O>* __restrict__ wide_desc, long long n_resp, const A* __restrict__ adv,
    const I* __restrict__ tok_off) {
    const long long row = blockIdx.x;   // the grid has n_rows workgroups
    const ShortDesc<O> d = load_desc<O, kShortEnds>(short_desc + short_slot(row));
    // the whole descriptor in one round of loads: without this the part that the flag test
    // does not need is fetched after the branch, one more wait
#pragma unroll
    for (int i = 0; i < DescLayout<O, kShortEnds>::kWords; i += 4) asm volatile("" : : "s"(d.u[i]));
    if (!desc_flagged(d)) fill_row<O, kShortEnds>(d, out, row, n_rows, n_tokens, skew);
    else fill_flagged_row<A, O, I>(wide_desc, n_resp, adv, tok_off, out, row, n_rows, n_tokens, skew);
}

template <typename O>
static long long rows_for(int64_t n_tokens, int skew) {
    return (n_tokens + skew + RowOf<O>::kRowElems - 1) / RowOf<O>::kRowElems;
}

// Workspace: the short descriptors (whole blocks of rows), then the wide ones (one slot
// per row), both 256-byte aligned.
template <typename O>
static size_t short_area_bytes(long long n_rows) {
    return ((size_t)short_slots(n_rows) * sizeof(ShortDesc<O>) + 255) & ~(size_t)255;
}
template <typename O>
static size_t workspace_for(long long n_rows) {
    return short_area_bytes<O>(n_rows) + (((size_t)n_rows * sizeof(WideDesc<O>) + 255) & ~(size_t)255);
}

template <typename A, typename O, typename I>
static int launch_broadcast(int64_t n_resp, const void* adv, const void* tok_off, void* out, int64_t n_tokens,
                            int32_t* dev_status, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    const int skew = (int)((reinterpret_cast<uintptr_t>(out) & 15) / sizeof(O));
    const long long n_rows = rows_for<O>(n_tokens, skew);
    if (n_rows > INT_MAX) return HORA_ERR_UNSUPPORTED;
    if (workspace_for<O>(n_rows) > workspace_bytes) return HORA_ERR_WORKSPACE;
    ShortDesc<O>* short_desc = (ShortDesc<O>*)workspace;
    WideDesc<O>* wide_desc = (WideDesc<O>*)((char*)workspace + short_area_bytes<O>(n_rows));
    long long blocks1 = (n_resp + kThreads - 1) / kThreads;
    if (blocks1 > 65536) blocks1 = 65536;
    hipLaunchKernelGGL((k_row_desc<A, O, I>), dim3((unsigned)blocks1), dim3(kThreads), 0, stream,
                       (long long)n_resp, (const A*)adv, (const I*)tok_off, (long long)n_tokens, skew, n_rows,
                       short_desc, wide_desc, dev_status);
    if (n_rows > 0)
        hipLaunchKernelGGL((k_token_fill<A, O, I>), dim3((unsigned)n_rows), dim3(kBcastThreads), 0, stream,
                           (const ShortDesc<O>*)short_desc, (O*)out, (long long)n_tokens, n_rows, skew,
                           (const WideDesc<O>*)wide_desc, (long long)n_resp, (const A*)adv, (const I*)tok_off);
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

}  // namespace hora

using namespace hora;

extern "C" size_t hora_token_broadcast_workspace_bytes(int64_t n_tokens, int32_t out_t) {
    if (n_tokens < 0 || (out_t != HORA_F32 && out_t != HORA_F64)) return 0;
    // the largest skew a caller's pointer can have gives the most rows
    const size_t bytes = out_t == HORA_F32 ? workspace_for<float>(rows_for<float>(n_tokens, 3))
                                           : workspace_for<double>(rows_for<double>(n_tokens, 1));
    return bytes == 0 ? 256 : bytes;
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
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return HORA_ERR_WORKSPACE;
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
