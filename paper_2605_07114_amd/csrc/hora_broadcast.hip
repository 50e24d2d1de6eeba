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

// Row descriptor with E ends for S value streams, an array of 32-bit words (little endian):
//   words [0, E/2)              ends[k], 16 bits each: end of the k-th response that
//                               intersects the row, as an element index relative to the
//                               row, clamped to [0, row length]; unused entries hold the
//                               row length
//   then (E+1)*S values of type O   vals[k*S + s]: value of stream s for that response
//   wide descriptors (E = kEnds) then hold one word `first`: index of the response that
//   holds the row's first token, bit 31 set when more than E+1 responses intersect the
//   row; short ones (E = kShortEnds) carry their flag in bit 31 of word 0 instead (the
//   top bit of ends[1], which needs 12 of its 16 bits).
// Padded to a power of two.  One stream: short 32 / 64 bytes, wide 64 / 128 bytes (float /
// double); two streams: short 64 / 128, wide 128 / 256.
template <typename O, int E, int S> struct DescLayout {
    static constexpr bool kWide = E == kEnds;
    static constexpr int kValWords = (int)(sizeof(O) / 4);
    static constexpr int kEndWords = E / 2;
    static constexpr int kValBase = kValWords == 2 ? (kEndWords + 1) / 2 * 2 : kEndWords;   // doubles on even words
    static constexpr int kFirstWord = kValBase + (E + 1) * S * kValWords;
    static constexpr int kUsed = kFirstWord + (kWide ? 1 : 0);
    static constexpr int kWords = kUsed <= 4 ? 4 : kUsed <= 8 ? 8 : kUsed <= 16 ? 16 : kUsed <= 32 ? 32 : 64;
    static constexpr int kBytes = kWords * 4;
};
static_assert(kEnds % 2 == 0 && kShortEnds % 2 == 0 && kShortEnds < kEnds, "two ends per word");
static_assert(DescLayout<float, kShortEnds, 1>::kBytes == 32 && DescLayout<double, kShortEnds, 1>::kBytes == 64, "short");
static_assert(DescLayout<float, kEnds, 1>::kBytes == 64 && DescLayout<double, kEnds, 1>::kBytes == 128, "wide");
static_assert(DescLayout<float, kShortEnds, 2>::kBytes == 64 && DescLayout<double, kShortEnds, 2>::kBytes == 128, "short, two streams");
static_assert(DescLayout<float, kEnds, 2>::kBytes == 128 && DescLayout<double, kEnds, 2>::kBytes == 256, "wide, two streams");
static_assert(DescLayout<double, kEnds, 2>::kUsed <= 64, "the widest descriptor fits");
template <typename O, int E, int S> struct alignas(DescLayout<O, E, S>::kBytes) Desc { unsigned u[DescLayout<O, E, S>::kWords]; };
template <typename O, int S> using WideDesc = Desc<O, kEnds, S>;
template <typename O, int S> using ShortDesc = Desc<O, kShortEnds, S>;

__device__ __forceinline__ unsigned val_word(float v, int) { return __float_as_uint(v); }
__device__ __forceinline__ unsigned val_word(double v, int half) {
    return (unsigned)(half ? __double2hiint(v) : __double2loint(v));
}

// One descriptor, fetched with 16-byte loads (scalar loads when the address is uniform).
template <typename O, int E, int S>
__device__ __forceinline__ Desc<O, E, S> load_desc(const Desc<O, E, S>* __restrict__ src) {
    Desc<O, E, S> x;
    const v4u* q = reinterpret_cast<const v4u*>(src);
#pragma unroll
    for (int i = 0; i < DescLayout<O, E, S>::kWords / 4; ++i) {
        const v4u w = q[i];
        x.u[4 * i] = w.x; x.u[4 * i + 1] = w.y; x.u[4 * i + 2] = w.z; x.u[4 * i + 3] = w.w;
    }
    return x;
}
template <typename O, int E, int S>
__device__ __forceinline__ void store_desc(Desc<O, E, S>* __restrict__ dst, const Desc<O, E, S>& d) {
    v4u* q = reinterpret_cast<v4u*>(dst);
#pragma unroll
    for (int i = 0; i < DescLayout<O, E, S>::kWords / 4; ++i) {
        const v4u w = {d.u[4 * i], d.u[4 * i + 1], d.u[4 * i + 2], d.u[4 * i + 3]};
        q[i] = w;
    }
}
template <typename O, int E, int S>
__device__ __forceinline__ int desc_end(const Desc<O, E, S>& x, int k) {
    const unsigned pair = x.u[k >> 1];
    return (int)((k & 1) ? (pair >> 16) & 0x7fffu : pair & 0xffffu);
}
// value of stream st for the k-th response of the descriptor
template <int E, int S>
__device__ __forceinline__ float desc_val(const Desc<float, E, S>& x, int k, int st) {
    return __uint_as_float(x.u[DescLayout<float, E, S>::kValBase + k * S + st]);
}
template <int E, int S>
__device__ __forceinline__ double desc_val(const Desc<double, E, S>& x, int k, int st) {
    return __hiloint2double((int)x.u[DescLayout<double, E, S>::kValBase + 2 * (k * S + st) + 1],
                            (int)x.u[DescLayout<double, E, S>::kValBase + 2 * (k * S + st)]);
}
template <typename O, int S>
__device__ __forceinline__ unsigned desc_first(const WideDesc<O, S>& x) { return x.u[DescLayout<O, kEnds, S>::kFirstWord]; }
template <typename O, int S>
__device__ __forceinline__ bool desc_flagged(const ShortDesc<O, S>& x) { return (x.u[0] & kOverflowBit) != 0; }

// Fills the ends and values of a descriptor from the ends e[] (tokens, clamped) and the
// values v[][stream] of consecutive responses, for the row whose element 0 is token row_first.
template <typename O, int E, int S, int N>
__device__ __forceinline__ void set_desc(Desc<O, E, S>& d, const long long (&e)[N], const O (&v)[N][S], long long row_first) {
    static_assert(N >= E + 1, "enough responses loaded");
    constexpr int kRowElems = RowOf<O>::kRowElems;
    typedef DescLayout<O, E, S> L;
#pragma unroll
    for (int i = 0; i < L::kWords; ++i) d.u[i] = 0u;
#pragma unroll
    for (int k = 0; k < E; ++k) {
        long long rel = e[k] - row_first;
        rel = rel < 0 ? 0 : (rel > kRowElems ? kRowElems : rel);
        d.u[k >> 1] |= (unsigned)rel << (16 * (k & 1));
    }
#pragma unroll
    for (int k = 0; k < E + 1; ++k)
#pragma unroll
        for (int st = 0; st < S; ++st)
#pragma unroll
            for (int h = 0; h < L::kValWords; ++h)
                d.u[L::kValBase + (k * S + st) * L::kValWords + h] = val_word(v[k][st], h);
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
// move any access outside the buffers.  With two streams (S = 2) the descriptors carry the
// values of both per-response arrays, so that pass 2 fetches one descriptor per row for both
// outputs.
// ----------------------------------------------------------------------------------
template <typename A, int S> struct Streams { const A* p[S]; };
template <typename O, int S> struct Outputs { O* p[S]; };

template <typename A, typename O, typename I, int S>
__global__ __launch_bounds__(kThreads) void k_row_desc(long long n_resp, Streams<A, S> adv,
                                                       const I* __restrict__ tok_off, long long n_tokens, int skew,
                                                       long long n_rows, ShortDesc<O, S>* __restrict__ short_desc,
                                                       WideDesc<O, S>* __restrict__ wide_desc, int32_t* dev_status) {
    constexpr int kRowElems = RowOf<O>::kRowElems;
    const long long stride = (long long)gridDim.x * kThreads;
    bool bad = false;
    for (long long j = (long long)blockIdx.x * kThreads + threadIdx.x; j < n_resp; j += stride) {
        // the loads a short descriptor needs up front (one round trip): the start of the
        // response, the ends of the kShortVals responses from it on, and their values
        long long a = (long long)tok_off[j];
        long long e[kVals];
        O v[kVals][S];
#pragma unroll
        for (int k = 0; k < kShortVals; ++k) {
            e[k] = j + k < n_resp ? (long long)tok_off[j + 1 + k] : n_tokens;
#pragma unroll
            for (int st = 0; st < S; ++st) v[k][st] = j + k < n_resp ? (O)adv.p[st][j + k] : (O)0;
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
            ShortDesc<O, S> d;
            set_desc<O, kShortEnds, S, kVals>(d, e, v, row_first);
            if (wide) d.u[0] |= kOverflowBit;
            store_desc<O, kShortEnds, S>(short_desc + short_slot(r), d);
            if (wide) {
                if (!have_rest) {   // a second round of loads, for the few rows that need it
#pragma unroll
                    for (int k = kShortVals; k < kVals; ++k) {
                        long long x = j + k < n_resp ? (long long)tok_off[j + 1 + k] : n_tokens;
                        e[k] = x < 0 ? 0 : (x > n_tokens ? n_tokens : x);
#pragma unroll
                        for (int st = 0; st < S; ++st) v[k][st] = j + k < n_resp ? (O)adv.p[st][j + k] : (O)0;
                    }
                    have_rest = true;
                }
                WideDesc<O, S> x;
                set_desc<O, kEnds, S, kVals>(x, e, v, row_first);
                x.u[DescLayout<O, kEnds, S>::kFirstWord] = (unsigned)j | (e[kVals - 1] < row_end ? kOverflowBit : 0u);
                store_desc<O, kEnds, S>(wide_desc + r, x);
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

// One wavefront's part of a row for stream kSt (row_thread: the thread's index within the row).
template <typename O, int E, int S, int kSt>
__device__ __forceinline__ void fill_row(const Desc<O, E, S>& d, O* __restrict__ out, long long row, long long n_rows,
                                         long long n_tokens, int skew, int row_thread) {
    constexpr int kLaneElems = RowOf<O>::kLaneElems;
    constexpr int kWaveElems = RowOf<O>::kWaveElems;
    const long long row_first = row * RowOf<O>::kRowElems - skew;
    const int r0 = row_thread * kLaneElems;
    int e[E];
    O v[E + 1];
#pragma unroll
    for (int k = 0; k < E; ++k) e[k] = desc_end(d, k);
#pragma unroll
    for (int k = 0; k < E + 1; ++k) v[k] = desc_val(d, k, kSt);
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
                                                   long long n_rows, long long n_tokens, int skew, int row_thread) {
    constexpr int kLaneElems = RowOf<O>::kLaneElems;
    const long long row_first = row * RowOf<O>::kRowElems - skew;
    const int r0 = row_thread * kLaneElems;
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
template <typename A, typename O, typename I, int S, int kSt>
__device__ __forceinline__ void fill_flagged_row(const WideDesc<O, S>* __restrict__ wide_desc, long long n_resp,
                                                 const A* __restrict__ adv, const I* __restrict__ tok_off,
                                                 O* __restrict__ out, long long row, long long n_rows,
                                                 long long n_tokens, int skew, int row_thread) {
    const WideDesc<O, S> x = load_desc<O, kEnds, S>(wide_desc + row);
    const unsigned first = desc_first(x);
    if (first & kOverflowBit)
        fill_row_by_search<A, O, I>(first, n_resp, adv, tok_off, out, row, n_rows, n_tokens, skew, row_thread);
    else fill_row<O, kEnds, S, kSt>(x, out, row, n_rows, n_tokens, skew, row_thread);
}

template <typename A, typename O, typename I, int S, int kSt>
__device__ __forceinline__ void fill_stream(const ShortDesc<O, S>& d, const WideDesc<O, S>* __restrict__ wide_desc,
                                            long long n_resp, const A* __restrict__ adv,
                                            const I* __restrict__ tok_off, O* __restrict__ out, long long row,
                                            long long n_rows, long long n_tokens, int skew, int row_thread) {
    if (!desc_flagged(d)) fill_row<O, kShortEnds, S, kSt>(d, out, row, n_rows, n_tokens, skew, row_thread);
    else fill_flagged_row<A, O, I, S, kSt>(wide_desc, n_resp, adv, tok_off, out, row, n_rows, n_tokens, skew, row_thread);
}

// One workgroup per row and stream.  With two streams the grid holds all rows of the first
// stream, then all rows of the second: measured on large_bcast, workgroups that write both
// streams of a row (64 bytes per lane, or 32 bytes per lane from twice as many threads) reach
// 5.5 - 5.7 TB/s because the memory then sees two interleaved write streams, against 6.4 TB/s
// for one stream after the other; what the two-stream call saves is the second pass 1 and the
// second launch, not the descriptor fetch.
// (eight wavefronts per SIMD: the bytes in flight per compute unit are what hides the
// latency of the stores, so the register count is held to what full occupancy allows)
template <typename A, typename O, typename I, int S>
__global__ __launch_bounds__(kBcastThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_token_fill(
    // what every row needs comes first: the leading kernel arguments arrive in registers
    const ShortDesc<O, S>* __restrict__ short_desc, Outputs<O, S> out, long long n_tokens, long long n_rows, int skew,
    const WideDesc<O, S>* __restrict__ wide_desc, long long n_resp, Streams<A, S> adv,
    const I* __restrict__ tok_off) {
    const bool second = S == 2 && (long long)blockIdx.x >= n_rows;   // the grid has S * n_rows workgroups
    const long long row = (long long)blockIdx.x - (second ? n_rows : 0);
    const ShortDesc<O, S> d = load_desc<O, kShortEnds, S>(short_desc + short_slot(row));
    // the whole descriptor in one round of loads: without this the part that the flag test
    // does not need is fetched after the branch, one more wait
#pragma unroll
    for (int i = 0; i < DescLayout<O, kShortEnds, S>::kWords; i += 4) asm volatile("" : : "s"(d.u[i]));
    if constexpr (S == 1) {
        fill_stream<A, O, I, 1, 0>(d, wide_desc, n_resp, adv.p[0], tok_off, out.p[0], row, n_rows, n_tokens, skew,
                                   (int)threadIdx.x);
    } else {
        if (!second)
            fill_stream<A, O, I, 2, 0>(d, wide_desc, n_resp, adv.p[0], tok_off, out.p[0], row, n_rows, n_tokens, skew,
                                       (int)threadIdx.x);
        else
            fill_stream<A, O, I, 2, 1>(d, wide_desc, n_resp, adv.p[1], tok_off, out.p[1], row, n_rows, n_tokens, skew,
                                       (int)threadIdx.x);
    }
}

template <typename O>
static long long rows_for(int64_t n_tokens, int skew) {
    return (n_tokens + skew + RowOf<O>::kRowElems - 1) / RowOf<O>::kRowElems;
}

// Workspace: the short descriptors (whole blocks of rows), then the wide ones (one slot
// per row), both 256-byte aligned.
template <typename O, int S>
static size_t short_area_bytes(long long n_rows) {
    return ((size_t)short_slots(n_rows) * sizeof(ShortDesc<O, S>) + 255) & ~(size_t)255;
}
template <typename O, int S>
static size_t workspace_for(long long n_rows) {
    return short_area_bytes<O, S>(n_rows) + (((size_t)n_rows * sizeof(WideDesc<O, S>) + 255) & ~(size_t)255);
}

template <typename A, typename O, typename I, int S>
static int launch_broadcast(int64_t n_resp, const void* const* adv, const void* tok_off, void* const* out,
                            int64_t n_tokens, int32_t* dev_status, void* workspace, size_t workspace_bytes,
                            hipStream_t stream) {
    const int skew = (int)((reinterpret_cast<uintptr_t>(out[0]) & 15) / sizeof(O));
    const long long n_rows = rows_for<O>(n_tokens, skew);
    if (n_rows * S > INT_MAX) return HORA_ERR_UNSUPPORTED;
    if (workspace_for<O, S>(n_rows) > workspace_bytes) return HORA_ERR_WORKSPACE;
    ShortDesc<O, S>* short_desc = (ShortDesc<O, S>*)workspace;
    WideDesc<O, S>* wide_desc = (WideDesc<O, S>*)((char*)workspace + short_area_bytes<O, S>(n_rows));
    Streams<A, S> in;
    Outputs<O, S> dst;
    for (int st = 0; st < S; ++st) { in.p[st] = (const A*)adv[st]; dst.p[st] = (O*)out[st]; }
    long long blocks1 = (n_resp + kThreads - 1) / kThreads;
    if (blocks1 > 65536) blocks1 = 65536;
    hipLaunchKernelGGL((k_row_desc<A, O, I, S>), dim3((unsigned)blocks1), dim3(kThreads), 0, stream,
                       (long long)n_resp, in, (const I*)tok_off, (long long)n_tokens, skew, n_rows,
                       short_desc, wide_desc, dev_status);
    if (n_rows > 0)
        hipLaunchKernelGGL((k_token_fill<A, O, I, S>), dim3((unsigned)(n_rows * S)), dim3(kBcastThreads), 0, stream,
                           (const ShortDesc<O, S>*)short_desc, dst, (long long)n_tokens, n_rows, skew,
                           (const WideDesc<O, S>*)wide_desc, (long long)n_resp, in, (const I*)tok_off);
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

template <int S>
static size_t broadcast_workspace_bytes(int64_t n_tokens, int32_t out_t) {
    if (n_tokens < 0 || (out_t != HORA_F32 && out_t != HORA_F64)) return 0;
    // the largest skew a caller's pointer can have gives the most rows
    const size_t bytes = out_t == HORA_F32 ? workspace_for<float, S>(rows_for<float>(n_tokens, 3))
                                           : workspace_for<double, S>(rows_for<double>(n_tokens, 1));
    return bytes == 0 ? 256 : bytes;
}

// Argument checks and dispatch shared by the one- and the two-stream entry point.
template <int S>
static int broadcast_entry(int64_t n_resp, const void* const* adv, int32_t adv_t, const void* tok_off, int32_t off_t,
                           void* const* tok_adv, int32_t out_t, int64_t n_tokens, int32_t* dev_status,
                           void* workspace, size_t workspace_bytes, hipStream_t s) {
    if (n_resp < 0 || n_tokens < 0 || !dev_status) return HORA_ERR_INVALID_ARG;
    if (adv_t != HORA_F32 && adv_t != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (out_t != HORA_F32 && out_t != HORA_F64) return HORA_ERR_INVALID_ARG;
    if (off_t != HORA_I32 && off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (adv_t == HORA_F32 && out_t == HORA_F64) return HORA_ERR_INVALID_ARG;  // never widen
    if (n_resp == 0) return n_tokens == 0 ? HORA_OK : HORA_ERR_INVALID_ARG;
    if (n_resp >= (1ll << 31)) return HORA_ERR_UNSUPPORTED;
    if (!tok_off) return HORA_ERR_INVALID_ARG;
    if (off_t == HORA_I32 && n_tokens >= (1ll << 31)) return HORA_ERR_INVALID_ARG;
    const uintptr_t amask = adv_t == HORA_F32 ? 3 : 7, omask = out_t == HORA_F32 ? 3 : 7,
                    imask = off_t == HORA_I32 ? 3 : 7;
    for (int st = 0; st < S; ++st) {
        if (!adv[st]) return HORA_ERR_INVALID_ARG;
        if (n_tokens > 0 && !tok_adv[st]) return HORA_ERR_INVALID_ARG;
        if ((reinterpret_cast<uintptr_t>(adv[st]) & amask) || (reinterpret_cast<uintptr_t>(tok_adv[st]) & omask))
            return HORA_ERR_INVALID_ARG;
        // the outputs share one row grid: their 16-byte misalignment must be the same
        if ((reinterpret_cast<uintptr_t>(tok_adv[st]) & 15) != (reinterpret_cast<uintptr_t>(tok_adv[0]) & 15))
            return HORA_ERR_INVALID_ARG;
    }
    if (reinterpret_cast<uintptr_t>(tok_off) & imask) return HORA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return HORA_ERR_WORKSPACE;
#define HORA_BCAST(A, O)                                                                                       \
    (off_t == HORA_I32 ? launch_broadcast<A, O, int32_t, S>(n_resp, adv, tok_off, tok_adv, n_tokens,           \
                                                            dev_status, workspace, workspace_bytes, s)         \
                       : launch_broadcast<A, O, long long, S>(n_resp, adv, tok_off, tok_adv, n_tokens,         \
                                                              dev_status, workspace, workspace_bytes, s))
    if (adv_t == HORA_F32) return HORA_BCAST(float, float);
    if (out_t == HORA_F32) return HORA_BCAST(double, float);
    return HORA_BCAST(double, double);
#undef HORA_BCAST
}

}  // namespace hora

using namespace hora;

extern "C" size_t hora_token_broadcast_workspace_bytes(int64_t n_tokens, int32_t out_t) {
    return broadcast_workspace_bytes<1>(n_tokens, out_t);
}

extern "C" size_t hora_token_broadcast2_workspace_bytes(int64_t n_tokens, int32_t out_t) {
    return broadcast_workspace_bytes<2>(n_tokens, out_t);
}

extern "C" int hora_token_broadcast(int64_t n_resp, const void* adv, int32_t adv_t, const void* tok_off,
                                    int32_t off_t, void* tok_adv, int32_t out_t, int64_t n_tokens,
                                    int32_t* dev_status, void* workspace, size_t workspace_bytes, void* stream) {
    const void* in[1] = {adv};
    void* out[1] = {tok_adv};
    return broadcast_entry<1>(n_resp, in, adv_t, tok_off, off_t, out, out_t, n_tokens, dev_status, workspace,
                              workspace_bytes, (hipStream_t)stream);
}

extern "C" int hora_token_broadcast2(int64_t n_resp, const void* adv_a, const void* adv_b, int32_t adv_t,
                                     const void* tok_off, int32_t off_t, void* tok_a, void* tok_b, int32_t out_t,
                                     int64_t n_tokens, int32_t* dev_status, void* workspace, size_t workspace_bytes,
                                     void* stream) {
    const void* in[2] = {adv_a, adv_b};
    void* out[2] = {tok_a, tok_b};
    return broadcast_entry<2>(n_resp, in, adv_t, tok_off, off_t, out, out_t, n_tokens, dev_status, workspace,
                              workspace_bytes, (hipStream_t)stream);
}
