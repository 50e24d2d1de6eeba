// Pieces shared by the two allocation methods (class histogram and threshold search):
// the launch plan, the workspace layout, and the tie pass that turns (gains above tau,
// tied flag) per prompt into delta, utilities and group offsets.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hora.h"
#include "hora_device.h"
#include "hora_alloc_common.h"

namespace hora {

constexpr int kBig = 1024;                    // threads per workgroup of the allocation kernels
constexpr int kBigWaves = kBig / kWave;       // 16
constexpr int kItems = 4;                     // consecutive prompts per thread and tile
constexpr int kTile = kBig * kItems;          // 4096 prompts
constexpr int kMaxBlocks = 256;               // workgroups of the allocation passes (a power of two)
constexpr int kMaxClasses = HORA_CLASS_MAX_G0 + 1;
constexpr int kMinRow = 32;                   // gain-table row length (a power of two), at least
constexpr int kMaxRow = 512;                  // ... and at most
constexpr int kTableCap = 2 * kMaxClasses * kMinRow;   // doubles per table (4096: rows of 512 up to G0 = 7, of 256 up to G0 = 15)
constexpr unsigned kTiedBit = 0x80000000u;

// ---- threshold search (any posterior) ------------------------------------------------
constexpr int kWinOct = 4;        // octaves of detail a tile keeps of its coarse count (the last ones it walked)
constexpr int kSubBins = 4;       // intervals per octave of the coarse count (two mantissa bits)
constexpr int kListCap = 4096;    // gains a workgroup can set aside for the passes that follow
constexpr long long kCollectMax = (long long)kMaxBlocks * kListCap / 2;   // brackets up to this size are set aside
constexpr unsigned kFlagPending = 1u;      // Bracket::flags: the totals of the last pass have not been applied yet
constexpr unsigned kFlagCollected = 2u;    // ... the last pass left (or kept) the bracket's gains in the lists

struct Bracket {                  // state of the threshold search between two passes
    unsigned long long lo;        // count_gt(lo) >= budget
    unsigned long long hi;        // count_gt(hi) <  budget
    unsigned long long above;     // pairs whose gain is > hi
    unsigned int done;            // 1: the bracket has closed, tau = hi; 2: ran out of gains
    unsigned int flags;           // kFlagPending, kFlagCollected
};
struct AllocHeader {              // 256 bytes at the start of the workspace
    Bracket slot[2];              // pass p reads slot[p & 1] and writes slot[(p + 1) & 1]
    long long inside;             // pairs in the bracket of slot[0] as the coarse count left it (-1: not known)
    unsigned long long tau;       // tau once the search has ended
    unsigned int lists_ok;        // no workgroup ran out of room in its list (written between passes)
    unsigned int pad0;
    unsigned long long ck_top;    // the coarse count left every prompt's walk state at its first gain <= this pattern
    unsigned int pad1[2];
    unsigned long long pad[19];
};
static_assert(sizeof(Bracket) == 32, "bracket size");
static_assert(sizeof(AllocHeader) == 256, "header size");

// What a tile of kTile prompts knows after the coarse count: it walked every prompt down to
// the bottom of octave `stop` (gains in (2^-(stop+1), 2^-stop]) and kept the per-interval
// counts of its last kWinOct octaves; everything above them is in cum_top.
struct CoarseSlot {
    unsigned long long cnt[kWinOct][kSubBins];   // [octave & (kWinOct - 1)][interval]
    unsigned long long cum_top;                  // pairs above the kept octaves
    int stop;                                    // last octave walked
    int exhausted;                               // no prompt of the tile has a gain below it (cap, depth bound, underflow)
};
static_assert(sizeof(CoarseSlot) == 144, "coarse slot size");

struct SelectBins : TallyBins {};  // per-interval tallies of one workgroup in one search pass
// One SelectBins per workgroup (kMaxBlocks of them) and one more for their totals: every
// workgroup stores its tallies with plain stores, a small kernel adds them up.  Atomics of
// all workgroups on one set of intervals serialise at the memory side (hundreds of them
// per address and pass, each a round trip), which cost more than the walks themselves.

struct Plan {
    long long chunk;  // prompts per workgroup, a multiple of kTile
    int nb;           // workgroups
};

inline Plan make_plan(int64_t n) {
    long long tiles = (n + kTile - 1) / kTile;
    long long tpb = (tiles + kMaxBlocks - 1) / kMaxBlocks;
    if (tpb < 1) tpb = 1;
    Plan p;
    p.chunk = tpb * kTile;
    p.nb = (int)((n + p.chunk - 1) / p.chunk);
    if (p.nb < 1) p.nb = 1;
    return p;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
    AllocHeader* header;
    SelectBins* bins;       // [kMaxBlocks + 1]
    int* class_hist;        // [kMaxClasses][kMaxBlocks]: prompts of class c in workgroup b   (CLASS)
    double* gain_table;     // [nc][row]: M_c(l)                                            (CLASS)
    double* surv_table;     // [nc][row]: E_c(l)                                            (CLASS)
    long long* block_ksum;  // [kMaxBlocks] sum of k_i per workgroup
    long long* block_tied;  // [kMaxBlocks] tied prompts per workgroup
    unsigned long long* lists;   // [kMaxBlocks][kListCap] gains set aside by the search passes
    int* list_count;             // [kMaxBlocks] entries in each list, -1 when it did not fit
    CoarseSlot* coarse;          // [tiles]
    double* ck_g;                // [n] walk state of every prompt between the kernels of the search: a gain ...
    int32_t* ck_l;               // [n] ... and its index l
    size_t bytes;
};

// Everything but the coarse slots is sized for kMaxBlocks workgroups and kMaxClasses classes
// whatever n and g0 are; what grows with n (the coarse slots, one per tile of kTile prompts, and
// the walk states, one per prompt) comes last, so that a workspace that served one batch serves
// every smaller one.
inline Workspace carve(void* base, int64_t n) {
    Workspace w;
    char* ptr = (char*)base;
    size_t off = 0;
    w.header = (AllocHeader*)(ptr + off);
    off += sizeof(AllocHeader);
    w.bins = (SelectBins*)(ptr + off);
    off += (size_t)(kMaxBlocks + 1) * sizeof(SelectBins);   // bins[kMaxBlocks]: the totals
    w.class_hist = (int*)(ptr + off);
    off += align256((size_t)kMaxClasses * kMaxBlocks * sizeof(int));
    w.gain_table = (double*)(ptr + off);
    off += align256((size_t)kTableCap * sizeof(double));
    w.surv_table = (double*)(ptr + off);
    off += align256((size_t)kTableCap * sizeof(double));
    w.block_ksum = (long long*)(ptr + off);
    off += align256((size_t)kMaxBlocks * sizeof(long long));
    w.block_tied = (long long*)(ptr + off);
    off += align256((size_t)kMaxBlocks * sizeof(long long));
    w.lists = (unsigned long long*)(ptr + off);
    off += align256((size_t)kMaxBlocks * kListCap * sizeof(unsigned long long));
    w.list_count = (int*)(ptr + off);
    off += align256((size_t)kMaxBlocks * sizeof(int));
    w.coarse = (CoarseSlot*)(ptr + off);
    const size_t tiles = (size_t)((n > 0 ? n : 1) + kTile - 1) / kTile;
    off += align256(tiles * sizeof(CoarseSlot));
    const size_t padded = tiles * (size_t)kTile;
    w.ck_g = (double*)(ptr + off);
    off += align256(padded * sizeof(double));
    w.ck_l = (int32_t*)(ptr + off);
    off += align256(padded * sizeof(int32_t));
    w.bytes = off;
    return w;
}

struct CommonArgs {
    int64_t n;
    int32_t g0;
    int64_t budget;
    int32_t delta_max;
    int32_t* delta;
    double* util;
    void* group_off;
    int32_t off_t;
    hora_alloc_summary* summary;
    int32_t* dev_status;
    void* workspace;
    size_t workspace_bytes;
    hipStream_t stream;
};

inline int check_launch() { return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP; }

// The threshold search for the two kinds of posterior (defined with its kernels).
int run_bisect_counts(const CountsSource& src, const CommonArgs& a, const Plan& p, const Workspace& w);
int run_bisect_posterior(const PosteriorSource& src, const CommonArgs& a, const Plan& p, const Workspace& w);

// ----------------------------------------------------------------------------------
// Tie resolution and output of one tile of a workgroup's chunk, shared by both methods.
//
// Every thread holds kItems consecutive prompts with k (gains above tau) and the tied
// flag.  A workgroup scan of the tied flags gives each prompt the number of tied prompts
// before it; the first r of them (by index) win one more unit.  The group offset of
// prompt i is g0*i + sum_{i'<i} k_i' + min(tied prompts before i, r).
// ----------------------------------------------------------------------------------
struct EmitCarry {
    long long rank_base;   // tied prompts with a lower index than the current tile
    long long ks_base;     // sum of k over prompts with a lower index than the current tile
};

struct EmitShared {        // LDS exchange between the wavefronts of a workgroup, double-buffered
    int tied[2][kBigWaves];
    long long ksum[2][kBigWaves];
};

template <typename V, typename T>
__device__ __forceinline__ void store_items(T* __restrict__ dst, long long pos, long long end, bool vec_ok,
                                            const T (&x)[kItems]) {
    constexpr int kPer = (int)(sizeof(V) / sizeof(T));
    if (vec_ok && pos + kItems <= end) {
#pragma unroll
        for (int q = 0; q < kItems / kPer; ++q) {
            V v;
#pragma unroll
            for (int i = 0; i < kPer; ++i) v[i] = x[q * kPer + i];
            *reinterpret_cast<V*>(dst + pos + q * kPer) = v;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            if (pos + j < end) dst[pos + j] = x[j];
    }
}

// kTiedOnly: delta already holds k for every prompt that is not tied (the caller's kernel
// before stored it): only threads with a tied prompt among theirs store delta again.
template <int kOff, bool kTiedOnly = false>
__device__ __forceinline__ void emit_tile(int tile_parity, long long pos, long long end, long long n, int g0,
                                          long long r, const int (&kk)[kItems], const int (&td)[kItems],
                                          EmitCarry& carry, int (&dd)[kItems], bool (&win)[kItems],
                                          int32_t* __restrict__ delta, void* __restrict__ group_off, bool d_vec,
                                          bool o_vec, EmitShared* sh) {
    const int w = wave_id();
    // tied prompts before this thread inside the wavefront: ballots, no data movement
    int t_before = 0, t_wave = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const unsigned long long m = __ballot(td[j] != 0);
        t_before += lanes_below(m);
        t_wave += __popcll(m);
    }
    if constexpr (kOff == 1) {
        // 32-bit offsets: the caller has checked that the last offset, n * g0 + budget, is below
        // 2^31, so every sum of k and every offset fits 32 bits; ranks are counted from
        // min(tied prompts before the tile, r), which decides the same winners and offsets
        // (a rank only matters below r) and keeps them below 2^32 whatever n is.
        int ks = 0;
#pragma unroll
        for (int j = 0; j < kItems; ++j) ks += kk[j];
        const int ks_incl = wave_incl_scan_i32(ks);
        const int ks_wave = wave_last_i32(ks_incl);
        if (lane_id() == 0) {
            sh->tied[tile_parity][w] = t_wave;
            sh->ksum[tile_parity][w] = (long long)ks_wave;
        }
        __syncthreads();
        const int lane = lane_id();
        const int t_in = lane < kBigWaves ? sh->tied[tile_parity][lane] : 0;
        const int t_scan = wave_incl_scan_i32(t_in);
        const int t_total = __builtin_amdgcn_readlane(t_scan, kBigWaves - 1);
        const int t_lower = w > 0 ? __builtin_amdgcn_readlane(t_scan, w - 1) : 0;
        const int q_in = lane < kBigWaves ? (int)sh->ksum[tile_parity][lane] : 0;
        const int q_scan = wave_incl_scan_i32(q_in);
        const int ks_total = __builtin_amdgcn_readlane(q_scan, kBigWaves - 1);
        const int ks_lower = w > 0 ? __builtin_amdgcn_readlane(q_scan, w - 1) : 0;
        const unsigned r32 = r > 0 ? (unsigned)r : 0u;   // (r <= budget < 2^31; negative only after an error that is reported)
        const unsigned rank_base = carry.rank_base < r ? (unsigned)carry.rank_base : r32;
        unsigned rank = rank_base + (unsigned)(t_lower + t_before);
        int kprior = (int)carry.ks_base + ks_lower + (ks_incl - ks);
        // g0 * pos is below 2^31 (or g0 is 0): the low 32 bits of the product are the product
        const int first = (int)((unsigned)g0 * (unsigned)(unsigned long long)pos);
        int32_t o32[kItems + 1];
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            o32[j] = first + g0 * j + kprior + (int)(rank < r32 ? rank : r32);
            win[j] = td[j] && rank < r32;
            dd[j] = kk[j] + (win[j] ? 1 : 0);
            rank += (unsigned)td[j];
            kprior += kk[j];
        }
        o32[kItems] = first + g0 * kItems + kprior + (int)(rank < r32 ? rank : r32);
        if constexpr (kTiedOnly) {
            bool any_tied = false;
#pragma unroll
            for (int j = 0; j < kItems; ++j) any_tied |= td[j] != 0;
            if (any_tied) store_items<v4i, int32_t>(delta, pos, end, d_vec, dd);
        } else {
            store_items<v4i, int32_t>(delta, pos, end, d_vec, dd);
        }
        int32_t* go = reinterpret_cast<int32_t*>(group_off);
        int32_t first_four[kItems];
#pragma unroll
        for (int j = 0; j < kItems; ++j) first_four[j] = o32[j];
        store_items<v4i, int32_t>(go, pos, end, o_vec, first_four);
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            if (pos + j == n - 1) go[n] = o32[j + 1];
        carry.rank_base += t_total;
        carry.ks_base += ks_total;
        return;
    }
    long long ks = 0, ks_incl = 0, ks_wave = 0;
    if (kOff != 0) {
#pragma unroll
        for (int j = 0; j < kItems; ++j) ks += kk[j];
        ks_incl = wave_incl_scan_i64(ks);
        ks_wave = ((long long)wave_last_i32((int)(ks_incl >> 32)) << 32) |
                  (unsigned)wave_last_i32((int)(ks_incl & 0xffffffffll));
    }
    if (lane_id() == 0) {
        sh->tied[tile_parity][w] = t_wave;
        if (kOff != 0) sh->ksum[tile_parity][w] = ks_wave;
    }
    __syncthreads();
    // totals of the lower wavefronts: lanes 0..15 hold one wavefront's total each, a DPP
    // prefix sum inside the first row of 16 lanes gives every wavefront its base
    const int lane = lane_id();
    const int t_in = lane < kBigWaves ? sh->tied[tile_parity][lane] : 0;
    const int t_scan = wave_incl_scan_i32(t_in);
    const int t_total = __builtin_amdgcn_readlane(t_scan, kBigWaves - 1);
    const int t_lower = w > 0 ? __builtin_amdgcn_readlane(t_scan, w - 1) : 0;
    long long ks_lower = 0, ks_total = 0;
    if (kOff != 0) {
        const long long q_in = lane < kBigWaves ? sh->ksum[tile_parity][lane] : 0;
        const long long q_scan = wave_incl_scan_i64(q_in);
        const int q_lo = (int)(q_scan & 0xffffffffll), q_hi = (int)(q_scan >> 32);
        ks_total = ((long long)__builtin_amdgcn_readlane(q_hi, kBigWaves - 1) << 32) |
                   (unsigned)__builtin_amdgcn_readlane(q_lo, kBigWaves - 1);
        if (w > 0)
            ks_lower = ((long long)__builtin_amdgcn_readlane(q_hi, w - 1) << 32) |
                       (unsigned)__builtin_amdgcn_readlane(q_lo, w - 1);
    }
    long long rank = carry.rank_base + t_lower + t_before;
    long long kprior = carry.ks_base + ks_lower + (ks_incl - ks);
    long long off[kItems + 1];
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        off[j] = (long long)g0 * (pos + j) + kprior + (rank < r ? rank : r);
        win[j] = td[j] && rank < r;
        dd[j] = kk[j] + (win[j] ? 1 : 0);
        rank += td[j];
        kprior += kk[j];
    }
    off[kItems] = (long long)g0 * (pos + kItems) + kprior + (rank < r ? rank : r);

    if constexpr (kTiedOnly) {
        bool any_tied = false;
#pragma unroll
        for (int j = 0; j < kItems; ++j) any_tied |= td[j] != 0;
        if (any_tied) store_items<v4i, int32_t>(delta, pos, end, d_vec, dd);
    } else {
        store_items<v4i, int32_t>(delta, pos, end, d_vec, dd);
    }
    if (kOff == 2) {
        long long* go = reinterpret_cast<long long*>(group_off);
        long long o64[kItems];
#pragma unroll
        for (int j = 0; j < kItems; ++j) o64[j] = off[j];
        store_items<v2l, long long>(go, pos, end, o_vec, o64);
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            if (pos + j == n - 1) go[n] = off[j + 1];
    }
    carry.rank_base += t_total;
    carry.ks_base += ks_total;
}

__device__ __forceinline__ void load_items_i32(const int32_t* __restrict__ src, long long pos, long long end,
                                               bool vec_ok, int fill, int (&v)[kItems]) {
    if (vec_ok && pos + kItems <= end) {
#pragma unroll
        for (int q = 0; q < kItems / 4; ++q) {
            const v4i x = *reinterpret_cast<const v4i*>(src + pos + 4 * q);
            v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kItems; ++j) v[j] = (pos + j < end) ? src[pos + j] : fill;
    }
}


}  // namespace hora
