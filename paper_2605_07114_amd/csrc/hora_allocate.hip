// Phase-B allocation kernels and entry points (Sec. 3.2, Alg. 1, Prop. 1, App. A).
//
// The allocation is the set of the `budget` largest marginal gains over all
// (prompt, l) pairs, ordered by (canonical binary64 gain descending, prompt index
// ascending).  Because every prompt's gain sequence decreases strictly, this set is
// described by a threshold tau (the budget-th largest gain): prompt i gets
//     delta_i = #{l : M_i(l) > tau} + [M_i(k_i) == tau and rank_i < r],
// where rank_i counts the prompts tied at tau with a lower index and
// r = budget - sum_i #{l : M_i(l) > tau}.
//
// Two ways to find tau:
//  CLASS  (shared prior): gains depend on c_i only.  Pass 1 takes a histogram of c per
//         workgroup and evaluates the G0+1 gain sequences once into a table.  Pass 2
//         (every workgroup on its own, no grid-wide wait) ranks the table entries
//         against the histogram to find tau, then writes its share of the outputs.
//  BISECT (any posterior): the bracket of tau's bit pattern is narrowed in passes; in
//         each pass every prompt walks its gains down to the bracket (a monotone
//         search) and the gains inside it are tallied per interval, so that a pass
//         cuts the bracket 128-fold or more (a 256-way bisection step).
// Both resolve the ties at tau by prompt index with prefix counts.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>
#include <mutex>

#include "hora.h"
#include "hora_device.h"
#include "hora_alloc_common.h"

namespace hora {

constexpr int kBig = 1024;                    // threads per workgroup of the pass-1 / pass-2 / write kernels
constexpr int kBigWaves = kBig / kWave;       // 16
constexpr int kItems = 4;                     // consecutive prompts per thread and tile
constexpr int kTile = kBig * kItems;          // 4096 prompts
constexpr int kMaxBlocks = 256;               // workgroups of the allocation passes (a power of two)
constexpr int kMaxClasses = HORA_CLASS_MAX_G0 + 1;
constexpr int kMinRow = 32;                   // gain-table row length (a power of two), at least
constexpr int kMaxRow = 256;                  // ... and at most
constexpr int kTableCap = kMaxClasses * kMinRow;   // doubles per table (2048)
constexpr unsigned kTiedBit = 0x80000000u;
constexpr int kPairCap = 16384;               // (table entry, class) pairs ranked one per thread when they fit

constexpr int kSoloMaxPrompts = 2048;   // up to here one workgroup searches alone
constexpr int kParallelPasses = 7;      // launched grid-wide; a single-workgroup finisher covers the rest
constexpr unsigned long long kWindowStep = 4ull << 52;   // 4 exponent steps of the bit pattern: a factor 16 in value
constexpr int kSoloMaxPasses = 512 + 10;   // windows from the largest gain down to zero, plus the narrowing passes
constexpr int kListCap = 1024;             // gains a workgroup can set aside for the passes that follow
constexpr long long kCollectMax = 65536;   // a bracket with no more pairs than this is set aside (256 per workgroup on average)
constexpr unsigned kFlagPending = 1u;      // Bracket::flags: the totals of the last pass have not been applied yet
constexpr unsigned kFlagCollected = 2u;    // ... the last pass left (or kept) the bracket's gains in the lists

struct Bracket {                  // state of the threshold search between two passes
    unsigned long long lo;        // count_gt(lo) >= budget
    unsigned long long hi;        // count_gt(hi) <  budget
    unsigned long long above;     // pairs whose gain is > hi
    unsigned int done;            // 1: the bracket has closed, tau = hi; 2: ran out of gains
    unsigned int flags;           // kFlagPending, kFlagCollected
};
struct AllocHeader {              // 256 bytes at the start of the workspace, zero at rest
    unsigned long long unused0;
    unsigned long long hi;        // bits of max_i M_i(0), gathered with atomicMax
    Bracket slot[2];              // pass p reads slot[p & 1] and writes slot[(p + 1) & 1]
    unsigned long long hi_cur;    // tau once the search has ended
    unsigned int lists_ok;        // no workgroup ran out of room in its list (written between passes)
    unsigned int pad0;
    unsigned long long pad[20];
};
static_assert(sizeof(Bracket) == 32, "bracket size");
static_assert(sizeof(AllocHeader) == 256, "header size");

struct SelectBins {               // per-interval tallies of one workgroup in one search pass
    unsigned long long cnt[kBins];       // pairs whose gain falls into the interval
    unsigned long long vmax[kBins];      // largest gain pattern seen in the interval
    unsigned long long vmin_inv[kBins];  // ~(smallest gain pattern seen in the interval)
};
// One SelectBins per workgroup (kMaxBlocks of them) and one more for their totals: every
// workgroup stores its tallies with plain stores, a small kernel adds them up.  Atomics of
// all workgroups on one set of intervals serialise at the memory side (hundreds of them
// per address and pass, each a round trip), which cost more than the walks themselves.

struct BisectSolution {           // written by k_bisect_scan, read by k_bisect_write
    long long r;                  // units for the prompts tied at tau
    long long pad[31];
};
static_assert(sizeof(BisectSolution) == 256, "solution size");

struct Plan {
    long long chunk;  // prompts per workgroup, a multiple of kTile
    int nb;           // workgroups
};

static Plan make_plan(int64_t n) {
    long long tiles = (n + kTile - 1) / kTile;
    long long tpb = (tiles + kMaxBlocks - 1) / kMaxBlocks;
    if (tpb < 1) tpb = 1;
    Plan p;
    p.chunk = tpb * kTile;
    p.nb = (int)((n + p.chunk - 1) / p.chunk);
    if (p.nb < 1) p.nb = 1;
    return p;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
    AllocHeader* header;
    BisectSolution* sol;
    SelectBins* bins;
    int* class_hist;        // [kMaxClasses][kMaxBlocks]: prompts of class c in workgroup b
    double* gain_table;     // [nc][row]: M_c(l)
    double* surv_table;     // [nc][row]: E_c(l)
    long long* block_ksum;  // [nb] sums, then exclusive prefixes, of k_i          (BISECT)
    long long* block_tied;  // [nb] sums, then exclusive prefixes, of tied flags   (BISECT)
    unsigned long long* lists;   // [kMaxBlocks][kListCap] gains set aside by the search passes (BISECT)
    int* list_count;             // [kMaxBlocks] entries in each list, -1 when it did not fit
    size_t bytes;
};

// The arrays are sized for kMaxBlocks workgroups and kMaxClasses classes whatever n and
// g0 are, so that a workspace that served one batch serves every other one.
static Workspace carve(void* base) {
    Workspace w;
    char* ptr = (char*)base;
    size_t off = 0;
    w.header = (AllocHeader*)(ptr + off);
    off += sizeof(AllocHeader);
    w.sol = (BisectSolution*)(ptr + off);
    off += sizeof(BisectSolution);
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
    w.bytes = off;
    return w;
}

// ----------------------------------------------------------------------------------
// Gain / utility tables (Eq. 3, Eq. 5): one thread per posterior, l-major output so
// that the stores of a wavefront are contiguous.
// ----------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_gain_table(long long n, const double* __restrict__ alpha,
                                                         const double* __restrict__ beta, int count,
                                                         double* __restrict__ gains,
                                                         double* __restrict__ util) {
    long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    double a = alpha[i], b = beta[i];
    double s = a + b;
    double m = gain_first(a, s);
    double e = 1.0;
    double lf = 0.0;
    for (int l = 0; l < count; ++l) {
        if (gains) gains[(long long)l * n + i] = m;
        if (util) util[(long long)l * n + i] = 1.0 - e;
        m = gain_next(m, b, s, lf);
        e = surv_next(e, b, s, lf);
        lf += 1.0;
    }
}

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

template <int kOff>
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

    store_items<v4i, int32_t>(delta, pos, end, d_vec, dd);
    if (kOff == 1) {
        int32_t* go = reinterpret_cast<int32_t*>(group_off);
        int32_t o32[kItems];
#pragma unroll
        for (int j = 0; j < kItems; ++j) o32[j] = (int32_t)off[j];
        store_items<v4i, int32_t>(go, pos, end, o_vec, o32);
#pragma unroll
        for (int j = 0; j < kItems; ++j)
            if (pos + j == n - 1) go[n] = (int32_t)off[j + 1];
    } else if (kOff == 2) {
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

// ----------------------------------------------------------------------------------
// CLASS pass 1: per-workgroup histogram of c (lane k of every wavefront accumulates the
// count of class k from wavefront ballots), and, in one extra workgroup, the gain and
// survival tables of the G0+1 classes.
// ----------------------------------------------------------------------------------
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

__global__ __launch_bounds__(kBig) void k_class_hist(const int32_t* __restrict__ c, long long n, int g0,
                                                     double alpha0, double beta0, long long chunk, int nb, int row,
                                                     int* __restrict__ class_hist, double* __restrict__ gain_table,
                                                     double* __restrict__ surv_table, int32_t* dev_status) {
    __shared__ int s_cnt[kBigWaves][kWave];
    const int lane = lane_id();
    if ((int)blockIdx.x == nb) {   // the extra workgroup: tables, one lane per class
        if (threadIdx.x <= (unsigned)g0) {
            const double a = alpha0 + (double)lane;
            const double b = beta0 + (double)(g0 - lane);
            const double s = a + b;
            double m = gain_first(a, s);
            double e = 1.0;
            double lf = 0.0;
            double* grow = gain_table + (long long)lane * row;
            double* srow = surv_table + (long long)lane * row;
            for (int l = 0; l < row; ++l) {
                grow[l] = m;
                srow[l] = e;
                e = surv_next(e, b, s, lf);
                m = gain_next(m, b, s, lf);
                lf += 1.0;
            }
        }
        return;
    }
    const long long base = (long long)blockIdx.x * chunk;
    const long long end = base + chunk < n ? base + chunk : n;
    const bool vec_ok = (reinterpret_cast<uintptr_t>(c) & 15) == 0;
    int cnt = 0;
    bool bad = false;
    for (long long t0 = base; t0 < end; t0 += kTile) {
        const long long pos = t0 + (long long)threadIdx.x * kItems;
        int v[kItems];
        load_items_i32(c, pos, end, vec_ok, -1, v);
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            if (pos + j < end) {
                if (v[j] < 0 || v[j] > g0) { bad = true; v[j] = v[j] < 0 ? 0 : g0; }
            } else {
                v[j] = -1;
            }
        }
        for (int k = 0; k <= g0; ++k) {
            int pop = 0;
#pragma unroll
            for (int j = 0; j < kItems; ++j) pop += __popcll(__ballot(v[j] == k));
            if (lane == k) cnt += pop;
        }
    }
    s_cnt[wave_id()][lane] = cnt;
    __syncthreads();
    if (threadIdx.x <= (unsigned)g0) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < kBigWaves; ++w) tot += s_cnt[w][threadIdx.x];
        class_hist[(long long)threadIdx.x * kMaxBlocks + blockIdx.x] = tot;
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

// ----------------------------------------------------------------------------------
// CLASS solve, run by every workgroup of pass 2 on its own copy of the tables.
//
// Table entry (c, l) with value v is the threshold iff
//     count_gt(v) < budget <= count_gt(v) + count_eq(v),
// with count_gt(v) = sum_c' n_c' #{l' : M_c'(l') > v} and count_eq(v) the prompts whose
// next gain equals v.  Rows hold `len` gains followed by zeros up to the row length (a
// power of two), so each count is a branch-free binary search; four rows are searched
// in lockstep to overlap their LDS latencies.  The answer is only accepted when no
// populated class has all its `len` gains above v (unless the row ends at the cap):
// otherwise gains beyond the table would be missing from the counts, and the class-level
// greedy below decides instead.
// ----------------------------------------------------------------------------------
struct ClassSolution {      // LDS
    unsigned long long tau_bits;
    long long r;
    long long tie_prompts;
    int found;
    int win;                  // a table entry whose value is tau (pairs path)
    int k[kMaxClasses];
    int tied[kMaxClasses];
    double u0[kMaxClasses];   // U_c(k_c)
    double u1[kMaxClasses];   // U_c(k_c + 1)
};

// #{l : row[l] > v} for a decreasing row of `row_len` (power of two) entries whose last
// entry is not above v.
__device__ __forceinline__ int row_count_above(const double* row, int row_len, unsigned long long v) {
    int pos = 0;
    for (int step = row_len >> 1; step > 0; step >>= 1)
        if (gain_bits(row[pos + step - 1]) > v) pos += step;
    return pos;
}

__device__ void solve_by_table(int nc, int row_len, int len, bool rows_end_at_cap, long long budget,
                               const long long* s_n, const double* s_gain, const double* s_surv,
                               unsigned short* s_pair, ClassSolution* sol) {
    if (threadIdx.x == 0) sol->found = 0;
    __syncthreads();
    const int row_shift = __ffs(row_len) - 1;
    const int cands = nc * row_len;
    if (cands * nc <= kPairCap) {
        // Small tables: one thread per (entry, class) pair does one binary search, then one
        // thread per entry adds up its nc results.  Pair value: #{l' : M_class(l') > v} in
        // the low 15 bits, bit 15 set when the class's next gain equals v.
        for (int pair = (int)threadIdx.x; pair < cands * nc; pair += kBig) {
            const int idx = pair / nc, cls = pair - idx * nc;
            const unsigned long long v = gain_bits(s_gain[idx]);
            const double* row = s_gain + cls * row_len;
            const int pos = row_count_above(row, row_len, v);
            s_pair[pair] = (unsigned short)(pos | (gain_bits(row[pos]) == v ? 0x8000 : 0));
        }
        __syncthreads();
        for (int idx = (int)threadIdx.x; idx < cands; idx += kBig) {
            const int c = idx >> row_shift, l = idx & (row_len - 1);
            if (l >= len || s_n[c] == 0) continue;
            long long gt = 0, eq = 0;
            bool complete = true;
            for (int cls = 0; cls < nc; ++cls) {
                const int pr = s_pair[idx * nc + cls];
                const int pos = pr & 0x7fff;
                const long long n2 = s_n[cls];
                gt += n2 * pos;
                if (pr & 0x8000) eq += n2;
                if (n2 != 0 && pos >= len && !rows_end_at_cap) complete = false;
            }
            if (complete && gt < budget && budget <= gt + eq) {
                // every such thread writes the same values, except for `win`: entries of equal
                // value have equal pairs, so whichever lands serves
                sol->tau_bits = gain_bits(s_gain[idx]);
                sol->r = budget - gt;
                sol->tie_prompts = eq;
                sol->found = 1;
                sol->win = idx;
            }
        }
        __syncthreads();
        // the per-class results are at hand in the winning entry's pairs: one thread per class
        if (sol->found && threadIdx.x < (unsigned)nc) {
            const int cls = (int)threadIdx.x;
            const int pr = s_pair[sol->win * nc + cls];
            const int pos = pr & 0x7fff;
            sol->k[cls] = pos;
            sol->tied[cls] = (pr & 0x8000) ? 1 : 0;
            sol->u0[cls] = 1.0 - s_surv[cls * row_len + pos];
            sol->u1[cls] = 1.0 - s_surv[cls * row_len + (pos + 1 < row_len ? pos + 1 : pos)];
        }
        __syncthreads();
        return;
    } else
    for (int idx = (int)threadIdx.x; idx < cands; idx += kBig) {
        const int c = idx >> row_shift, l = idx & (row_len - 1);
        if (l >= len || s_n[c] == 0) continue;
        const unsigned long long v = gain_bits(s_gain[idx]);
        long long gt = 0, eq = 0;
        bool complete = true;
        for (int c0 = 0; c0 < nc; c0 += 4) {
            const double* rows[4];
            long long n2[4];
            int pos[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool in = c0 + i < nc;
                rows[i] = s_gain + (in ? c0 + i : 0) * row_len;
                n2[i] = in ? s_n[c0 + i] : 0;
                pos[i] = 0;
            }
            for (int step = row_len >> 1; step > 0; step >>= 1) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (gain_bits(rows[i][pos[i] + step - 1]) > v) pos[i] += step;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                gt += n2[i] * pos[i];
                if (gain_bits(rows[i][pos[i]]) == v) eq += n2[i];
                if (n2[i] != 0 && pos[i] >= len && !rows_end_at_cap) complete = false;
            }
        }
        if (complete && gt < budget && budget <= gt + eq) {   // every such thread writes the same values
            sol->tau_bits = v;
            sol->r = budget - gt;
            sol->tie_prompts = eq;
            sol->found = 1;
        }
    }
    __syncthreads();
    if (sol->found && threadIdx.x < (unsigned)nc) {
        const int c = (int)threadIdx.x;
        const double* row = s_gain + c * row_len;
        const int cnt = row_count_above(row, row_len, sol->tau_bits);
        sol->k[c] = cnt;
        sol->tied[c] = gain_bits(row[cnt]) == sol->tau_bits ? 1 : 0;
        sol->u0[c] = 1.0 - s_surv[c * row_len + cnt];
        sol->u1[c] = 1.0 - s_surv[c * row_len + (cnt + 1 < row_len ? cnt + 1 : cnt)];
    }
    __syncthreads();
}

// Class-level greedy, for allocations deeper than the table.  Lane c of wavefront 0 owns
// class c: its posterior, its position l_c and the current gain.  Each round takes the
// largest current gain over the classes that still have prompts and room below the cap;
// all classes tied at that value advance together, consuming n_c units each.  The round
// in which the remaining budget no longer covers the tied classes fixes tau.  This is
// Alg. 1's greedy loop run on classes: prompts of one class have identical sequences, so
// the greedy hands them their l-th unit in one uninterrupted run.
__device__ void solve_by_greedy(int g0, double alpha0, double beta0, long long cap_eff, bool depth_capped,
                                long long budget, const long long* s_n, ClassSolution* sol, int32_t* dev_status) {
    if (wave_id() == 0) {
        const int nc = g0 + 1;
        const int lane = lane_id();
        const bool has = lane < nc;
        const long long ncount = has ? s_n[lane] : 0;
        const double a = alpha0 + (double)(has ? lane : 0);
        const double b = beta0 + (double)(has ? g0 - lane : 0);
        const double s = a + b;
        double g = gain_first(a, s);
        double e = 1.0;
        double lf = 0.0;
        long long k = 0;
        long long remaining = budget;
        unsigned long long tau_bits = 0;
        long long tie_prompts = 0;
        bool tied = false;
        while (remaining > 0) {
            const bool active = has && ncount > 0 && k < cap_eff;
            const unsigned long long key = active ? gain_bits(g) : 0ull;
            unsigned long long best = 0;
            for (int j = 0; j < nc; ++j) {
                unsigned long long kj = read_lane_u64(key, j);
                best = kj > best ? kj : best;
            }
            if (best == 0) {  // nothing left to give to: cannot happen when budget <= n * cap
                report(dev_status, depth_capped ? HORA_ERR_UNSUPPORTED : HORA_ERR_INFEASIBLE);
                break;
            }
            const bool at_best = active && key == best;
            const unsigned long long mine = at_best ? (unsigned long long)ncount : 0ull;
            long long tsum = 0;
            for (int j = 0; j < nc; ++j) tsum += (long long)read_lane_u64(mine, j);
            tau_bits = best;
            if (tsum >= remaining) {  // the budget ends inside this round
                tied = at_best;
                tie_prompts = tsum;
                break;
            }
            remaining -= tsum;
            if (at_best) {
                e = surv_next(e, b, s, lf);
                g = gain_next(g, b, s, lf);
                lf += 1.0;
                k += 1;
                // a class stopped by the depth bound rather than by the caller's cap: the result
                // is no longer the optimum of the problem that was asked
                if (depth_capped && k >= cap_eff) report(dev_status, HORA_ERR_UNSUPPORTED);
            }
        }
        sol->k[lane] = has ? (int)k : 0;
        sol->tied[lane] = (has && tied) ? 1 : 0;
        sol->u0[lane] = 1.0 - e;
        sol->u1[lane] = 1.0 - surv_next(e, b, s, lf);
        if (lane == 0) {
            sol->tau_bits = tau_bits;
            sol->r = tie_prompts > 0 ? remaining : 0;
            sol->tie_prompts = tie_prompts;
            sol->found = 1;
        }
    }
    __syncthreads();
}

// Baseline rules the paper compares with (Sec. 5, Table 2 "hard-first"; the fixed-group
// baseline of Sec. 4), expressed in the terms of the tie pass: every eligible prompt gets
// `each` units and counts as tied, and the first `rest` of them by index get one more.
// rule 1: uniform, every prompt is eligible.  rule 2: hard-first, only prompts with
// c_i = 0 are; the split inside the eligible set is even (the paper does not say), and a
// batch without such a prompt falls back to uniform.
__device__ void solve_by_rule(int rule, int g0, double alpha0, double beta0, long long cap_eff, bool depth_capped,
                              long long budget, const long long* s_n, ClassSolution* sol, int32_t* dev_status) {
    if (wave_id() == 0) {
        const int nc = g0 + 1;
        const int lane = lane_id();
        const bool has = lane < nc;
        const long long ncount = has ? s_n[lane] : 0;
        long long total = 0;
        for (int j = 0; j < nc; ++j) total += (long long)read_lane_u64((unsigned long long)ncount, j);
        const long long hard = (long long)read_lane_u64((unsigned long long)ncount, 0);
        const bool all = rule == 1 || hard == 0;
        const long long eligible = all ? total : hard;
        long long each = eligible > 0 ? budget / eligible : 0;
        const long long rest = eligible > 0 ? budget - each * eligible : 0;
        if (each + (rest > 0 ? 1 : 0) > cap_eff) {   // uniform
            if (lane == 0) report(dev_status, depth_capped ? HORA_ERR_UNSUPPORTED : HORA_ERR_INFEASIBLE);
            each = cap_eff > 0 ? cap_eff - 1 : 0;    // (keeps the walk below within the depth bound)
        }
        const bool mine = has && (all || lane == 0);
        const long long k = mine ? each : 0;
        const double a = alpha0 + (double)(has ? lane : 0);
        const double b = beta0 + (double)(has ? g0 - lane : 0);
        const double s = a + b;
        double e = 1.0, lf = 0.0;
        for (long long l = 0; l < k; ++l) {
            e = surv_next(e, b, s, lf);
            lf += 1.0;
        }
        sol->k[lane] = (int)k;
        sol->tied[lane] = mine ? 1 : 0;
        sol->u0[lane] = 1.0 - e;
        sol->u1[lane] = 1.0 - surv_next(e, b, s, lf);
        if (lane == 0) {
            sol->tau_bits = 0ull;
            sol->r = rest;
            sol->tie_prompts = eligible;
            sol->found = 1;
        }
    }
    __syncthreads();
}

// ----------------------------------------------------------------------------------
// CLASS pass 2: solve (redundantly per workgroup), then write the workgroup's chunk.
// kOff: 0 no offsets, 1 int32 offsets, 2 int64 offsets.
// ----------------------------------------------------------------------------------
template <int kOff>
__global__ __launch_bounds__(kBig) void k_class_write(const int32_t* __restrict__ c, long long n, int g0,
                                                          double alpha0, double beta0, long long budget, int cap,
                                                          long long chunk, int nb, int row_len,
                                                          const int* __restrict__ class_hist,
                                                          const double* __restrict__ gain_table,
                                                          const double* __restrict__ surv_table,
                                                          int32_t* __restrict__ delta, double* __restrict__ util,
                                                          void* __restrict__ group_off,
                                                          hora_alloc_summary* __restrict__ summary,
                                                          int32_t* dev_status, int rule) {
    __shared__ double s_gain[kTableCap];
    __shared__ double s_surv[kTableCap];
    __shared__ long long s_part[2][kMaxClasses * kMaxBlocks / kWave];
    __shared__ long long s_n[kMaxClasses];       // prompts per class, whole batch
    __shared__ long long s_before[kMaxClasses];  // prompts per class in workgroups before this one
    __shared__ ClassSolution s_sol;
    __shared__ EmitShared s_emit;
    __shared__ unsigned short s_pair[kPairCap];

    const int nc = g0 + 1;
    const int lane = lane_id();
    const long long base = (long long)blockIdx.x * chunk;
    const long long end = base + chunk < n ? base + chunk : n;
    const bool c_vec = (reinterpret_cast<uintptr_t>(c) & 15) == 0;
    const bool d_vec = (reinterpret_cast<uintptr_t>(delta) & 15) == 0;
    const bool u_vec = (reinterpret_cast<uintptr_t>(util) & 15) == 0;
    const bool o_vec = (reinterpret_cast<uintptr_t>(group_off) & 15) == 0;
    // the caller's cap, and the library's own bound on the depth of one prompt
    const long long cap_user = cap > 0 ? (long long)cap : LLONG_MAX;
    const bool depth_capped = cap_user > (long long)HORA_MAX_DEPTH;
    const long long cap_eff = depth_capped ? (long long)HORA_MAX_DEPTH : cap_user;
    const int len = cap_eff < row_len - 1 ? (int)cap_eff : row_len - 1;   // usable gains per row
    const bool rows_end_at_cap = cap_eff <= row_len - 1;

    // Every global load of the prologue is issued before the first one is used (the
    // first tile of c, the two tables, the histogram): one round trip to memory instead
    // of one per stage.
    constexpr int kTableLoads = kTableCap / kBig;                   // table entries per thread
    constexpr int kHistLoads = kMaxClasses * kMaxBlocks / kBig;     // histogram entries per thread
    const int table_len = nc * row_len;
    const int entries = nc * kMaxBlocks;
    double tg[kTableLoads], ts[kTableLoads];
    int hh[kHistLoads];
#pragma unroll
    for (int q = 0; q < kTableLoads; ++q) {
        const int i = q * kBig + (int)threadIdx.x;
        tg[q] = i < table_len ? gain_table[i] : 0.0;
        ts[q] = i < table_len ? surv_table[i] : 0.0;
    }
#pragma unroll
    for (int q = 0; q < kHistLoads; ++q) {
        const int idx = q * kBig + (int)threadIdx.x;
        hh[q] = (idx < entries && (idx & (kMaxBlocks - 1)) < nb) ? class_hist[idx] : 0;
    }
    int first_tile[kItems];
    load_items_i32(c, base + (long long)threadIdx.x * kItems, end, c_vec, -1, first_tile);

    // tables into LDS, gains beyond `len` replaced by zeros
#pragma unroll
    for (int q = 0; q < kTableLoads; ++q) {
        const int i = q * kBig + (int)threadIdx.x;
        if (i < table_len) {
            s_gain[i] = (i & (row_len - 1)) < len ? tg[q] : 0.0;
            s_surv[i] = ts[q];
        }
    }

    // class totals and the part that lies before this workgroup: the counts of class c
    // are kMaxBlocks consecutive entries, so every wavefront sums entries of one class
#pragma unroll
    for (int q = 0; q < kHistLoads; ++q) {
        const int i0 = q * kBig;
        if (i0 < entries) {   // uniform
            const int idx = i0 + (int)threadIdx.x;
            const int b = idx & (kMaxBlocks - 1);
            const long long tot_w = wave_total_i64((long long)hh[q]);
            const long long bef_w = wave_total_i64(b < (int)blockIdx.x ? (long long)hh[q] : 0ll);
            if (lane == 0 && idx < entries) { s_part[0][idx >> 6] = tot_w; s_part[1][idx >> 6] = bef_w; }
        }
    }
    __syncthreads();
    if (threadIdx.x < (unsigned)nc) {
        constexpr int kSlots = kMaxBlocks / kWave;
        long long tot = 0, bef = 0;
#pragma unroll
        for (int q = 0; q < kSlots; ++q) {
            tot += s_part[0][threadIdx.x * kSlots + q];
            bef += s_part[1][threadIdx.x * kSlots + q];
        }
        s_n[threadIdx.x] = tot;
        s_before[threadIdx.x] = bef;
    }
    __syncthreads();

    if (budget > 0 && rule != 0) {
        solve_by_rule(rule, g0, alpha0, beta0, cap_eff, depth_capped, budget, s_n, &s_sol, dev_status);
    } else if (budget > 0) {
        solve_by_table(nc, row_len, len, rows_end_at_cap, budget, s_n, s_gain, s_surv, s_pair, &s_sol);
        if (!s_sol.found)
            solve_by_greedy(g0, alpha0, beta0, cap_eff, depth_capped, budget, s_n, &s_sol, dev_status);
    } else {
        if (threadIdx.x < kMaxClasses) {
            s_sol.k[threadIdx.x] = 0;
            s_sol.tied[threadIdx.x] = 0;
            s_sol.u0[threadIdx.x] = 0.0;
            s_sol.u1[threadIdx.x] = 0.0;
        }
        if (threadIdx.x == 0) { s_sol.tau_bits = 0; s_sol.r = 0; s_sol.tie_prompts = 0; s_sol.found = 1; }
        __syncthreads();
    }
    const long long r = s_sol.r;
    if (summary && blockIdx.x == 0 && threadIdx.x == 0) {
        summary->tau = __longlong_as_double((long long)s_sol.tau_bits);
        summary->count_gt = budget - r;
        summary->tie_units = r;
        summary->tie_prompts = s_sol.tie_prompts;
    }

    // what the workgroups before this one hold: lane c takes class c, the wavefront adds up
    long long tied_before = 0, units_before = 0;
    if (lane < nc) {
        const long long bef = s_before[lane];
        tied_before = s_sol.tied[lane] ? bef : 0;
        units_before = bef * s_sol.k[lane];
    }
    EmitCarry carry = {wave_total_i64(tied_before), wave_total_i64(units_before)};

    int parity = 0;
    for (long long t0 = base; t0 < end; t0 += kTile, parity ^= 1) {
        const long long pos = t0 + (long long)threadIdx.x * kItems;
        int cls[kItems], kk[kItems], td[kItems], dd[kItems];
        bool win[kItems];
        if (t0 == base) {
#pragma unroll
            for (int j = 0; j < kItems; ++j) cls[j] = first_tile[j];
        } else {
            load_items_i32(c, pos, end, c_vec, -1, cls);
        }
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            if (pos + j < end) {
                const int x = cls[j] < 0 ? 0 : (cls[j] > g0 ? g0 : cls[j]);
                cls[j] = x;
                kk[j] = s_sol.k[x];
                td[j] = s_sol.tied[x];
            } else {
                cls[j] = 0; kk[j] = 0; td[j] = 0;
            }
        }
        emit_tile<kOff>(parity, pos, end, n, g0, r, kk, td, carry, dd, win, delta, group_off, d_vec, o_vec,
                        &s_emit);
        if (util) {
            double uu[kItems];
#pragma unroll
            for (int j = 0; j < kItems; ++j) uu[j] = win[j] ? s_sol.u1[cls[j]] : s_sol.u0[cls[j]];
            store_items<v2d, double>(util, pos, end, u_vec, uu);
        }
    }
}

// ----------------------------------------------------------------------------------
// BISECT pass 0: the largest gain hi = max_i M_i(0), gathered with integer atomicMax (few
// workgroups: atomics on one address serialise).
// ----------------------------------------------------------------------------------
template <class Src>
__global__ __launch_bounds__(kBig) void k_select_top(Src src, long long n, AllocHeader* __restrict__ hdr,
                                                     int32_t* dev_status) {
    __shared__ unsigned long long s_red[kBigWaves];
    unsigned long long hi = 0;
    bool bad = false;
    const long long stride = (long long)gridDim.x * kBig;
    for (long long i = (long long)blockIdx.x * kBig + threadIdx.x; i < n; i += stride) {
        double a, b;
        bad |= !src.load(i, a, b);
        const unsigned long long gb = gain_bits(gain_first(a, a + b));
        hi = gb > hi ? gb : hi;
    }
    hi = wave_max_u64(hi);
    if (lane_id() == 0) s_red[wave_id()] = hi;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long block_hi = 0;
        for (int i = 0; i < kBigWaves; ++i) block_hi = s_red[i] > block_hi ? s_red[i] : block_hi;
        atomicMax(&hdr->hi, block_hi);   // the first search pass turns it into the first window
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}

// ----------------------------------------------------------------------------------
// BISECT search pass.  Invariant: exactly `above` pairs have a gain > hi_cur, and
// above < budget.  The bracket (lo, hi] is cut into at most kBins intervals of 2^shift bit
// patterns.  Every prompt walks its gains from l = 0 down to lo (a monotone search) and
// the gains inside the bracket are tallied per interval, together with the largest and the
// smallest pattern seen there.  If the running count from the top interval down reaches
// the budget in interval j, the bracket shrinks to the gains that actually occur there,
// (min - 1, max], and closes when min == max (tau is that gain): each such pass cuts the
// bracket at least 128-fold; with real-valued posteriors it keeps ~1/256 of the gains of
// the pass before, with a shared prior (few distinct gains, each repeated) it closes in
// two passes.  Otherwise the whole window lies above tau: its count is added to `above`
// and the next window, a factor 16 further down in value (4 exponent steps of the bit
// pattern), is taken.  Searching window by window from the top keeps the walks short: a
// window's count is a small multiple of the one before, so the work stays a small
// multiple of the budget, whereas a bracket from a guaranteed lower bound (such as the
// smallest ceil(budget/n)-th gain) can lie orders of magnitude below tau and make every
// prompt walk thousands of steps.
//
// kSolo = false: every workgroup tallies its share into a slot of its own; k_select_reduce
// adds the slots up, and every workgroup of the next pass moves the bracket by those
// totals for itself (the same arithmetic on the same numbers in every workgroup), which
// takes a few microseconds less than a one-workgroup kernel in between that has to pull
// all slots through one compute unit.  The bracket is kept twice: pass p reads slot
// p & 1, which nobody writes meanwhile, and its first workgroup stores the moved bracket
// in the other slot for pass p + 1.
// kSolo = true: one workgroup repeats passes over all prompts until the bracket closes.
// It runs after the grid-wide passes and normally finds the bracket closed already; it is
// there so that a fixed, small number of launches is correct for any input.
// ----------------------------------------------------------------------------------
struct SelectShared {
    unsigned long long cnt[kBins];
    unsigned long long vmax[kBins];
    unsigned long long vmin_inv[kBins];
    long long red[kBigWaves];
    unsigned long long lo, hi;
    long long above;
    long long inside;   // pairs in the bracket after a step that narrowed it (-1: not known)
    int done;
    int hit;            // the last step narrowed the bracket (it did not move to the next window)
    int list_n;         // gains this workgroup has set aside in this pass
};

// The step that ends a search pass, run by a whole workgroup: thread t < kBins holds the
// tally (cj, mx, mn) of interval kBins - 1 - t (thread 0 the top one), the other threads
// zeros.  Finds the interval in which the running count from the top reaches the budget
// and shrinks the bracket to the gains seen there, or, when the whole window lies above
// tau, takes the next window.
__device__ __forceinline__ void move_bracket(SelectShared& sh, unsigned long long cj, unsigned long long mx,
                                             unsigned long long mn, long long budget) {
    const unsigned long long lo = sh.lo;
    const long long start = sh.above;   // pairs above the bracket
    if (cj > (unsigned long long)budget) cj = (unsigned long long)budget;
    __syncthreads();                                     // sh.red is free, the bracket has been read
    // pairs in higher intervals: exclusive prefix over the threads
    const long long incl = wave_incl_scan<long long>((long long)cj);
    if (lane_id() == kWave - 1) sh.red[wave_id()] = incl;
    __syncthreads();
    long long before = start + incl - (long long)cj;
    long long total = 0;
    for (int i = 0; i < kBigWaves; ++i) {
        if (i < wave_id()) before += sh.red[i];
        total += sh.red[i];
    }
    if (start + total < budget) {                       // uniform: the whole window is above tau
        if (threadIdx.x == 0) {
            sh.above = start + total;
            sh.hi = lo;
            sh.lo = lo > kWindowStep ? lo - kWindowStep : 0ull;
            if (lo == 0ull) sh.done = 2;                // no gains left: the budget does not fit
            sh.hit = 0;
            sh.inside = -1;
        }
    } else if (cj != 0 && before < budget && budget <= before + (long long)cj) {   // exactly one thread
        sh.above = before;
        sh.hi = mx;
        sh.lo = mn - 1ull;
        sh.done = (mx == mn) ? 1 : 0;
        sh.hit = 1;
        sh.inside = (long long)cj;                      // (a count cut off at the budget is no larger than the true one)
    }
    __syncthreads();
}

template <class Src, bool kSolo>
__global__ __launch_bounds__(kBig) void k_select_pass(Src src, long long n, long long budget, long long limit,
                                                      int pass, AllocHeader* __restrict__ hdr,
                                                      SelectBins* __restrict__ bins,
                                                      unsigned long long* __restrict__ lists,
                                                      int* __restrict__ list_count) {
    __shared__ SelectShared sh;
    // the bracket this pass works on: the stored one, moved by the totals of the pass before
    const Bracket* in = &hdr->slot[pass & 1];
    const bool pending = pass > 0 && (in->flags & kFlagPending) != 0 && in->done == 0;   // uniform
    {
        const SelectBins* totals = bins + kMaxBlocks;
        const int j = kBins - 1 - (int)threadIdx.x;   // thread 0 owns the top interval
        unsigned long long cj = 0, mx = 0, mn = 0;
        if (pending && threadIdx.x < kBins) {
            cj = totals->cnt[j];
            mx = totals->vmax[j];
            mn = ~totals->vmin_inv[j];
        }
        if (threadIdx.x == 0) {
            if (pass == 0) {   // the first window, from the largest gain down
                const unsigned long long all_hi = hdr->hi;
                sh.hi = all_hi;
                sh.lo = all_hi > kWindowStep ? all_hi - kWindowStep : 0ull;
                sh.above = 0;
                sh.done = 0;
            } else {
                sh.lo = in->lo; sh.hi = in->hi; sh.above = (long long)in->above; sh.done = (int)in->done;
            }
            sh.hit = 0;
            sh.inside = -1;
            sh.list_n = 0;
        }
        __syncthreads();
        if (pending) move_bracket(sh, cj, mx, mn, budget);
    }
    // Where this pass gets the gains of its bracket from.  A bracket that has been narrowed
    // to few pairs is set aside while it is walked once more (kCollect: every workgroup
    // keeps the gains it finds in a list of its own); the passes after that tally from the
    // lists instead of walking every prompt again (kFromLists) -- brackets only shrink
    // from there on, so the lists stay a superset of what is needed.  A list that does not
    // fit (lists_ok == 0) only means that the next pass walks again.
    enum { kWalk = 0, kCollect = 1, kFromLists = 2 };
    int mode = kWalk;
    if (!kSolo && pending && sh.hit && !sh.done) {
        if ((in->flags & kFlagCollected) != 0 && hdr->lists_ok != 0) mode = kFromLists;
        else if (sh.inside <= kCollectMax) mode = kCollect;
    }
    if (!kSolo && blockIdx.x == 0 && threadIdx.x == 0) {   // for the next pass
        Bracket* out = &hdr->slot[(pass + 1) & 1];
        out->lo = sh.lo; out->hi = sh.hi; out->above = (unsigned long long)sh.above;
        out->done = (unsigned)sh.done;
        // this pass tallies unless the search has ended
        out->flags = (sh.done ? 0u : kFlagPending) | (mode != kWalk ? kFlagCollected : 0u);
    }
    const int iters = kSolo ? kSoloMaxPasses : 1;
    for (int iter = 0; iter < iters; ++iter) {
        if (sh.done) break;
        const unsigned long long lo = sh.lo, hi = sh.hi;
        const unsigned long long width = hi - lo;                  // >= 1
        const int bitlen = width > 1 ? 64 - __clzll((long long)(width - 1)) : 0;   // bits of width - 1
        const int shift = bitlen > 8 ? bitlen - 8 : 0;             // (width - 1) >> shift < kBins
        if (threadIdx.x < kBins) { sh.cnt[threadIdx.x] = 0; sh.vmax[threadIdx.x] = 0; sh.vmin_inv[threadIdx.x] = 0; }
        __syncthreads();

        const long long stride = (long long)gridDim.x * kBig;
        const int lane = lane_id();
        if (mode == kFromLists) {   // (never in the solo kernel)
            const int have = list_count[blockIdx.x];
            const unsigned long long* mine = lists + (long long)blockIdx.x * kListCap;
            for (int e = (int)threadIdx.x; e < have; e += kBig) {
                const unsigned long long v = mine[e];
                if (v > lo && v <= hi) {
                    const int j = (int)((v - lo - 1ull) >> shift);
                    atomicAdd(&sh.cnt[j], 1ull);
                    atomicMax(&sh.vmax[j], v);
                    atomicMax(&sh.vmin_inv[j], ~v);
                }
            }
        } else
        // all wavefronts run the same number of rounds, so that the ballots below see whole wavefronts
        for (long long i0 = (long long)blockIdx.x * kBig; i0 < n; i0 += stride) {
            const long long i = i0 + threadIdx.x;
            double a = 1.0, b = 1.0;
            if (i < n) src.load(i, a, b);
            const double s = a + b;
            double g = gain_first(a, s);
            double lf = 0.0;
            long long k = 0;
            unsigned long long gb = gain_bits(g);
            bool active = i < n && k < limit && gb > lo;
            while (__ballot(active)) {
                const bool inside = active && gb <= hi;
                if (mode == kCollect && inside) {
                    const int at = atomicAdd(&sh.list_n, 1);
                    if (at < kListCap) lists[(long long)blockIdx.x * kListCap + at] = gb;
                }
                // lanes that hold the same gain (common under a shared prior) tally once:
                // up to 8 distinct gains per step through a leader, the rest lane by lane
                unsigned long long pending = __ballot(inside);
                for (int round = 0; round < 8 && pending; ++round) {
                    const int leader = __ffsll((long long)pending) - 1;
                    const unsigned long long v = read_lane_u64(gb, leader);
                    const unsigned long long same = __ballot(inside && gb == v);
                    // gains that do not repeat (per-prompt posteriors): no point in more rounds
                    if (round == 0 && same == (1ull << leader)) break;
                    if (lane == leader) {
                        const int j = (int)((v - lo - 1ull) >> shift);
                        // no result is used: the three updates are issued without a wait
                        atomicAdd(&sh.cnt[j], (unsigned long long)__popcll(same));
                        atomicMax(&sh.vmax[j], v);
                        atomicMax(&sh.vmin_inv[j], ~v);
                    }
                    pending &= ~same;
                }
                if (inside && ((pending >> lane) & 1ull)) {
                    const int j = (int)((gb - lo - 1ull) >> shift);
                    atomicAdd(&sh.cnt[j], 1ull);
                    atomicMax(&sh.vmax[j], gb);
                    atomicMax(&sh.vmin_inv[j], ~gb);
                }
                if (active) {
                    g = gain_next(g, b, s, lf);
                    lf += 1.0;
                    k += 1;
                    gb = gain_bits(g);
                    active = k < limit && gb > lo;
                }
            }
        }
        __syncthreads();   // the workgroup's tallies are complete
        if (!kSolo) {
            // this workgroup's tallies to its own slot (all of them: the slot holds no state);
            // k_select_reduce adds the slots up after this kernel has ended
            if (mode == kCollect && threadIdx.x == 0) list_count[blockIdx.x] = sh.list_n <= kListCap ? sh.list_n : -1;
            SelectBins* mine = bins + blockIdx.x;
            if (threadIdx.x < kBins) {
                const unsigned long long c0 = sh.cnt[threadIdx.x];
                mine->cnt[threadIdx.x] = c0 > (unsigned long long)budget ? (unsigned long long)budget : c0;
                mine->vmax[threadIdx.x] = sh.vmax[threadIdx.x];
                mine->vmin_inv[threadIdx.x] = sh.vmin_inv[threadIdx.x];
            }
            return;
        }
        // tallies of interval j = kBins - 1 - thread: thread 0 owns the top interval
        const int j = kBins - 1 - (int)threadIdx.x;
        unsigned long long cj = 0, mx = 0, mn = 0;
        if (threadIdx.x < kBins) {
            cj = sh.cnt[j];
            mx = sh.vmax[j];
            mn = ~sh.vmin_inv[j];
        }
        move_bracket(sh, cj, mx, mn, budget);
    }
    if (kSolo && threadIdx.x == 0) hdr->hi_cur = sh.hi;   // tau
}

// ----------------------------------------------------------------------------------
// Between two grid-wide search passes: the interval tallies of the workgroups are added up
// (counts) and combined (largest, smallest gain) into bins[kMaxBlocks].  kReduceBins
// intervals per workgroup, 32 lanes per interval striding over the slots.  A kernel of its
// own rather than "the workgroup that finishes last": the device-wide fences that pattern
// needs (write back and invalidate the L2 of every die) cost several times the pass itself
// on this part.
// ----------------------------------------------------------------------------------
constexpr int kReduceBins = kThreads / 32;   // 8 intervals per workgroup of 256 threads

__global__ __launch_bounds__(kThreads) void k_select_reduce(int nb, int pass, AllocHeader* __restrict__ hdr,
                                                            SelectBins* __restrict__ bins,
                                                            const int* __restrict__ list_count) {
    const unsigned flags = hdr->slot[(pass + 1) & 1].flags;
    if ((flags & kFlagPending) == 0) return;   // pass `pass` did not tally: the search has ended
    if (blockIdx.x == 0 && (flags & kFlagCollected) != 0) {   // did every workgroup's list fit?
        static_assert(kMaxBlocks <= kThreads, "one thread per list");
        const int any_bad = __syncthreads_or((int)threadIdx.x < nb && list_count[threadIdx.x] < 0 ? 1 : 0);
        if (threadIdx.x == 0) hdr->lists_ok = any_bad ? 0u : 1u;
    }
    const int bin = (int)blockIdx.x * kReduceBins + (int)threadIdx.x / 32;
    const int sub = (int)threadIdx.x & 31;
    unsigned long long c = 0, mx = 0, mn = 0;
    constexpr int kPer = kMaxBlocks / 32;                 // slots per lane, all loads issued at once
    unsigned long long pc[kPer], pm[kPer], pn[kPer];
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
        const int wg = sub + 32 * t;
        const bool in = wg < nb;
        pc[t] = in ? bins[wg].cnt[bin] : 0ull;
        pm[t] = in ? bins[wg].vmax[bin] : 0ull;
        pn[t] = in ? bins[wg].vmin_inv[bin] : 0ull;
    }
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
        c += pc[t];
        mx = pm[t] > mx ? pm[t] : mx;
        mn = pn[t] > mn ? pn[t] : mn;
    }
#pragma unroll
    for (int d = 16; d > 0; d >>= 1) {
        c += (unsigned long long)__shfl_xor((long long)c, d, 32);
        const unsigned long long om = (unsigned long long)__shfl_xor((long long)mx, d, 32);
        const unsigned long long on = (unsigned long long)__shfl_xor((long long)mn, d, 32);
        mx = om > mx ? om : mx;
        mn = on > mn ? on : mn;
    }
    if (sub == 0) {
        SelectBins* totals = bins + kMaxBlocks;
        totals->cnt[bin] = c;
        totals->vmax[bin] = mx;
        totals->vmin_inv[bin] = mn;
    }
}

// ----------------------------------------------------------------------------------
// BISECT finalize: with tau = hi_cur, k_i = #{l : M_i(l) > tau} and the tied flag go
// to delta[i] (flag in bit 31), the survival product E_i(k_i) to util[i]; per-workgroup
// sums go to block_ksum / block_tied.
// ----------------------------------------------------------------------------------
template <class Src>
__global__ __launch_bounds__(kBig) void k_bisect_finalize(Src src, long long n, long long chunk, long long budget,
                                                          long long limit, const AllocHeader* __restrict__ hdr,
                                                          int32_t* __restrict__ delta, double* __restrict__ util,
                                                          long long* __restrict__ block_ksum,
                                                          long long* __restrict__ block_tied) {
    __shared__ long long s_red[2][kBigWaves];
    const unsigned long long tau_bits = budget > 0 ? hdr->hi_cur : ~0ull;
    const long long base = (long long)blockIdx.x * chunk;
    const long long end = base + chunk < n ? base + chunk : n;
    long long ks = 0, ts = 0;
    for (long long i = base + threadIdx.x; i < end; i += kBig) {
        double a, b, g, lf, e;
        src.load(i, a, b);
        const long long k = walk_above<true>(a, b, tau_bits, limit, g, lf, e);
        const bool tied = (k < limit) && (gain_bits(g) == tau_bits);
        delta[i] = (int32_t)((unsigned)k | (tied ? kTiedBit : 0u));
        if (util) util[i] = e;
        ks += k;
        ts += tied ? 1 : 0;
    }
    ks = wave_total_i64(ks);
    ts = wave_total_i64(ts);
    if (lane_id() == 0) { s_red[0][wave_id()] = ks; s_red[1][wave_id()] = ts; }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long ksum = 0, tsum = 0;
        for (int i = 0; i < kBigWaves; ++i) { ksum += s_red[0][i]; tsum += s_red[1][i]; }
        block_ksum[blockIdx.x] = ksum;
        block_tied[blockIdx.x] = tsum;
    }
}

// BISECT scan (one workgroup): exclusive prefixes over the workgroups, r, the report,
// and the header back to its rest state.
__global__ __launch_bounds__(kThreads) void k_bisect_scan(int nb, long long budget, AllocHeader* __restrict__ hdr,
                                                          BisectSolution* __restrict__ sol,
                                                          long long* __restrict__ block_ksum,
                                                          long long* __restrict__ block_tied,
                                                          hora_alloc_summary* __restrict__ summary,
                                                          int32_t* dev_status) {
    __shared__ long long s_scan[kWaves];
    long long kcarry = 0, tcarry = 0;
    for (int b0 = 0; b0 < nb; b0 += kThreads) {
        const int b = b0 + (int)threadIdx.x;
        const long long kv = b < nb ? block_ksum[b] : 0;
        const long long tv = b < nb ? block_tied[b] : 0;
        long long ktot, ttot;
        const long long kex = block_excl_scan<long long>(kv, s_scan, ktot);
        const long long tex = block_excl_scan<long long>(tv, s_scan, ttot);
        if (b < nb) {
            block_ksum[b] = kcarry + kex;
            block_tied[b] = tcarry + tex;
        }
        kcarry += ktot;
        tcarry += ttot;
    }
    if (threadIdx.x == 0) {
        const long long r = budget - kcarry;
        if (r < 0 || r > tcarry) report(dev_status, HORA_ERR_RANGE);  // invalid posteriors upstream
        sol->r = r;
        if (summary) {
            summary->tau = budget > 0 ? __longlong_as_double((long long)hdr->hi_cur) : 0.0;
            summary->count_gt = kcarry;
            summary->tie_units = r;
            summary->tie_prompts = tcarry;
        }
        hdr->hi = 0ull;
        hdr->hi_cur = 0ull;
        for (int i = 0; i < 2; ++i) {
            hdr->slot[i].lo = 0ull; hdr->slot[i].hi = 0ull; hdr->slot[i].above = 0ull;
            hdr->slot[i].done = 0u; hdr->slot[i].flags = 0u;
        }
        hdr->lists_ok = 0u;
    }
}

// BISECT write: delta[i] holds k_i with the tied flag in bit 31 and util[i] the survival
// product E_i(k_i); a winner's utility takes one more step of the product.
template <class Src, int kOff>
__global__ __launch_bounds__(kBig) void k_bisect_write(Src src, long long n, int g0, long long chunk,
                                                           const BisectSolution* __restrict__ sol,
                                                           const long long* __restrict__ block_ksum,
                                                           const long long* __restrict__ block_tied,
                                                           int32_t* __restrict__ delta, double* __restrict__ util,
                                                           void* __restrict__ group_off) {
    __shared__ EmitShared s_emit;
    const long long r = sol->r;
    const long long base = (long long)blockIdx.x * chunk;
    const long long end = base + chunk < n ? base + chunk : n;
    const bool d_vec = (reinterpret_cast<uintptr_t>(delta) & 15) == 0;
    const bool u_vec = (reinterpret_cast<uintptr_t>(util) & 15) == 0;
    const bool o_vec = (reinterpret_cast<uintptr_t>(group_off) & 15) == 0;
    EmitCarry carry = {block_tied[blockIdx.x], block_ksum[blockIdx.x]};
    int parity = 0;
    for (long long t0 = base; t0 < end; t0 += kTile, parity ^= 1) {
        const long long pos = t0 + (long long)threadIdx.x * kItems;
        int raw[kItems];
        load_items_i32(delta, pos, end, d_vec, 0, raw);
        int kk[kItems], td[kItems], dd[kItems];
        bool win[kItems];
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            kk[j] = (int)((unsigned)raw[j] & ~kTiedBit);
            td[j] = ((unsigned)raw[j] & kTiedBit) ? 1 : 0;
        }
        emit_tile<kOff>(parity, pos, end, n, g0, r, kk, td, carry, dd, win, delta, group_off, d_vec, o_vec,
                        &s_emit);
        if (util) {
            double uu[kItems];
#pragma unroll
            for (int j = 0; j < kItems; ++j) {
                double e = 1.0;
                if (pos + j < end) {
                    e = util[pos + j];
                    if (win[j]) {
                        double a, b;
                        src.load(pos + j, a, b);
                        e = surv_next(e, b, a + b, (double)kk[j]);
                    }
                }
                uu[j] = 1.0 - e;
            }
            store_items<v2d, double>(util, pos, end, u_vec, uu);
        }
    }
}

template <typename T>
__global__ void k_store_one(T* p, T v) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *p = v;
}

__global__ void k_zero_summary(hora_alloc_summary* s) {
    if (blockIdx.x == 0 && threadIdx.x == 0) { s->tau = 0.0; s->count_gt = 0; s->tie_units = 0; s->tie_prompts = 0; }
}

// ----------------------------------------------------------------------------------
// Host side
// ----------------------------------------------------------------------------------
static int check_launch() { return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP; }

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

static int validate_common(const CommonArgs& a) {
    if (a.n < 0 || a.g0 < 0 || a.budget < 0) return HORA_ERR_INVALID_ARG;
    if (!a.dev_status) return HORA_ERR_INVALID_ARG;
    if (a.n > 0 && !a.delta) return HORA_ERR_INVALID_ARG;
    if (a.group_off && a.off_t != HORA_I32 && a.off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (a.budget >= (1ll << 52)) return HORA_ERR_UNSUPPORTED;
    if (a.n >= (1ll << 40)) return HORA_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(a.delta) & 3) || (reinterpret_cast<uintptr_t>(a.util) & 7) ||
        (reinterpret_cast<uintptr_t>(a.dev_status) & 3))
        return HORA_ERR_INVALID_ARG;
    if (a.group_off) {
        const uintptr_t mask = a.off_t == HORA_I32 ? 3 : 7;
        if (reinterpret_cast<uintptr_t>(a.group_off) & mask) return HORA_ERR_INVALID_ARG;
    }
    if (a.budget > 0 && a.n == 0) return HORA_ERR_INFEASIBLE;
    if (a.delta_max > 0 && a.budget > 0 && (a.budget + a.delta_max - 1) / a.delta_max > a.n)
        return HORA_ERR_INFEASIBLE;
    // more than n * HORA_MAX_DEPTH units: some prompt would have to go deeper than the bound
    // (n < 2^40 and the bound is 2^20, so the product fits)
    if (a.n > 0 && a.budget > a.n * (long long)HORA_MAX_DEPTH) return HORA_ERR_UNSUPPORTED;
    if (a.group_off && a.off_t == HORA_I32) {
        const long long total = a.n * (long long)a.g0 + a.budget;
        if (total >= (1ll << 31)) return HORA_ERR_INVALID_ARG;
    }
    return HORA_OK;
}

static int handle_empty(const CommonArgs& a) {  // n == 0 (budget == 0 checked before)
    if (a.group_off) {
        if (a.off_t == HORA_I32) hipLaunchKernelGGL(k_store_one<int32_t>, 1, 1, 0, a.stream, (int32_t*)a.group_off, 0);
        else hipLaunchKernelGGL(k_store_one<long long>, 1, 1, 0, a.stream, (long long*)a.group_off, 0ll);
    }
    if (a.summary) hipLaunchKernelGGL(k_zero_summary, 1, 1, 0, a.stream, a.summary);
    return check_launch();
}

// Row length of the gain table (a power of two; the last entry is padding): long enough
// for a few times the mean allocation, within what fits the table.  The class-level
// greedy covers whatever is deeper.
static int table_row(int nc, int64_t n, int64_t budget, int32_t delta_max) {
    int fit = kMinRow;
    while (fit * 2 * nc <= kTableCap && fit * 2 <= kMaxRow) fit *= 2;
    const long long mean = (budget + n - 1) / n;
    long long need = 4 * mean + 1;
    if (delta_max > 0 && need > (long long)delta_max + 1) need = (long long)delta_max + 1;
    int row = kMinRow;
    while (row < need && row < fit) row *= 2;
    return row;
}

static int run_class(const int32_t* c, double alpha0, double beta0, const CommonArgs& a, const Plan& p,
                     const Workspace& w, int rule) {
    const int nc = a.g0 + 1;
    const int row = table_row(nc, a.n, a.budget, a.delta_max);
    const int cap = a.delta_max > 0 ? a.delta_max : 0;
    hipLaunchKernelGGL(k_class_hist, dim3(p.nb + 1), dim3(kBig), 0, a.stream, c, (long long)a.n, (int)a.g0,
                       alpha0, beta0, p.chunk, p.nb, row, w.class_hist, w.gain_table, w.surv_table,
                       a.dev_status);
    const int mode = a.group_off ? (a.off_t == HORA_I32 ? 1 : 2) : 0;
#define HORA_LAUNCH_CLASS_WRITE(M)                                                                              \
    hipLaunchKernelGGL((k_class_write<M>), dim3(p.nb), dim3(kBig), 0, a.stream, c, (long long)a.n,          \
                       (int)a.g0, alpha0, beta0, (long long)a.budget, cap, p.chunk, p.nb, row, w.class_hist,   \
                       w.gain_table, w.surv_table, a.delta, a.util, a.group_off, a.summary, a.dev_status, rule)
    if (mode == 0) HORA_LAUNCH_CLASS_WRITE(0);
    else if (mode == 1) HORA_LAUNCH_CLASS_WRITE(1);
    else HORA_LAUNCH_CLASS_WRITE(2);
#undef HORA_LAUNCH_CLASS_WRITE
    return check_launch();
}

static int run_small(const CountsSource& src, const CommonArgs& a) {
    return allocate_small_counts(src, a.n, a.g0, a.budget, a.delta_max, a.delta, a.util, a.group_off, a.off_t,
                                 a.summary, a.dev_status, a.stream);
}
static int run_small(const PosteriorSource& src, const CommonArgs& a) {
    return allocate_small_posterior(src, a.n, a.g0, a.budget, a.delta_max, a.delta, a.util, a.group_off, a.off_t,
                                    a.summary, a.dev_status, a.stream);
}

template <class Src>
static int run_bisect(const Src& src, const CommonArgs& a, const Plan& p, const Workspace& w) {
    const long long n = a.n;
    // a batch that one workgroup can hold: one launch does the whole search and the outputs
    if (n <= kSoloMaxPrompts) return run_small(src, a);
    long long limit = a.delta_max > 0 ? (long long)a.delta_max : a.budget;
    if (limit > a.budget) limit = a.budget;
    if (a.budget > 0) {
        long long blocks = (n + kBig - 1) / kBig;
        if (blocks > kMaxBlocks) blocks = kMaxBlocks;
        hipLaunchKernelGGL((k_select_top<Src>), dim3((unsigned)blocks), dim3(kBig), 0, a.stream, src, n, w.header,
                           a.dev_status);
        for (int pass = 0; pass < kParallelPasses; ++pass) {
            hipLaunchKernelGGL((k_select_pass<Src, false>), dim3((unsigned)blocks), dim3(kBig), 0, a.stream, src,
                               n, (long long)a.budget, limit, pass, w.header, w.bins, w.lists, w.list_count);
            hipLaunchKernelGGL(k_select_reduce, dim3(kBins / kReduceBins), dim3(kThreads), 0, a.stream, (int)blocks,
                               pass, w.header, w.bins, (const int*)w.list_count);
        }
        hipLaunchKernelGGL((k_select_pass<Src, true>), dim3(1), dim3(kBig), 0, a.stream, src, n,
                           (long long)a.budget, limit, kParallelPasses, w.header, w.bins, w.lists, w.list_count);
    }
    hipLaunchKernelGGL((k_bisect_finalize<Src>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, p.chunk,
                       (long long)a.budget, limit, w.header, a.delta, a.util, w.block_ksum, w.block_tied);
    hipLaunchKernelGGL(k_bisect_scan, dim3(1), dim3(kThreads), 0, a.stream, p.nb, (long long)a.budget, w.header,
                       w.sol, w.block_ksum, w.block_tied, a.summary, a.dev_status);
    const int mode = a.group_off ? (a.off_t == HORA_I32 ? 1 : 2) : 0;
#define HORA_LAUNCH_BISECT_WRITE(M)                                                                      \
    hipLaunchKernelGGL((k_bisect_write<Src, M>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, (int)a.g0, \
                       p.chunk, w.sol, w.block_ksum, w.block_tied, a.delta, a.util, a.group_off)
    if (mode == 0) HORA_LAUNCH_BISECT_WRITE(0);
    else if (mode == 1) HORA_LAUNCH_BISECT_WRITE(1);
    else HORA_LAUNCH_BISECT_WRITE(2);
#undef HORA_LAUNCH_BISECT_WRITE
    return check_launch();
}

// ----------------------------------------------------------------------------------
// Workspace for callers that cannot allocate (hora_allocate_static): a file-scope device
// array, one copy per GPU, held until the process ends.  Its name is a host-side stand-in
// for the symbol, not a device address; the address on the current device comes from
// hipGetSymbolAddress, is looked up once per device and is what every launch gets.
// The array starts zero-filled like any device global, which is the state the allocation
// kernels expect of a workspace and leave behind.
// ----------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = (size_t)HORA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // per device: address of that device's copy of `scratch`

static int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HORA_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return HORA_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return HORA_OK;
}

int allocate_shared_prior(int64_t n, int32_t g0, const int32_t* c, double alpha0, double beta0, int64_t budget,
                          int32_t delta_max, int32_t method, int32_t* delta, double* util, void* group_off,
                          int32_t off_t, hora_alloc_summary* summary, int32_t* dev_status, void* workspace,
                          size_t workspace_bytes, hipStream_t stream);

}  // namespace hora

using namespace hora;

extern "C" {

size_t hora_allocate_workspace_bytes(int64_t n, int32_t g0) {
    if (n < 0 || g0 < 0) return 0;
    Workspace w = carve(nullptr);
    return w.bytes;
}

int hora_marginal_gains(int64_t n, const double* alpha, const double* beta, int32_t count, double* gains,
                        double* util, void* stream) {
    if (n < 0 || count < 0) return HORA_ERR_INVALID_ARG;
    if (n == 0 || count == 0 || (!gains && !util)) return HORA_OK;
    if (!alpha || !beta) return HORA_ERR_INVALID_ARG;
    const long long blocks = (n + kThreads - 1) / kThreads;
    if (blocks > INT_MAX) return HORA_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_gain_table, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream, (long long)n,
                       alpha, beta, (int)count, gains, util);
    return check_launch();
}

int hora_allocate(int64_t n, int32_t g0, const int32_t* c, double alpha0, double beta0, int64_t budget,
                  int32_t delta_max, int32_t method, int32_t* delta, double* util, void* group_off, int32_t off_t,
                  hora_alloc_summary* summary, int32_t* dev_status, void* workspace, size_t workspace_bytes,
                  void* stream) {
    return allocate_shared_prior(n, g0, c, alpha0, beta0, budget, delta_max, method, delta, util, group_off, off_t,
                                 summary, dev_status, workspace, workspace_bytes, (hipStream_t)stream);
}

int hora_allocate_static(int64_t n, int32_t g0, const int32_t* c, double alpha0, double beta0, int64_t budget,
                         int32_t delta_max, int32_t method, int32_t* delta, double* util, void* group_off,
                         int32_t off_t, hora_alloc_summary* summary, int32_t* dev_status, void* stream) {
    if (n > (int64_t)HORA_STATIC_MAX_PROMPTS) return HORA_ERR_UNSUPPORTED;
    if (n >= 0 && g0 >= 0 && carve(nullptr).bytes > kStaticScratchBytes) return HORA_ERR_UNSUPPORTED;
    void* ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc != HORA_OK) return rc;
    return allocate_shared_prior(n, g0, c, alpha0, beta0, budget, delta_max, method, delta, util, group_off, off_t,
                                 summary, dev_status, ptr, kStaticScratchBytes, (hipStream_t)stream);
}

}  // extern "C"

namespace hora {

int allocate_shared_prior(int64_t n, int32_t g0, const int32_t* c, double alpha0, double beta0, int64_t budget,
                          int32_t delta_max, int32_t method, int32_t* delta, double* util, void* group_off,
                          int32_t off_t, hora_alloc_summary* summary, int32_t* dev_status, void* workspace,
                          size_t workspace_bytes, hipStream_t stream) {
    CommonArgs a{n, g0, budget, delta_max, delta, util, group_off, off_t, summary, dev_status,
                 workspace, workspace_bytes, stream};
    int rc = validate_common(a);
    if (rc != HORA_OK) return rc;
    if (!(alpha0 > 0.0) || !(beta0 > 0.0) || !std::isfinite(alpha0) || !std::isfinite(beta0))
        return HORA_ERR_INVALID_ARG;
    if (method != HORA_ALLOC_AUTO && method != HORA_ALLOC_CLASS && method != HORA_ALLOC_BISECT)
        return HORA_ERR_INVALID_ARG;
    if (method == HORA_ALLOC_CLASS && g0 > HORA_CLASS_MAX_G0) return HORA_ERR_UNSUPPORTED;
    if (method == HORA_ALLOC_AUTO) method = g0 <= HORA_CLASS_MAX_G0 ? HORA_ALLOC_CLASS : HORA_ALLOC_BISECT;
    if (n == 0) return handle_empty(a);
    if (!c || (reinterpret_cast<uintptr_t>(c) & 3)) return HORA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return HORA_ERR_WORKSPACE;
    Workspace w = carve(workspace);
    if (workspace_bytes < w.bytes) return HORA_ERR_WORKSPACE;
    const Plan p = make_plan(n);
    if (method == HORA_ALLOC_BISECT) {
        CountsSource src{c, g0, alpha0, beta0};
        return run_bisect(src, a, p, w);
    }
    return run_class(c, alpha0, beta0, a, p, w, 0);
}

}  // namespace hora

extern "C" {

int hora_allocate_baseline(int64_t n, int32_t g0, const int32_t* c, double alpha0, double beta0, int64_t budget,
                           int32_t delta_max, int32_t rule, int32_t* delta, double* util, void* group_off,
                           int32_t off_t, hora_alloc_summary* summary, int32_t* dev_status, void* workspace,
                           size_t workspace_bytes, void* stream) {
    CommonArgs a{n, g0, budget, delta_max, delta, util, group_off, off_t, summary, dev_status,
                 workspace, workspace_bytes, (hipStream_t)stream};
    if (rule != HORA_RULE_UNIFORM && rule != HORA_RULE_HARD_FIRST) return HORA_ERR_INVALID_ARG;
    // feasibility depends on the rule (hard-first needs the data): checked on the device
    CommonArgs host = a;
    host.delta_max = 0;
    int rc = validate_common(host);
    if (rc != HORA_OK) return rc;
    if (!(alpha0 > 0.0) || !(beta0 > 0.0) || !std::isfinite(alpha0) || !std::isfinite(beta0))
        return HORA_ERR_INVALID_ARG;
    if (g0 > HORA_CLASS_MAX_G0) return HORA_ERR_UNSUPPORTED;
    if (delta_max > 0 && budget > 0 && (budget + delta_max - 1) / delta_max > n) return HORA_ERR_INFEASIBLE;
    if (n == 0) return handle_empty(a);
    if (!c || (reinterpret_cast<uintptr_t>(c) & 3)) return HORA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return HORA_ERR_WORKSPACE;
    Workspace w = carve(workspace);
    if (workspace_bytes < w.bytes) return HORA_ERR_WORKSPACE;
    const Plan p = make_plan(n);
    return run_class(c, alpha0, beta0, a, p, w, rule == HORA_RULE_UNIFORM ? 1 : 2);
}

int hora_allocate_posterior(int64_t n, int32_t g0, const double* alpha, const double* beta, int64_t budget,
                            int32_t delta_max, int32_t* delta, double* util, void* group_off, int32_t off_t,
                            hora_alloc_summary* summary, int32_t* dev_status, void* workspace,
                            size_t workspace_bytes, void* stream) {
    CommonArgs a{n, g0, budget, delta_max, delta, util, group_off, off_t, summary, dev_status,
                 workspace, workspace_bytes, (hipStream_t)stream};
    int rc = validate_common(a);
    if (rc != HORA_OK) return rc;
    if (n == 0) return handle_empty(a);
    if (!alpha || !beta || (reinterpret_cast<uintptr_t>(alpha) & 7) || (reinterpret_cast<uintptr_t>(beta) & 7))
        return HORA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return HORA_ERR_WORKSPACE;
    Workspace w = carve(workspace);
    if (workspace_bytes < w.bytes) return HORA_ERR_WORKSPACE;
    const Plan p = make_plan(n);
    PosteriorSource src{alpha, beta};
    return run_bisect(src, a, p, w);
}

}  // extern "C"
