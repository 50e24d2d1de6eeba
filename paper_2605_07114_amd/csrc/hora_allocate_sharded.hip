// Phase-B allocation on independent shards of the batch (App. C: the paper runs Phase B
// on four mini-batches of Gamma/4 prompts, and Prop. 1 then holds inside each shard).
//
// One workgroup owns one shard and finds its threshold gain tau on its own, so there is
// no grid-wide dependency; then it writes the shard's outputs with the ties at tau
// resolved by prompt index.  The result of a shard equals that of hora_allocate on the
// shard's prompts and budget.  Two ways to find tau:
//  by table (shared prior): gains depend on c only, so a set-up kernel evaluates the
//    G0+1 gain sequences (once: the workspace keeps them for later calls with the same
//    prior); a shard takes the histogram of its c and searches the bit pattern of tau in
//    passes of 256 intervals over the table entries, each entry weighted by its class
//    count.  No division in the shard's workgroup.
//  by walks (any posterior, and allocations deeper than the table): windows of the bit
//    pattern are searched from the largest gain down, every prompt walking its gain
//    recurrence down to the window.
//
// Group offsets run over the whole batch, so they need the budgets of the earlier
// shards: the set-up kernel also writes their exclusive prefix sums.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"
#include "hora_alloc_common.h"

namespace hora {

constexpr int kShardThreads = 256;
constexpr int kShardWaves = kShardThreads / kWave;
constexpr int kPrefixThreads = 1024;
constexpr int kPrefixChunk = 8 * kPrefixThreads;   // shards per prefix-sum workgroup
constexpr unsigned kShardTiedBit = 0x80000000u;
constexpr unsigned long long kWindowStep = 4ull << 52;   // 4 exponent steps: a factor 16 in value
// Windows from the largest gain down to zero (at most 2047 / 4), plus the narrowing passes
// inside the window that holds tau (each cuts the bracket at least 128-fold).
constexpr int kShardMaxPasses = 512 + 10;
constexpr int kShardTableCap = 8192;     // entries of the gain table (and of the survival table)
constexpr int kShardMaxDepth = 512;      // gains per class in the table, at most

// Start of the workspace: says which tables the workspace holds, so that a call with the
// same prior, G0 and depth as the one before reuses them (the sequences are walked one
// division after the other, which costs more than a whole small call).  Zero = none.
struct ShardTableKey {
    unsigned long long magic;
    double alpha0, beta0;
    int g0, depth;
    int usable, pad0;
    unsigned long long pad[27];
};
static_assert(sizeof(ShardTableKey) == 256, "key size");
constexpr unsigned long long kTableMagic = 0x484f52415461626cull;
constexpr int kShardMaxClasses = HORA_CLASS_MAX_G0 + 1;
constexpr int kLevelBlock = 64;          // sorted levels per coarse block (one wavefront evaluates a block)
constexpr int kMaxCoarse = kShardTableCap / kLevelBlock;
constexpr int kWaveShardMax = 1024;      // larger shards go to the workgroup-per-shard kernel
constexpr int kWaveShardMeanMax = 256;   // mean shard size up to which the wavefront-per-shard kernel is used

// u16 entries per sorted level (the per-class counts of one level are one 32- or 128-byte row)
__host__ __device__ inline int level_stride(int nc) { return nc <= 16 ? 16 : 64; }

struct ShardWorkspace {
    ShardTableKey* key;
    double* gain_table;              // [nc][depth]  M_c(l)
    double* surv_table;              // [nc][depth]  E_c(l)
    unsigned long long* level_bits;  // [nc * usable depth] all table gains, sorted descending
    unsigned short* level_kge;       // [levels][stride]: #{l : M_c(l) >= that level's gain}
    int* todo;                       // [0]: number of shards left to the workgroup-per-shard kernel; then their ids
    long long* prefix;               // [n_shards] budget given to earlier shards
    size_t bytes;
};

__host__ inline ShardWorkspace carve_shards(void* base, int64_t n_shards) {
    ShardWorkspace w;
    char* ptr = (char*)base;
    size_t off = 0;
    const size_t ns = (size_t)(n_shards > 0 ? n_shards : 1);
    w.key = (ShardTableKey*)(ptr + off); off += sizeof(ShardTableKey);
    w.gain_table = (double*)(ptr + off); off += (size_t)kShardTableCap * sizeof(double);
    w.surv_table = (double*)(ptr + off); off += (size_t)kShardTableCap * sizeof(double);
    w.level_bits = (unsigned long long*)(ptr + off); off += (size_t)kShardTableCap * sizeof(unsigned long long);
    w.level_kge = (unsigned short*)(ptr + off); off += (size_t)kShardTableCap * 64 * sizeof(unsigned short);
    w.prefix = (long long*)(ptr + off); off += (ns * sizeof(long long) + 255) & ~(size_t)255;
    w.todo = (int*)(ptr + off); off += ((ns + 1) * sizeof(int) + 255) & ~(size_t)255;
    w.bytes = off;
    return w;
}

// Set-up.  Workgroup 0 resets the list of left-over shards.  Workgroups 2, 3, ...: exclusive
// prefix sums of the shard budgets, kPrefixChunk shards each (negative budgets count as 0; the
// shard's own workgroup reports them).
// Workgroup 1: the gain and survival sequences of the G0+1 classes, one thread per class
// (Sec. 3.2 stable update; App. A), `depth` entries each; then all gains l < usable of all
// classes sorted descending into "levels": the position of a gain is the number of gains
// above it plus, among equal gains, the number of lower classes that hold it, and every
// level carries, per class, the number of that class's gains >= the level.  With these a
// shard finds its threshold by a search over levels: count_ge(level) = sum_c n_c * kge_c.
__global__ __launch_bounds__(kPrefixThreads) void k_shard_setup(long long n_shards,
                                                                const long long* __restrict__ shard_budget,
                                                                long long* __restrict__ prefix, int g0,
                                                                double alpha0, double beta0, int depth,
                                                                int usable, ShardTableKey* __restrict__ key,
                                                                double* __restrict__ gain_table,
                                                                double* __restrict__ surv_table,
                                                                unsigned long long* __restrict__ level_bits,
                                                                unsigned short* __restrict__ level_kge,
                                                                int* __restrict__ todo) {
    __shared__ unsigned long long s_raw[kShardTableCap];   // workgroup 0: wavefront totals; workgroup 1: the gains
    long long* s_tot = reinterpret_cast<long long*>(s_raw);
    if (blockIdx.x == 1) {
        if (depth == 0) return;
        const bool cached = key->magic == kTableMagic && key->alpha0 == alpha0 && key->beta0 == beta0 &&
                            key->g0 == g0 && key->depth == depth && key->usable == usable;
        if (cached) return;   // uniform: every thread reads the same key
        __syncthreads();      // all threads have read the key before thread 0 clears it
        if (threadIdx.x == 0) key->magic = 0ull;
        if (threadIdx.x <= (unsigned)g0) {
            const int cls = (int)threadIdx.x;
            const double a = alpha0 + (double)cls;
            const double b = beta0 + (double)(g0 - cls);
            const double s = a + b;
            double m = gain_first(a, s), e = 1.0, lf = 0.0;
            for (int l = 0; l < depth; ++l) {
                gain_table[cls * depth + l] = m;
                surv_table[cls * depth + l] = e;
                s_raw[cls * depth + l] = gain_bits(m);
                e = surv_next(e, b, s, lf);
                m = gain_next(m, b, s, lf);
                lf += 1.0;
            }
        }
        __syncthreads();
        // levels: one entry (class, l) at a time per thread; two rounds of searches, the first
        // for the entry's position, the second to write the per-class counts there
        const int nc = g0 + 1;
        const int stride = level_stride(nc);
        for (int e = (int)threadIdx.x; e < nc * usable; e += kPrefixThreads) {
            const int cls = e / usable, l = e - cls * usable;
            const unsigned long long v = s_raw[cls * depth + l];
            int pos_of = 0;
            for (int round = 0; round < 2; ++round) {
                int rank = 0, order = 0;
                for (int c2 = 0; c2 < nc; ++c2) {
                    const unsigned long long* row = s_raw + c2 * depth;
                    int lo = 0, hi = usable;          // first index whose gain is <= v
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if (row[mid] > v) lo = mid + 1; else hi = mid;
                    }
                    const int eq = (lo < usable && row[lo] == v) ? 1 : 0;
                    rank += lo;
                    if (c2 < cls) order += eq;
                    if (round == 1) level_kge[(long long)pos_of * stride + c2] = (unsigned short)(lo + eq);
                }
                pos_of = rank + order;
            }
            level_bits[pos_of] = v;
        }
        __threadfence();
        __syncthreads();
        if (threadIdx.x == 0) {
            key->alpha0 = alpha0; key->beta0 = beta0; key->g0 = g0; key->depth = depth; key->usable = usable;
            __threadfence();
            key->magic = kTableMagic;
        }
        return;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) todo[0] = 0;
    if (!prefix || blockIdx.x == 0) return;
    // Workgroup 2 + k: chunk k of kPrefixChunk shards.  It first adds up every budget before
    // its chunk (all loads independent of one another), then scans its own chunk: thread t
    // owns 8 consecutive shards (contiguous 64-byte loads and stores).
    constexpr int kPer = kPrefixChunk / kPrefixThreads;
    const long long base = (long long)(blockIdx.x - 2) * kPrefixChunk;
    long long earlier = 0;
    for (long long i = threadIdx.x; i < base; i += kPrefixThreads) {
        const long long v = shard_budget[i];
        earlier += v > 0 ? v : 0;
    }
    const long long first = base + (long long)threadIdx.x * kPer;
    long long b[kPer];
    long long sum = 0;
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        const long long v = first + k < n_shards ? shard_budget[first + k] : 0;
        b[k] = v > 0 ? v : 0;
        sum += b[k];
    }
    earlier = wave_sum<long long>(earlier);
    const long long incl = wave_incl_scan<long long>(sum);
    if (lane_id() == kWave - 1) { s_tot[wave_id()] = incl; s_tot[kPrefixThreads / kWave + wave_id()] = earlier; }
    __syncthreads();
    long long run = incl - sum;
    for (int w = 0; w < kPrefixThreads / kWave; ++w) {
        if (w < wave_id()) run += s_tot[w];
        run += s_tot[kPrefixThreads / kWave + w];
    }
#pragma unroll
    for (int k = 0; k < kPer; ++k) {
        if (first + k < n_shards) prefix[first + k] = run;
        run += b[k];
    }
}

struct ShardShared {
    TallyBins bins;
    unsigned long long red_u[2][kShardWaves];
    long long red_i[2][kShardWaves];
    unsigned long long lo, hi;   // bracket of tau's bit pattern
    long long above;             // pairs whose gain is > hi
    int done;                    // 1: hi is tau; 2: ran out of gains
    int by_table;                // the table search settled tau and the per-class results below
    long long n_cls[kShardMaxClasses];   // prompts of the shard per class
    int k_cls[kShardMaxClasses];         // gains of the class above tau
    int tied_cls[kShardMaxClasses];      // the class's next gain equals tau
    double e_cls[kShardMaxClasses];      // E_c(k_c)
};

// sums (a, b) over the workgroup; every thread gets both totals
__device__ __forceinline__ void shard_sum2(long long& a, long long& b, ShardShared& sh) {
    a = wave_sum<long long>(a);
    b = wave_sum<long long>(b);
    __syncthreads();
    if (lane_id() == 0) { sh.red_i[0][wave_id()] = a; sh.red_i[1][wave_id()] = b; }
    __syncthreads();
    a = 0; b = 0;
#pragma unroll
    for (int w = 0; w < kShardWaves; ++w) { a += sh.red_i[0][w]; b += sh.red_i[1][w]; }
}

// exclusive prefix sums of (a, b) over the threads of the workgroup, and the totals
__device__ __forceinline__ void shard_scan2(long long a, long long b, long long& a_ex, long long& b_ex,
                                            long long& a_tot, long long& b_tot, ShardShared& sh) {
    const long long ai = wave_incl_scan<long long>(a), bi = wave_incl_scan<long long>(b);
    __syncthreads();
    if (lane_id() == kWave - 1) { sh.red_i[0][wave_id()] = ai; sh.red_i[1][wave_id()] = bi; }
    __syncthreads();
    a_ex = ai - a; b_ex = bi - b; a_tot = 0; b_tot = 0;
#pragma unroll
    for (int w = 0; w < kShardWaves; ++w) {
        const long long x = sh.red_i[0][w], y = sh.red_i[1][w];
        if (w < wave_id()) { a_ex += x; b_ex += y; }
        a_tot += x; b_tot += y;
    }
}

// Class of prompt i (clamped like CountsSource::load); sources without classes never call it.
__device__ __forceinline__ int class_of(const CountsSource& src, long long i) {
    const int x = src.c[i];
    return x < 0 ? 0 : (x > src.g0 ? src.g0 : x);
}
__device__ __forceinline__ int class_of(const PosteriorSource&, long long) { return 0; }

// Threshold by walks.
// Invariant: exactly `above` pairs have a gain > hi, and above < budget.  A pass cuts
// (lo, hi] into at most kBins intervals of 2^shift bit patterns and tallies the gains
// that fall inside (every prompt walks its gains from l = 0 down to lo).  If the
// running count from the top reaches the budget inside interval j, the bracket
// shrinks to the gains that occur there, (min - 1, max], and closes when min == max:
// tau is that gain.  Otherwise the whole window lies above tau: it is added to
// `above` and the next window, a factor 16 further down in value (4 exponent steps of
// the bit pattern), is taken.  Going down window by window keeps the walks short: a
// window's count is a small multiple of the one before it, so the work is a small
// multiple of the budget, whereas a bracket from a guaranteed lower bound (e.g. the
// smallest ceil(budget/n)-th gain) can lie orders of magnitude below tau.
// Counts fit 63 bits: n < 2^40 and one prompt has far fewer than 2^22 gains per window
// for any threshold a budget below 2^52 can reach.
template <class Src>
__device__ bool threshold_by_walks(const Src& src, long long lo_i, long long hi_i, long long budget, long long limit,
                                   ShardShared& sh, bool& data_bad, unsigned long long& tau_bits) {
    const int lane = lane_id();
    unsigned long long top = 0;
    for (long long i = lo_i + threadIdx.x; i < hi_i; i += kShardThreads) {
        double a, b;
        data_bad |= !src.load(i, a, b);
        const unsigned long long gb = gain_bits(gain_first(a, a + b));
        top = gb > top ? gb : top;
    }
    top = wave_max_u64(top);
    if (lane == 0) sh.red_u[0][wave_id()] = top;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long all_top = 0;
        for (int w = 0; w < kShardWaves; ++w) all_top = sh.red_u[0][w] > all_top ? sh.red_u[0][w] : all_top;
        sh.hi = all_top;
        sh.lo = all_top > kWindowStep ? all_top - kWindowStep : 0ull;
        sh.above = 0;
        sh.done = 0;
    }
    __syncthreads();

    for (int pass = 0; pass < kShardMaxPasses; ++pass) {
        if (sh.done) break;   // uniform: written before the barrier that ends a pass
        const unsigned long long lo = sh.lo, hi_cur = sh.hi;
        const long long above = sh.above;
        const int shift = bracket_shift(lo, hi_cur);
        static_assert(kBins == kShardThreads, "one interval per thread");
        sh.bins.cnt[threadIdx.x] = 0; sh.bins.vmax[threadIdx.x] = 0; sh.bins.vmin_inv[threadIdx.x] = 0;
        __syncthreads();
        // every wavefront runs whole rounds, so that the ballots see all of its lanes
        for (long long i0 = lo_i; i0 < hi_i; i0 += kShardThreads) {
            const long long i = i0 + threadIdx.x;
            double a = 1.0, b = 1.0;
            if (i < hi_i) src.load(i, a, b);
            const double s = a + b;
            double g = gain_first(a, s);
            double lf = 0.0;
            long long k = 0;
            unsigned long long gb = gain_bits(g);
            bool active = i < hi_i && k < limit && gb > lo;
            while (__ballot(active)) {
                tally_gains(sh.bins, active && gb <= hi_cur, gb, lo, shift);
                if (active) {
                    g = gain_next(g, b, s, lf);
                    lf += 1.0;
                    k += 1;
                    gb = gain_bits(g);
                    active = k < limit && gb > lo;
                }
            }
        }
        __syncthreads();   // the tallies are complete
        // interval j = kBins - 1 - thread: thread 0 owns the top interval
        const int j = kBins - 1 - (int)threadIdx.x;
        const long long cj = (long long)sh.bins.cnt[j];
        const unsigned long long mx = sh.bins.vmax[j], mn = ~sh.bins.vmin_inv[j];
        long long before, unused_ex, total, unused_tot;
        shard_scan2(cj, 0, before, unused_ex, total, unused_tot, sh);
        before += above;
        if (above + total < budget) {          // uniform: the whole window is above tau
            if (threadIdx.x == 0) {
                sh.above = above + total;
                sh.hi = lo;
                sh.lo = lo > kWindowStep ? lo - kWindowStep : 0ull;
                if (lo == 0ull) sh.done = 2;   // no gains left: the budget does not fit
            }
        } else if (cj != 0 && before < budget && budget <= before + cj) {   // exactly one thread
            sh.above = before;
            sh.hi = mx;
            sh.lo = mn - 1ull;
            sh.done = (mx == mn) ? 1 : 0;
        }
        __syncthreads();
    }
    tau_bits = sh.hi;
    return sh.done == 1;   // anything else cannot happen with valid posteriors and a feasible budget
}

// Threshold by table (shared prior).  Returns false when the table is too shallow for
// this shard (some class would need gains beyond `depth`); the caller then walks.
// On success sh.k_cls / sh.tied_cls / sh.e_cls hold the per-class results.
template <class Src>
__device__ bool threshold_by_table(const Src& src, long long lo_i, long long hi_i, long long budget, long long limit,
                                   int depth, const double* __restrict__ gain_table,
                                   const double* __restrict__ surv_table, ShardShared& sh,
                                   bool& data_bad, unsigned long long& tau_bits) {
    const int nc = src.g0 + 1;
    const int dshift = __ffs(depth) - 1;
    const int lim = limit < depth ? (int)limit : depth;     // usable gains per class
    // histogram of c over the shard
    for (int j = (int)threadIdx.x; j < nc; j += kShardThreads) { sh.n_cls[j] = 0; sh.k_cls[j] = 0; sh.tied_cls[j] = 0; }
    __syncthreads();
    for (long long i = lo_i + threadIdx.x; i < hi_i; i += kShardThreads) {
        int x = src.c[i];
        if (x < 0 || x > src.g0) { data_bad = true; x = x < 0 ? 0 : src.g0; }
        atomicAdd((unsigned long long*)&sh.n_cls[x], 1ull);
    }
    __syncthreads();
    // bracket (0, largest first gain of a populated class]
    if (threadIdx.x == 0) {
        unsigned long long top = 0;
        for (int j = 0; j < nc; ++j) {
            const unsigned long long v = gain_bits(gain_table[j << dshift]);
            if (sh.n_cls[j] > 0 && v > top) top = v;
        }
        sh.lo = 0ull; sh.hi = top; sh.above = 0; sh.done = 0;
    }
    __syncthreads();
    for (int pass = 0; pass < kSelectPasses + 1; ++pass) {
        if (sh.done) break;
        const unsigned long long lo = sh.lo, hi_cur = sh.hi;
        const long long above = sh.above;
        const int shift = bracket_shift(lo, hi_cur);
        sh.bins.cnt[threadIdx.x] = 0; sh.bins.vmax[threadIdx.x] = 0; sh.bins.vmin_inv[threadIdx.x] = 0;
        __syncthreads();
        for (int cls = 0; cls < nc; ++cls) {            // rows of classes the shard does not hold are skipped
            const long long w = sh.n_cls[cls];
            if (w == 0) continue;
            const double* row = gain_table + (cls << dshift);
            for (int l = (int)threadIdx.x; l < lim; l += kShardThreads) {
                const unsigned long long v = gain_bits(row[l]);
                if (v > lo && v <= hi_cur) {
                    const int j = (int)((v - lo - 1ull) >> shift);
                    atomicAdd(&sh.bins.cnt[j], (unsigned long long)w);
                    atomicMax(&sh.bins.vmax[j], v);
                    atomicMax(&sh.bins.vmin_inv[j], ~v);
                }
            }
        }
        __syncthreads();
        const int j = kBins - 1 - (int)threadIdx.x;             // thread 0 owns the top interval
        const long long cj = (long long)sh.bins.cnt[j];
        const unsigned long long mx = sh.bins.vmax[j], mn = ~sh.bins.vmin_inv[j];
        long long before, unused_ex, total, unused_tot;
        shard_scan2(cj, 0, before, unused_ex, total, unused_tot, sh);
        before += above;
        if (above + total < budget) {                           // uniform: the table does not hold tau
            if (threadIdx.x == 0) sh.done = 2;
        } else if (cj != 0 && before < budget && budget <= before + cj) {   // exactly one thread
            sh.above = before;
            sh.hi = mx;
            sh.lo = mn - 1ull;
            sh.done = (mx == mn) ? 1 : 0;
        }
        __syncthreads();
    }
    if (sh.done != 1) return false;
    tau_bits = sh.hi;
    // gains above tau per class, and whether the next one equals tau
    for (int cls = 0; cls < nc; ++cls) {
        if (sh.n_cls[cls] == 0) continue;
        const double* row = gain_table + (cls << dshift);
        for (int l = (int)threadIdx.x; l < lim; l += kShardThreads) {
            const unsigned long long v = gain_bits(row[l]);
            if (v > tau_bits) atomicAdd(&sh.k_cls[cls], 1);
            if (v == tau_bits) sh.tied_cls[cls] = 1;
        }
    }
    if (threadIdx.x == 0) sh.by_table = 1;
    __syncthreads();
    if (threadIdx.x < (unsigned)nc) {
        const int cls = (int)threadIdx.x;
        const int k = sh.k_cls[cls];
        // a populated class with every table entry above tau, and more gains beyond the
        // table: those are missing from the counts
        if (sh.n_cls[cls] > 0 && k == lim && (long long)lim < limit) sh.by_table = 0;
        const double a = src.alpha0 + (double)cls, b = src.beta0 + (double)(src.g0 - cls);
        double e = surv_table[(cls << dshift) + (k < depth ? k : depth - 1)];
        if (k == depth) e = surv_next(e, b, a + b, (double)(depth - 1));
        sh.e_cls[cls] = e;
    }
    __syncthreads();
    return sh.by_table != 0;
}

// kOff: 0 no offsets, 1 int32 offsets, 2 int64 offsets.
// The work of one workgroup on the prompts [lo_i, hi_i) with `budget` units (validated by
// the caller): threshold, per-prompt results, tie pass, outputs.  off_base: rollouts that lie
// before the shard (g0 per earlier prompt is added here; the budgets of earlier shards come
// in); summary: this shard's report or NULL.
template <class Src, int kOff>
__device__ void shard_core(const Src& src, long long lo_i, long long hi_i, long long budget, long long off_base,
                           long long n, int g0, int cap, int depth, const double* __restrict__ gain_table,
                           const double* __restrict__ surv_table, int32_t* __restrict__ delta,
                           double* __restrict__ util, void* __restrict__ group_off,
                           hora_alloc_summary* __restrict__ summary, int32_t* dev_status) {
    __shared__ ShardShared sh;
    long long limit = cap > 0 ? (long long)cap : budget;
    if (limit > budget) limit = budget;
    const bool depth_capped = limit > (long long)HORA_MAX_DEPTH;   // the library's bound on one prompt's depth
    if (depth_capped) limit = (long long)HORA_MAX_DEPTH;

    // ---- threshold ---------------------------------------------------------------------
    unsigned long long tau_bits = ~0ull;   // budget 0: nothing is above tau
    bool data_bad = false;
    bool by_table = false;
    if (budget > 0) {
        if constexpr (Src::kHasClasses)
            if (depth > 0)
                by_table = threshold_by_table(src, lo_i, hi_i, budget, limit, depth, gain_table, surv_table, sh,
                                          data_bad, tau_bits);
        if (!by_table && !threshold_by_walks(src, lo_i, hi_i, budget, limit, sh, data_bad, tau_bits)) {
            if (threadIdx.x == 0) report(dev_status, HORA_ERR_RANGE);
            return;
        }
    }

    // ---- k_i, tied flag and E_i(k_i) per prompt; totals --------------------------------
    long long ks = 0, ts = 0;
    for (long long i = lo_i + threadIdx.x; i < hi_i; i += kShardThreads) {
        long long k;
        bool tied;
        double e;
        if (by_table) {
            const int x = class_of(src, i);
            k = sh.k_cls[x];
            tied = sh.tied_cls[x] != 0;
            e = sh.e_cls[x];
        } else {
            double a, b, g, lf;
            data_bad |= !src.load(i, a, b);
            k = walk_above<true>(a, b, tau_bits, limit, g, lf, e);
            tied = (k < limit) && (gain_bits(g) == tau_bits);
            if (depth_capped && k == limit && gain_bits(g) > tau_bits) report(dev_status, HORA_ERR_UNSUPPORTED);
        }
        delta[i] = (int32_t)((unsigned)k | (tied ? kShardTiedBit : 0u));
        if (util) util[i] = e;
        ks += k;
        ts += tied ? 1 : 0;
    }
    if (data_bad) report(dev_status, HORA_ERR_RANGE);
    shard_sum2(ks, ts, sh);
    const long long r = budget - ks;
    if ((r < 0 || r > ts) && threadIdx.x == 0) report(dev_status, HORA_ERR_RANGE);
    if (summary && threadIdx.x == 0) {
        summary->tau = budget > 0 ? __longlong_as_double((long long)tau_bits) : 0.0;
        summary->count_gt = ks;
        summary->tie_units = r;
        summary->tie_prompts = ts;
    }

    // ---- ties by prompt index, final delta, utilities, offsets -------------------------
    long long rank_base = 0, k_base = 0;
    for (long long i0 = lo_i; i0 < hi_i; i0 += kShardThreads) {
        const long long i = i0 + threadIdx.x;
        const bool in = i < hi_i;
        const unsigned raw = in ? (unsigned)delta[i] : 0u;     // written above by this same thread
        const long long kk = (long long)(raw & ~kShardTiedBit);
        const long long td = (raw & kShardTiedBit) ? 1 : 0;
        long long k_ex, t_ex, k_tot, t_tot;
        shard_scan2(kk, td, k_ex, t_ex, k_tot, t_tot, sh);
        const long long rank = rank_base + t_ex;
        const bool win = td && rank < r;
        if (in) {
            delta[i] = (int32_t)(kk + (win ? 1 : 0));
            if (util) {
                double e = util[i];
                if (win) {
                    double a, b;
                    src.load(i, a, b);
                    e = surv_next(e, b, a + b, (double)kk);
                }
                util[i] = 1.0 - e;
            }
            if (kOff != 0) {
                const long long off = (long long)g0 * i + off_base + k_base + k_ex + (rank < r ? rank : r);
                const long long next = off + g0 + kk + (win ? 1 : 0);
                if (kOff == 1) {
                    reinterpret_cast<int32_t*>(group_off)[i] = (int32_t)off;
                    if (i == n - 1) {
                        reinterpret_cast<int32_t*>(group_off)[n] = (int32_t)next;
                        if (next >= (1ll << 31)) report(dev_status, HORA_ERR_RANGE);   // total does not fit
                    }
                } else {
                    reinterpret_cast<long long*>(group_off)[i] = off;
                    if (i == n - 1) reinterpret_cast<long long*>(group_off)[n] = next;
                }
            }
        }
        rank_base += t_tot;
        k_base += k_tot;
    }
}

// What is wrong with a shard's bounds or budget, if anything: HORA_ERR_RANGE when the shards do
// not tile [0, n) in order or the budget is negative, HORA_ERR_INFEASIBLE when the budget
// cannot be placed in the shard, HORA_ERR_UNSUPPORTED when it is beyond the depth bound.
__device__ __forceinline__ int check_shard(long long shard, long long n_shards, long long n, long long lo_i,
                                           long long hi_i, long long budget, int cap) {
    if (lo_i < 0 || hi_i < lo_i || hi_i > n || budget < 0 || (shard == 0 && lo_i != 0) ||
        (shard == n_shards - 1 && hi_i != n))
        return HORA_ERR_RANGE;
    const long long size = hi_i - lo_i;
    if ((budget > 0 && size == 0) || (cap > 0 && budget > size * (long long)cap)) return HORA_ERR_INFEASIBLE;
    if (budget > size * (long long)HORA_MAX_DEPTH || budget >= (1ll << 52)) return HORA_ERR_UNSUPPORTED;
    return HORA_OK;
}

// Loads and checks one shard's bounds and budget, then runs shard_core on it.
template <class Src, int kOff>
__device__ void shard_by_workgroup(const Src& src, long long shard, long long n, int g0, long long n_shards,
                                   const long long* __restrict__ shard_off,
                                   const long long* __restrict__ shard_budget, int cap,
                                   const long long* __restrict__ prefix, int depth,
                                   const double* __restrict__ gain_table, const double* __restrict__ surv_table,
                                   int32_t* __restrict__ delta, double* __restrict__ util,
                                   void* __restrict__ group_off, hora_alloc_summary* __restrict__ summary,
                                   int32_t* dev_status) {
    const long long lo_i = shard_off[shard], hi_i = shard_off[shard + 1];
    const long long budget = shard_budget[shard];
    const int wrong = check_shard(shard, n_shards, n, lo_i, hi_i, budget, cap);
    if (wrong != HORA_OK) {
        if (threadIdx.x == 0) report(dev_status, wrong);
        return;
    }
    shard_core<Src, kOff>(src, lo_i, hi_i, budget, kOff != 0 ? prefix[shard] : 0, n, g0, cap, depth, gain_table,
                          surv_table, delta, util, group_off, summary ? summary + shard : nullptr, dev_status);
}

// A whole batch as one shard, for batches small enough for one workgroup: one launch in place
// of the pass-by-pass search (any posterior; the arguments have been checked on the host).
template <class Src, int kOff>
__global__ __launch_bounds__(kShardThreads) void k_whole_batch(Src src, long long n, int g0, long long budget, int cap,
                                                               int32_t* __restrict__ delta,
                                                               double* __restrict__ util,
                                                               void* __restrict__ group_off,
                                                               hora_alloc_summary* __restrict__ summary,
                                                               int32_t* dev_status) {
    shard_core<Src, kOff>(src, 0, n, budget, 0, n, g0, cap, 0, nullptr, nullptr, delta, util, group_off, summary,
                          dev_status);
}

template <class Src>
static int launch_whole_batch(const Src& src, int64_t n, int32_t g0, int64_t budget, int32_t delta_max,
                              int32_t* delta, double* util, void* group_off, int32_t off_t,
                              hora_alloc_summary* summary, int32_t* dev_status, hipStream_t stream) {
    const int cap = delta_max > 0 ? delta_max : 0;
    const int mode = group_off ? (off_t == HORA_I32 ? 1 : 2) : 0;
#define HORA_LAUNCH_WHOLE(M)                                                                                    \
    hipLaunchKernelGGL((k_whole_batch<Src, M>), dim3(1), dim3(kShardThreads), 0, stream, src, (long long)n,      \
                       (int)g0, (long long)budget, cap, delta, util, group_off, summary, dev_status)
    if (mode == 0) HORA_LAUNCH_WHOLE(0);
    else if (mode == 1) HORA_LAUNCH_WHOLE(1);
    else HORA_LAUNCH_WHOLE(2);
#undef HORA_LAUNCH_WHOLE
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}

int allocate_small_counts(const CountsSource& src, int64_t n, int32_t g0, int64_t budget, int32_t delta_max,
                          int32_t* delta, double* util, void* group_off, int32_t off_t, hora_alloc_summary* summary,
                          int32_t* dev_status, hipStream_t stream) {
    return launch_whole_batch(src, n, g0, budget, delta_max, delta, util, group_off, off_t, summary, dev_status, stream);
}
int allocate_small_posterior(const PosteriorSource& src, int64_t n, int32_t g0, int64_t budget, int32_t delta_max,
                             int32_t* delta, double* util, void* group_off, int32_t off_t,
                             hora_alloc_summary* summary, int32_t* dev_status, hipStream_t stream) {
    return launch_whole_batch(src, n, g0, budget, delta_max, delta, util, group_off, off_t, summary, dev_status, stream);
}

// One workgroup per shard.
template <class Src, int kOff>
__global__ __launch_bounds__(kShardThreads) void k_shard_allocate(Src src, long long n, int g0, long long n_shards,
                                                                  const long long* __restrict__ shard_off,
                                                                  const long long* __restrict__ shard_budget,
                                                                  int cap, const long long* __restrict__ prefix,
                                                                  int depth, const double* __restrict__ gain_table,
                                                                  const double* __restrict__ surv_table,
                                                                  int32_t* __restrict__ delta,
                                                                  double* __restrict__ util,
                                                                  void* __restrict__ group_off,
                                                                  hora_alloc_summary* __restrict__ summary,
                                                                  int32_t* dev_status) {
    shard_by_workgroup<Src, kOff>(src, (long long)blockIdx.x, n, g0, n_shards, shard_off, shard_budget, cap, prefix,
                                  depth, gain_table, surv_table, delta, util, group_off, summary, dev_status);
}

// The shards the wavefront-per-shard kernel left over (todo[0] of them, ids from todo[1]):
// a fixed number of workgroups takes them in turn.
template <class Src, int kOff>
__global__ __launch_bounds__(kShardThreads) void k_shard_allocate_todo(Src src, long long n, int g0,
                                                                       long long n_shards,
                                                                       const long long* __restrict__ shard_off,
                                                                       const long long* __restrict__ shard_budget,
                                                                       int cap, const long long* __restrict__ prefix,
                                                                       int depth,
                                                                       const double* __restrict__ gain_table,
                                                                       const double* __restrict__ surv_table,
                                                                       int32_t* __restrict__ delta,
                                                                       double* __restrict__ util,
                                                                       void* __restrict__ group_off,
                                                                       hora_alloc_summary* __restrict__ summary,
                                                                       const int* __restrict__ todo,
                                                                       int32_t* dev_status) {
    const int count = todo[0];
    for (int idx = (int)blockIdx.x; idx < count; idx += (int)gridDim.x) {
        shard_by_workgroup<Src, kOff>(src, (long long)todo[1 + idx], n, g0, n_shards, shard_off, shard_budget, cap,
                                      prefix, depth, gain_table, surv_table, delta, util, group_off, summary,
                                      dev_status);
        __syncthreads();   // the LDS state is reused by the next shard
    }
}

// ----------------------------------------------------------------------------------
// Wavefront per shard (shared prior, small shards).  A workgroup of four wavefronts takes
// four shards; nothing is shared between them but the coarse rows in LDS.
//  1. histogram of c: lane k counts class k (wavefront ballots);
//  2. coarse search: lane q evaluates count_ge of the last level of block q (the coarse
//     rows, one per 64 levels, are in LDS) and the first block that reaches the budget is
//     taken; fine search: lane t evaluates level 64 q + t of that block (one 32- or
//     128-byte row per lane from global memory).  tau is the first level whose count_ge
//     reaches the budget; the level before it gives the gains above tau per class;
//  3. outputs with the tie pass inside the wavefront (ballot + mbcnt ranks, DPP prefix sums
//     for the offsets).
// Two dependent global loads (the shard's c, then the block's rows) plus the per-class
// look-ups, instead of several passes with workgroup barriers.  A shard the table cannot
// settle (deeper than the table, more than kWaveShardMax prompts) is put on a list for the
// workgroup-per-shard code, which a second kernel runs afterwards.
// ----------------------------------------------------------------------------------
struct WaveScratch {          // per wavefront, LDS
    int k[kShardMaxClasses];
    int tied[kShardMaxClasses];
    double e[kShardMaxClasses];
    unsigned rows[2][8];      // the per-class counts of level tau and of the level before (16 classes or fewer)
};

template <int kOff>
__global__ __launch_bounds__(kShardThreads) void k_shard_allocate_waves(
    CountsSource src, long long n, long long n_shards, const long long* __restrict__ shard_off,
    const long long* __restrict__ shard_budget, int cap, const long long* __restrict__ prefix, int depth, int usable,
    const double* __restrict__ surv_table, const unsigned long long* __restrict__ level_bits,
    const unsigned short* __restrict__ level_kge, int* __restrict__ todo, int32_t* __restrict__ delta,
    double* __restrict__ util, void* __restrict__ group_off, hora_alloc_summary* __restrict__ summary,
    int32_t* dev_status) {
    __shared__ unsigned short s_coarse[kMaxCoarse * 64];
    __shared__ WaveScratch s_wave[kShardWaves];
    const int g0 = src.g0;
    const int nc = g0 + 1;
    const int stride = level_stride(nc);
    const int levels = nc * usable;
    const int n_coarse = (levels + kLevelBlock - 1) / kLevelBlock;
    // the shard's bounds and budget are requested first, so that they travel while the coarse
    // rows are staged (coarse row q = the last level of block q)
    const int lane = lane_id();
    const long long shard = (long long)blockIdx.x * kShardWaves + wave_id();
    const bool live = shard < n_shards;
    const long long lo_i = live ? shard_off[shard] : 0, hi_i = live ? shard_off[shard + 1] : 0;
    const long long budget = live ? shard_budget[shard] : 0;
    const long long before = (kOff != 0 && live) ? prefix[shard] : 0;   // units of the shards before this one
    for (int idx = (int)threadIdx.x; idx < n_coarse * stride; idx += kShardThreads) {
        const int q = idx / stride, k = idx - q * stride;
        int p = q * kLevelBlock + kLevelBlock - 1;
        if (p > levels - 1) p = levels - 1;
        s_coarse[idx] = level_kge[(long long)p * stride + k];
    }
    __syncthreads();
    if (!live) return;
    WaveScratch& ws = s_wave[wave_id()];
    const int wrong = check_shard(shard, n_shards, n, lo_i, hi_i, budget, cap);
    if (wrong != HORA_OK) {
        if (lane == 0) report(dev_status, wrong);
        return;
    }
    const long long size = hi_i - lo_i;
    if (size > kWaveShardMax) {
        if (lane == 0) todo[1 + atomicAdd(&todo[0], 1)] = (int)shard;
        return;
    }
    const long long limit = cap > 0 ? (budget < cap ? budget : (long long)cap) : budget;   // (the table is far shallower than the depth bound)

    // ---- 1. histogram: lane k ends up with the number of prompts of class k
    int n_mine = 0;
    bool data_bad = false;
    for (long long i0 = lo_i; i0 < hi_i; i0 += kWave) {
        const long long i = i0 + lane;
        int x = -1;
        if (i < hi_i) {
            x = src.c[i];
            if (x < 0 || x > g0) { data_bad = true; x = x < 0 ? 0 : g0; }
        }
        for (int k = 0; k < nc; ++k) {
            const int cnt = __popcll(__ballot(x == k));
            if (lane == k) n_mine += cnt;
        }
    }
    if (data_bad) report(dev_status, HORA_ERR_RANGE);

    // ---- 2. threshold
    int k_mine = 0, tied_mine = 0;            // lane c: gains of class c above tau; its next gain equals tau
    double e_mine = 1.0;                      // lane c: E_c(k_c)
    long long count_gt = 0, tie_prompts = 0;
    unsigned long long tau_bits = 0;
    bool settled = true;
    if (budget > 0) {
        // coarse: lane q (and q + 64) evaluates the last level of its block
        long long cq[2] = {0, 0};
        for (int k = 0; k < nc; ++k) {
            const long long nk = (long long)__builtin_amdgcn_readlane(n_mine, k);
            if (nk == 0) continue;            // uniform
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int q = lane + 64 * h;
                if (q < n_coarse) cq[h] += nk * (long long)s_coarse[q * stride + k];
            }
        }
        int block = -1;
        long long before_block = 0;           // count_ge of the last level of the block before
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (block < 0) {
                const unsigned long long reach = __ballot(lane + 64 * h < n_coarse && cq[h] >= budget);
                if (reach) {
                    const int first = __ffsll((long long)reach) - 1;
                    block = first + 64 * h;
                    if (first > 0) before_block = __shfl(cq[h], first - 1, kWave);
                    else if (h == 1) before_block = __shfl(cq[0], kWave - 1, kWave);
                }
            }
        }
        if (block < 0) {
            settled = false;                  // the table does not reach the budget
        } else {
            // fine: lane t evaluates level 64 * block + t
            const int p = block * kLevelBlock + lane;
            long long ct = 0;
            unsigned w[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};   // this lane's row (16 classes or fewer)
            if (p < levels) {
                const unsigned short* row = level_kge + (long long)p * stride;
                if (stride == 16) {
                    const uint4 r0 = *reinterpret_cast<const uint4*>(row);
                    const uint4 r1 = *reinterpret_cast<const uint4*>(row + 8);
                    w[0] = r0.x; w[1] = r0.y; w[2] = r0.z; w[3] = r0.w;
                    w[4] = r1.x; w[5] = r1.y; w[6] = r1.z; w[7] = r1.w;
#pragma unroll
                    for (int k = 0; k < 16; ++k) {
                        const long long nk = (long long)__builtin_amdgcn_readlane(n_mine, k);
                        const unsigned kge = (k & 1) ? (w[k >> 1] >> 16) : (w[k >> 1] & 0xffffu);
                        ct += nk * (long long)kge;    // lanes beyond nc hold n = 0
                    }
                } else {
                    for (int k = 0; k < nc; ++k) {
                        const long long nk = (long long)__builtin_amdgcn_readlane(n_mine, k);
                        ct += nk * (long long)row[k];
                    }
                }
            }
            const unsigned long long reach = __ballot(p < levels && ct >= budget);
            // reach != 0: the block's last level reaches the budget
            const int t = __ffsll((long long)reach) - 1;
            const int j = block * kLevelBlock + t;                 // tau = level j
            count_gt = t > 0 ? __shfl(ct, t - 1, kWave) : before_block;
            tau_bits = level_bits[j];
            if (stride == 16) {
                // the two rows are in the registers of lanes t and t - 1: hand them over through LDS
                // (level j - 1 of the first lane's block is the coarse row of the block before)
                if (lane == t || lane == t - 1) {
                    unsigned* dst = ws.rows[lane == t ? 0 : 1];
#pragma unroll
                    for (int q = 0; q < 8; ++q) dst[q] = w[q];
                }
            }
            if (lane < nc) {
                int ge, gt;
                if (stride == 16) {
                    const unsigned wge = ws.rows[0][lane >> 1];
                    ge = (int)((lane & 1) ? wge >> 16 : wge & 0xffffu);
                    if (t > 0) {
                        const unsigned wgt = ws.rows[1][lane >> 1];
                        gt = (int)((lane & 1) ? wgt >> 16 : wgt & 0xffffu);
                    } else {
                        gt = block > 0 ? (int)s_coarse[(block - 1) * stride + lane] : 0;
                    }
                } else {
                    ge = level_kge[(long long)j * stride + lane];
                    gt = j > 0 ? level_kge[(long long)(j - 1) * stride + lane] : 0;
                }
                k_mine = gt;
                tied_mine = ge - gt;
                // every usable gain of a class the shard holds is above tau and the sequence
                // goes on beyond the table: gains are missing from the counts
                if (n_mine > 0 && gt == usable && (long long)usable < limit) settled = false;
                const double a = src.alpha0 + (double)lane, b = src.beta0 + (double)(g0 - lane);
                double e = surv_table[lane * depth + (gt < depth ? gt : depth - 1)];
                if (gt == depth) e = surv_next(e, b, a + b, (double)(depth - 1));
                e_mine = e;
            }
            settled = __ballot(!settled) == 0;
            long long tp = tied_mine ? (long long)n_mine : 0;
            tie_prompts = wave_sum<long long>(tp);
        }
    }
    if (!settled) {
        if (lane == 0) todo[1 + atomicAdd(&todo[0], 1)] = (int)shard;
        return;
    }
    const long long r = budget - count_gt;
    if (summary && lane == 0) {
        summary[shard].tau = budget > 0 ? __longlong_as_double((long long)tau_bits) : 0.0;
        summary[shard].count_gt = count_gt;
        summary[shard].tie_units = r;
        summary[shard].tie_prompts = tie_prompts;
    }
    ws.k[lane] = k_mine;
    ws.tied[lane] = tied_mine;
    ws.e[lane] = e_mine;
    // (same wavefront reads them back below: LDS operations of a wavefront complete in order)

    // ---- 3. outputs
    const long long off_base = kOff != 0 ? (long long)g0 * lo_i + before : 0;
    long long rank_base = 0, given = 0;       // tied prompts / units handed out before this tile
    for (long long i0 = lo_i; i0 < hi_i; i0 += kWave) {
        const long long i = i0 + lane;
        const bool in = i < hi_i;
        int x = 0;
        if (in) {
            x = src.c[i];
            x = x < 0 ? 0 : (x > g0 ? g0 : x);
        }
        const int kk = in ? ws.k[x] : 0;
        const bool td = in && ws.tied[x] != 0;
        const unsigned long long tied_mask = __ballot(td);
        const long long rank = rank_base + lanes_below(tied_mask);
        const bool win = td && rank < r;
        const int dd = kk + (win ? 1 : 0);
        const int units = in ? g0 + dd : 0;
        const long long incl = wave_incl_scan_i64((long long)units);
        if (in) {
            delta[i] = dd;
            if (util) {
                double e = ws.e[x];
                if (win) {
                    const double a = src.alpha0 + (double)x, b = src.beta0 + (double)(g0 - x);
                    e = surv_next(e, b, a + b, (double)kk);
                }
                util[i] = 1.0 - e;
            }
            if (kOff != 0) {
                const long long off = off_base + given + incl - units;
                if (kOff == 1) {
                    reinterpret_cast<int32_t*>(group_off)[i] = (int32_t)off;
                    if (i == n - 1) {
                        reinterpret_cast<int32_t*>(group_off)[n] = (int32_t)(off + units);
                        if (off + units >= (1ll << 31)) report(dev_status, HORA_ERR_RANGE);   // total does not fit
                    }
                } else {
                    reinterpret_cast<long long*>(group_off)[i] = off;
                    if (i == n - 1) reinterpret_cast<long long*>(group_off)[n] = off + units;
                }
            }
        }
        rank_base += __popcll(tied_mask);
        given += __shfl(incl, kWave - 1, kWave);
    }
}

__global__ void k_store_zero_offset(void* group_off, int off64) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (off64) *reinterpret_cast<long long*>(group_off) = 0;
        else *reinterpret_cast<int32_t*>(group_off) = 0;
    }
}

static size_t sharded_workspace_bytes(int64_t n_shards) { return carve_shards(nullptr, n_shards).bytes; }

// Gains per class in the table: a power of two, as many as fit; no more than a cap asks for.
static int table_depth(int g0, int32_t delta_max) {
    const int nc = g0 + 1;
    if (nc > kShardMaxClasses) return 0;
    int depth = 1;
    while (depth * 2 * nc <= kShardTableCap && depth * 2 <= kShardMaxDepth) depth *= 2;
    if (delta_max > 0)
        while (depth / 2 >= delta_max && depth > 1) depth /= 2;
    return depth;
}

}  // namespace hora

using namespace hora;

extern "C" size_t hora_allocate_sharded_workspace_bytes(int64_t n_shards) {
    if (n_shards < 0) return 0;
    return sharded_workspace_bytes(n_shards);
}

extern "C" int hora_allocate_sharded(int64_t n, int32_t g0, const int32_t* c, double alpha0, double beta0,
                                     int64_t n_shards, const int64_t* shard_off, const int64_t* shard_budget,
                                     int32_t delta_max, int32_t* delta, double* util, void* group_off,
                                     int32_t off_t, hora_alloc_summary* summary, int32_t* dev_status,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    if (n < 0 || g0 < 0 || n_shards < 0 || !dev_status) return HORA_ERR_INVALID_ARG;
    if (!(alpha0 > 0.0) || !(beta0 > 0.0) || !std::isfinite(alpha0) || !std::isfinite(beta0))
        return HORA_ERR_INVALID_ARG;
    if (group_off && off_t != HORA_I32 && off_t != HORA_I64) return HORA_ERR_INVALID_ARG;
    if (n >= (1ll << 40) || n_shards > INT_MAX) return HORA_ERR_UNSUPPORTED;
    if (n > 0 && n_shards == 0) return HORA_ERR_INVALID_ARG;   // the shards must cover every prompt
    if (group_off && off_t == HORA_I32 && n * (long long)g0 >= (1ll << 31)) return HORA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(delta) & 3) || (reinterpret_cast<uintptr_t>(util) & 7) ||
        (reinterpret_cast<uintptr_t>(dev_status) & 3) || (reinterpret_cast<uintptr_t>(c) & 3) ||
        (reinterpret_cast<uintptr_t>(shard_off) & 7) || (reinterpret_cast<uintptr_t>(shard_budget) & 7) ||
        (reinterpret_cast<uintptr_t>(summary) & 7))
        return HORA_ERR_INVALID_ARG;
    if (group_off && (reinterpret_cast<uintptr_t>(group_off) & (off_t == HORA_I32 ? 3 : 7)))
        return HORA_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (n_shards == 0) {   // n == 0 too
        if (group_off) hipLaunchKernelGGL(k_store_zero_offset, 1, 1, 0, s, group_off, off_t == HORA_I64 ? 1 : 0);
        return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
    }
    if (!shard_off || !shard_budget) return HORA_ERR_INVALID_ARG;
    if (n > 0 && (!c || !delta)) return HORA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return HORA_ERR_WORKSPACE;
    if (workspace_bytes < sharded_workspace_bytes(n_shards)) return HORA_ERR_WORKSPACE;
    const ShardWorkspace w = carve_shards(workspace, n_shards);
    long long* prefix = group_off ? w.prefix : nullptr;
    const int depth = table_depth(g0, delta_max);
    const int usable = (delta_max > 0 && delta_max < depth) ? delta_max : depth;   // gains l < cap only
    const unsigned setup_blocks = 2 + (group_off ? (unsigned)((n_shards + kPrefixChunk - 1) / kPrefixChunk) : 0u);
    if (group_off && n == 0) hipLaunchKernelGGL(k_store_zero_offset, 1, 1, 0, s, group_off, off_t == HORA_I64 ? 1 : 0);
    hipLaunchKernelGGL(k_shard_setup, dim3(setup_blocks), dim3(kPrefixThreads), 0, s, (long long)n_shards,
                       (const long long*)shard_budget, prefix, (int)g0, alpha0, beta0, depth, usable, w.key,
                       w.gain_table, w.surv_table, w.level_bits, w.level_kge, w.todo);
    CountsSource src{c, g0, alpha0, beta0};
    const int cap = delta_max > 0 ? delta_max : 0;
    const int mode = group_off ? (off_t == HORA_I32 ? 1 : 2) : 0;
    // small shards: a wavefront per shard first; what it cannot settle is flagged for the
    // workgroup-per-shard kernel
    const bool waves = depth > 0 && n <= (long long)n_shards * kWaveShardMeanMax;
    if (waves) {
        const unsigned blocks = (unsigned)((n_shards + kShardWaves - 1) / kShardWaves);
#define HORA_LAUNCH_WAVES(M)                                                                                     \
    hipLaunchKernelGGL((k_shard_allocate_waves<M>), dim3(blocks), dim3(kShardThreads), 0, s, src, (long long)n,   \
                       (long long)n_shards, (const long long*)shard_off, (const long long*)shard_budget, cap,    \
                       prefix, depth, usable, w.surv_table, w.level_bits, w.level_kge, w.todo, delta, util,      \
                       group_off, summary, dev_status)
        if (mode == 0) HORA_LAUNCH_WAVES(0);
        else if (mode == 1) HORA_LAUNCH_WAVES(1);
        else HORA_LAUNCH_WAVES(2);
#undef HORA_LAUNCH_WAVES
    }
#define HORA_LAUNCH_SHARDS(M)                                                                                   \
    do {                                                                                                        \
        if (waves)                                                                                              \
            hipLaunchKernelGGL((k_shard_allocate_todo<CountsSource, M>), dim3(todo_blocks), dim3(kShardThreads), \
                               0, s, src, (long long)n, (int)g0, (long long)n_shards,                           \
                               (const long long*)shard_off, (const long long*)shard_budget, cap, prefix, depth, \
                               w.gain_table, w.surv_table, delta, util, group_off, summary, w.todo, dev_status); \
        else                                                                                                    \
            hipLaunchKernelGGL((k_shard_allocate<CountsSource, M>), dim3((unsigned)n_shards),                   \
                               dim3(kShardThreads), 0, s, src, (long long)n, (int)g0, (long long)n_shards,      \
                               (const long long*)shard_off, (const long long*)shard_budget, cap, prefix, depth, \
                               w.gain_table, w.surv_table, delta, util, group_off, summary, dev_status);        \
    } while (0)
    const unsigned todo_blocks = (unsigned)(n_shards < 1024 ? n_shards : 1024);
    if (mode == 0) HORA_LAUNCH_SHARDS(0);
    else if (mode == 1) HORA_LAUNCH_SHARDS(1);
    else HORA_LAUNCH_SHARDS(2);
#undef HORA_LAUNCH_SHARDS
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}
