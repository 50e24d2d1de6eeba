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

#include <type_traits>

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
constexpr int kPrefixGroups = 64;                  // prefix-sum workgroups of the set-up kernel, at most
constexpr unsigned kShardTiedBit = 0x80000000u;
constexpr unsigned long long kWindowStep = 4ull << 52;   // 4 exponent steps: a factor 16 in value
constexpr unsigned long long kOctaveStep = 1ull << 52;   // one exponent step: a factor 2
// Windows from the largest gain down to zero (at most 2047 of one octave), plus the narrowing
// passes inside the window that holds tau (each cuts the bracket at least 128-fold).
constexpr int kShardMaxPasses = 2048 + 10;
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

// The gain and survival sequences of the G0+1 classes, one thread per class (Sec. 3.2 stable
// update; App. A), `depth` entries each; then all gains l < usable of all classes sorted
// descending into "levels": the position of a gain is the number of gains above it plus, among
// equal gains, the number of lower classes that hold it, and every level carries, per class,
// the number of that class's gains >= the level.  With these a shard finds its threshold by a
// search over levels: count_ge(level) = sum_c n_c * kge_c.  Run by one whole workgroup; `raw`
// is where the searches read the gains' patterns from: LDS of nc * depth entries, or NULL to
// read them back from the table in global memory (slower; for callers short of LDS).
// The key is cleared first and set last, each side fenced, so that a reader that finds the key
// it wants finds complete tables.
__device__ void build_shard_tables(int g0, double alpha0, double beta0, int depth, int usable,
                                   ShardTableKey* __restrict__ key, double* __restrict__ gain_table,
                                   double* __restrict__ surv_table, unsigned long long* __restrict__ level_bits,
                                   unsigned short* __restrict__ level_kge, unsigned long long* raw) {
    if (threadIdx.x == 0) key->magic = 0ull;
    __threadfence();
    __syncthreads();
    if (threadIdx.x <= (unsigned)g0) {
        const int cls = (int)threadIdx.x;
        const double a = alpha0 + (double)cls;
        const double b = beta0 + (double)(g0 - cls);
        const double s = a + b;
        double m = gain_first(a, s), e = 1.0, lf = 0.0;
        for (int l = 0; l < depth; ++l) {
            gain_table[cls * depth + l] = m;
            surv_table[cls * depth + l] = e;
            if (raw) raw[cls * depth + l] = gain_bits(m);
            e = surv_next(e, b, s, lf);
            m = gain_next(m, b, s, lf);
            lf += 1.0;
        }
    }
    __threadfence();
    __syncthreads();
    const unsigned long long* bits = raw ? raw : reinterpret_cast<const unsigned long long*>(gain_table);
    // levels: one entry (class, l) at a time per thread; two rounds of searches, the first
    // for the entry's position, the second to write the per-class counts there
    const int nc = g0 + 1;
    const int stride = level_stride(nc);
    for (int e = (int)threadIdx.x; e < nc * usable; e += (int)blockDim.x) {
        const int cls = e / usable, l = e - cls * usable;
        const unsigned long long v = bits[cls * depth + l];
        int pos_of = 0;
        for (int round = 0; round < 2; ++round) {
            int rank = 0, order = 0;
            for (int c2 = 0; c2 < nc; ++c2) {
                const unsigned long long* row = bits + c2 * depth;
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
}

__device__ __forceinline__ bool shard_tables_match(const ShardTableKey* key, int g0, double alpha0, double beta0,
                                                   int depth, int usable) {
    return key->magic == kTableMagic && key->alpha0 == alpha0 && key->beta0 == beta0 && key->g0 == g0 &&
           key->depth == depth && key->usable == usable;
}

// Set-up for calls with many shards.  Workgroup 0 empties the list of left-over shards.  Workgroup 1: the tables, unless the workspace holds them
// already.  Workgroups 2, 3, ...: exclusive prefix sums of the shard budgets, `chunk`
// shards each (negative budgets count as 0; the shard's own workgroup reports them).
__global__ __launch_bounds__(kPrefixThreads) void k_shard_setup(long long n_shards, long long chunk,
                                                                const long long* __restrict__ shard_budget,
                                                                long long* __restrict__ prefix, int g0,
                                                                double alpha0, double beta0, int depth,
                                                                int usable, ShardTableKey* __restrict__ key,
                                                                double* __restrict__ gain_table,
                                                                double* __restrict__ surv_table,
                                                                unsigned long long* __restrict__ level_bits,
                                                                unsigned short* __restrict__ level_kge,
                                                                int* __restrict__ todo) {
    __shared__ unsigned long long s_raw[kShardTableCap];   // workgroup 1: the gains; prefix workgroups: wavefront totals
    long long* s_tot = reinterpret_cast<long long*>(s_raw);
    if (blockIdx.x == 1) {
        if (depth == 0) return;
        if (shard_tables_match(key, g0, alpha0, beta0, depth, usable)) return;   // uniform: every thread reads the same key
        __syncthreads();      // all threads have read the key before it is cleared
        build_shard_tables(g0, alpha0, beta0, depth, usable, key, gain_table, surv_table, level_bits, level_kge, s_raw);
        return;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) todo[0] = 0;   // the list of left-over shards starts empty
    if (!prefix || blockIdx.x == 0) return;
    // Workgroup 2 + k: chunk k of `chunk` shards (a multiple of the workgroup size; at most
    // kPrefixGroups chunks).  It first adds up every budget before its chunk (independent loads,
    // sixteen in flight per thread), then scans its own chunk: thread t owns chunk / kPrefixThreads
    // consecutive shards.
    const long long base = (long long)(blockIdx.x - 2) * chunk;
    long long earlier = 0;
    {
        long long i = threadIdx.x;
        for (; i + 15 * kPrefixThreads < base; i += 16 * kPrefixThreads) {
            long long v[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) v[q] = shard_budget[i + q * kPrefixThreads];
#pragma unroll
            for (int q = 0; q < 16; ++q) earlier += v[q] > 0 ? v[q] : 0;
        }
        for (; i < base; i += kPrefixThreads) {
            const long long v = shard_budget[i];
            earlier += v > 0 ? v : 0;
        }
    }
    const int per = (int)(chunk / kPrefixThreads);
    const long long first = base + (long long)threadIdx.x * per;
    long long sum = 0;
    for (int k = 0; k < per; ++k) {
        const long long v = first + k < n_shards ? shard_budget[first + k] : 0;
        sum += v > 0 ? v : 0;
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
    for (int k = 0; k < per; ++k) {
        if (first + k < n_shards) {
            prefix[first + k] = run;
            const long long v = shard_budget[first + k];
            run += v > 0 ? v : 0;
        }
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
// that fall inside (every prompt walks its gains down to lo: from the state the pass before
// left for the first two prompts of a thread, from l = 0 for the others).  If the
// running count from the top reaches the budget inside interval j, the bracket
// shrinks to the gains that occur there, (min - 1, max], and closes when min == max:
// tau is that gain.  Otherwise the whole window lies above tau: it is added to
// `above` and the next window further down in value is taken (one exponent step of the
// bit pattern, or four: see `window` below).  Going down window by window keeps the walks
// short: a window's count is a small multiple of the one before it, so the work is a small
// multiple of the budget, whereas a bracket from a guaranteed lower bound (e.g. the
// smallest ceil(budget/n)-th gain) can lie orders of magnitude below tau.
// Counts fit 63 bits: n < 2^40 and one prompt has far fewer than 2^22 gains per window
// for any threshold a budget below 2^52 can reach.
constexpr int kResume = 2;   // prompts per thread whose walk states are kept from pass to pass
struct WalkResume {          // per thread: the first state at or below the last pass's hi (at or above tau)
    double g[kResume], l[kResume];
    bool valid;
};

template <class Src>
__device__ bool threshold_by_walks(const Src& src, long long lo_i, long long hi_i, long long budget, long long limit,
                                   ShardShared& sh, bool& data_bad, unsigned long long& tau_bits, WalkResume& rs) {
    const int lane = lane_id();
    // Every walk of a window goes down to the window's lower end, past tau in the window that
    // holds it: with windows of a factor 16 a walk takes up to 16^(1/(1+alpha)) times the steps
    // it needs.  Where every walk goes on from pass to pass (see below) a window costs only its
    // barriers, so the windows are single octaves; larger shards, whose later prompts walk from
    // l = 0 in every pass, keep the wide ones.
    const unsigned long long window = hi_i - lo_i <= (long long)kResume * kShardThreads ? kOctaveStep : kWindowStep;
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
        // A prompt's gains add up to less than 1, so fewer than 1 / t of them exceed t and tau <=
        // size / budget: the first window reaches down to the bottom of the octave that holds
        // 2^-lumped, where 2^lumped <= budget / size (from the leading bits: at most one too small).
        const long long size = hi_i - lo_i;
        const int lumped = (63 - __clzll(budget)) - (63 - __clzll(size)) - 1;   // (budget, size > 0 here)
        const unsigned long long first_lo = lumped > 0 ? 0x3ff0000000000000ull - (unsigned long long)(lumped + 1) * kOctaveStep : ~0ull;
        unsigned long long lo0 = all_top > window ? all_top - window : 0ull;
        if (first_lo < lo0) lo0 = first_lo;
        sh.lo = lo0;
        sh.above = 0;
        sh.done = 0;
    }
    __syncthreads();

    // The first kResume prompts of a thread (all of them up to 512 prompts per shard) do not walk
    // from l = 0 again in every pass: a pass leaves each walk's first state at or below its hi
    // and the state it ended in (the first at or below its lo).  A bracket only moves down, so
    // the next pass goes on from the former, or from the latter when the bracket has moved to
    // the window below (its hi is the last pass's lo).  What the last pass leaves serves the
    // caller's output walk too: tau is the last hi.
    double (&at_hi_g)[kResume] = rs.g, (&at_hi_l)[kResume] = rs.l;
    double at_lo_g[kResume], at_lo_l[kResume];
    bool resumable = false;                  // the states above are those of the pass before
    unsigned long long last_lo = 0ull;       // ... whose bracket ended here
    for (int pass = 0; pass < kShardMaxPasses; ++pass) {
        if (sh.done) break;   // uniform: written before the barrier that ends a pass
        const unsigned long long lo = sh.lo, hi_cur = sh.hi;
        const long long above = sh.above;
        const int shift = bracket_shift(lo, hi_cur);
        static_assert(kBins == kShardThreads, "one interval per thread");
        sh.bins.cnt[threadIdx.x] = 0; sh.bins.vmax[threadIdx.x] = 0; sh.bins.vmin_inv[threadIdx.x] = 0;
        __syncthreads();
        const bool from_lo = resumable && hi_cur <= last_lo;   // uniform
        // one round of the workgroup: a prompt per thread, walked from (g, lf) down to lo; every
        // wavefront runs whole rounds, so that the ballots see all of its lanes
        auto walk_round = [&](long long i0, bool resume, double g0_, double l0_, double& hi_g, double& hi_l,
                              double& lo_g, double& lo_l) {
            const long long i = i0 + threadIdx.x;
            double a = 1.0, b = 1.0;
            if (i < hi_i) src.load(i, a, b);
            const double s = a + b;
            double g = resume ? g0_ : gain_first(a, s);
            double lf = resume ? l0_ : 0.0;
            long long k = (long long)lf;
            unsigned long long gb = gain_bits(g);
            bool active = i < hi_i && k < limit && gb > lo;
            bool kept = gb <= hi_cur;
            hi_g = g; hi_l = lf;
            while (__ballot(active)) {
                tally_gains(sh.bins, active && gb <= hi_cur, gb, lo, shift);
                if (active) {
                    g = gain_next(g, b, s, lf);
                    lf += 1.0;
                    k += 1;
                    gb = gain_bits(g);
                    active = k < limit && gb > lo;
                    if (!kept) { hi_g = g; hi_l = lf; kept = gb <= hi_cur; }
                }
            }
            lo_g = g; lo_l = lf;
        };
#pragma unroll
        for (int r = 0; r < kResume; ++r) {
            const long long i0 = lo_i + (long long)r * kShardThreads;
            if (i0 < hi_i)   // uniform
                walk_round(i0, resumable, from_lo ? at_lo_g[r] : at_hi_g[r], from_lo ? at_lo_l[r] : at_hi_l[r],
                           at_hi_g[r], at_hi_l[r], at_lo_g[r], at_lo_l[r]);
        }
        for (long long i0 = lo_i + (long long)kResume * kShardThreads; i0 < hi_i; i0 += kShardThreads) {
            double unused[4];
            walk_round(i0, false, 0.0, 0.0, unused[0], unused[1], unused[2], unused[3]);
        }
        resumable = true;
        last_lo = lo;
        __syncthreads();   // the tallies are complete
        // interval j = kBins - 1 - thread: thread 0 owns the top interval
        const int j = kBins - 1 - (int)threadIdx.x;
        const long long cj = (long long)sh.bins.cnt[j];
        const unsigned long long mx = sh.bins.vmax[j], mn = ~sh.bins.vmin_inv[j];
        // running count from the top interval down (the barrier above lies between the last
        // reads of the wavefront totals and these writes)
        const long long incl = (long long)wave_incl_scan_u64((unsigned long long)cj);
        if (lane == kWave - 1) sh.red_i[0][wave_id()] = incl;
        __syncthreads();
        long long before = above + incl - cj, total = 0;
#pragma unroll
        for (int w = 0; w < kShardWaves; ++w) {
            const long long x = sh.red_i[0][w];
            if (w < wave_id()) before += x;
            total += x;
        }
        if (above + total < budget) {          // uniform: the whole window is above tau
            if (threadIdx.x == 0) {
                sh.above = above + total;
                sh.hi = lo;
                sh.lo = lo > window ? lo - window : 0ull;
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
    rs.valid = resumable;
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
    WalkResume rs;
    rs.valid = false;
    if (budget > 0) {
        if constexpr (Src::kHasClasses)
            if (depth > 0)
                by_table = threshold_by_table(src, lo_i, hi_i, budget, limit, depth, gain_table, surv_table, sh,
                                          data_bad, tau_bits);
        if (!by_table && !threshold_by_walks(src, lo_i, hi_i, budget, limit, sh, data_bad, tau_bits, rs)) {
            if (threadIdx.x == 0) report(dev_status, HORA_ERR_RANGE);
            return;
        }
    }

    // ---- k_i, tied flag and E_i(k_i) per prompt; totals --------------------------------
    long long ks = 0, ts = 0;
    int round = 0;
    for (long long i = lo_i + threadIdx.x; i < hi_i; i += kShardThreads, ++round) {
        long long k;
        bool tied;
        double e;
        if (by_table) {
            const int x = class_of(src, i);
            k = sh.k_cls[x];
            tied = sh.tied_cls[x] != 0;
            e = sh.e_cls[x];
        } else {
            // the walk goes on from where the search left it (the first prompts of a thread), else
            // from l = 0, down to the first gain M(k) at or below tau; the survival product follows
            // from that gain: E(k) = M(k) (alpha + beta + k) / alpha (App. A: the ratio of the closed
            // forms of M and E), E(0) = 1
            double a, b;
            data_bad |= !src.load(i, a, b);
            const double s = a + b;
            double g = gain_first(a, s), lf = 0.0;
#pragma unroll
            for (int q = 0; q < kResume; ++q)
                if (rs.valid && round == q) { g = rs.g[q]; lf = rs.l[q]; }
            k = (long long)lf;
            while (k < limit && gain_bits(g) > tau_bits) {
                g = gain_next(g, b, s, lf);
                lf += 1.0;
                k += 1;
            }
            e = k > 0 ? (g * (s + lf)) / a : 1.0;
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
    long long before = 0;   // units handed to the shards before this one (only the offsets need it)
    if (kOff != 0) {
        if (prefix) {
            before = prefix[shard];
        } else {            // few shards: the workgroup adds their budgets up itself
            __shared__ long long s_before[kShardWaves];
            for (long long t = threadIdx.x; t < shard; t += kShardThreads) {
                const long long v = shard_budget[t];
                before += v > 0 ? v : 0;
            }
            before = block_sum<long long>(before, s_before);
        }
    }
    shard_core<Src, kOff>(src, lo_i, hi_i, budget, before, n, g0, cap, depth, gain_table, surv_table, delta, util,
                          group_off, summary ? summary + shard : nullptr, dev_status);
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

// The shards the group kernel left over when it runs without its own fallback (todo[0] of them,
// ids from todo[1]): a fixed number of workgroups takes them in turn.
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
// Small shards (shared prior): L lanes per shard, 64 / L shards per wavefront (the paper's
// shards hold 15 prompts: four of them share a wavefront).  Every cross-lane step stays
// inside the shard's L lanes, so shards of one wavefront do not wait for one another beyond
// running in lockstep.
//  1. histogram of c: lane k of the group counts class k (wavefront ballots, the group's bits);
//  2. coarse search: the group's lanes evaluate count_ge of the last level of every block of
//     64 sorted levels (32 for 16-lane groups; coarse rows in LDS); the first block that
//     reaches the budget is taken; fine search: the block's levels, L at a time (one 32- or
//     128-byte row each from global memory).  tau is the first level whose count_ge reaches the budget; the level before it
//     gives the gains above tau per class;
//  3. outputs with the tie pass inside the group (ballot + mbcnt ranks, group prefix sums for
//     the offsets).
// A shard the tables cannot settle (deeper than the tables, more than kWaveShardMax prompts,
// or no tables yet) is handed to the workgroup-per-shard code.
//  kFused (few shards, one launch per call): the same workgroup runs that code after its
//    groups are through; every group adds up the budgets before its shard itself; and when
//    the workspace does not hold the tables for this prior yet, workgroup 0 builds them at the
//    end, for the calls that follow.
//  otherwise (many shards): such shards go on a list that k_shard_allocate_todo works off;
//    keeping that code out of this kernel more than halves its register count, and with tens
//    of thousands of groups in flight the occupancy is what hides their memory round trips.
// ----------------------------------------------------------------------------------
constexpr long long kInlineShards = 256;   // up to here a call has no set-up launch

template <int L> struct GroupScratch {   // per shard of the workgroup, LDS
    int k[L];
    int tied[L];
    double e[L];
};

// Cross-lane steps inside a group of L lanes.  A group of 16 lanes is one row of the DPP
// cross-lane path: rotations and shifts inside the row are register moves (no LDS crossbar
// trip, which is what the general shuffles cost); 64-bit values move as two halves.
template <int kCtrl, int kBankMask>
__device__ __forceinline__ long long row_take(long long v) {
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)((unsigned long long)v & 0xffffffffull), kCtrl, 0xf,
                                               kBankMask, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)((unsigned long long)v >> 32), kCtrl, 0xf,
                                               kBankMask, true);
    return (long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned long long)(unsigned)lo);
}
template <int kCtrl, int kBankMask>
__device__ __forceinline__ int row_take(int v) {
    return __builtin_amdgcn_update_dpp(0, v, kCtrl, 0xf, kBankMask, true);
}

// The bits of a wavefront ballot that belong to the lane's group of L lanes (sub = the group's
// slot in the wavefront), moved down to bit 0: a 32-bit value for the groups that fit one.
template <int L>
__device__ __forceinline__ unsigned group_bits(unsigned long long ballot, int sub) {
    static_assert(L == 16 || L == 32, "narrow groups");
    const unsigned w = (L == 32 ? sub : (sub >> 1)) ? (unsigned)(ballot >> 32) : (unsigned)ballot;
    if constexpr (L == 32) return w;
    else return (w >> ((sub & 1) * 16)) & 0xffffu;
}

__device__ __forceinline__ int count_bits(unsigned m) { return __popc(m); }
__device__ __forceinline__ int count_bits(unsigned long long m) { return __popcll(m); }
// bits of m below bit sl (sl < 32 for the 32-bit form)
__device__ __forceinline__ int count_below(unsigned m, int sl) { return __popc(m & ((1u << sl) - 1u)); }
__device__ __forceinline__ int count_below(unsigned long long m, int sl) { return __popcll(m & ((1ull << sl) - 1ull)); }

template <typename T, int L>
__device__ __forceinline__ T group_sum(T v) {
    if constexpr (L == 16 && (sizeof(T) == 4 || sizeof(T) == 8)) {
        typedef typename std::conditional<sizeof(T) == 4, int, long long>::type R;
        R x = (R)v;
        x += row_take<0x128, 0xf>(x);   // row_ror:8
        x += row_take<0x124, 0xf>(x);   // row_ror:4
        x += row_take<0x122, 0xf>(x);   // row_ror:2
        x += row_take<0x121, 0xf>(x);   // row_ror:1
        return (T)x;
    } else {
#pragma unroll
        for (int d = L / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, L);
        return v;
    }
}
template <int L>
__device__ __forceinline__ int group_max(int v) {
    if constexpr (L == 16) {
        int o = row_take<0x128, 0xf>(v); v = o > v ? o : v;
        o = row_take<0x124, 0xf>(v); v = o > v ? o : v;
        o = row_take<0x122, 0xf>(v); v = o > v ? o : v;
        o = row_take<0x121, 0xf>(v); v = o > v ? o : v;
        return v;
    } else {
#pragma unroll
        for (int d = L / 2; d > 0; d >>= 1) {
            const int o = __shfl_xor(v, d, L);
            v = o > v ? o : v;
        }
        return v;
    }
}
template <int L>
__device__ __forceinline__ int group_incl_scan(int v, int sl) {
    if constexpr (L == 16) {
        // shifts by 1, 2, 3 inside the row, then by 4 and 8 with bank masks (lanes without a source add 0)
        int t = v + row_take<0x111, 0xf>(v) + row_take<0x112, 0xf>(v) + row_take<0x113, 0xf>(v);
        t += row_take<0x114, 0xe>(t);
        t += row_take<0x118, 0xc>(t);
        return t;
    } else {
#pragma unroll
        for (int d = 1; d < L; d <<= 1) {
            const int o = __shfl_up(v, d, L);
            if (sl >= d) v += o;
        }
        return v;
    }
}
// The value of the group's last lane, in every lane of the group.
template <int L>
__device__ __forceinline__ int group_last(int v) {
    if constexpr (L == 16) {
        // lane 15 of the row: keep it alone, then the row's sum
        return group_sum<int, L>((lane_id() & 15) == 15 ? v : 0);
    } else {
        return __shfl(v, L - 1, L);
    }
}

template <int kOff, int L, bool kFused>
__global__ __launch_bounds__(kShardThreads, (L == 16 && !kFused) ? 8 : 1) void k_shard_allocate_waves(
    CountsSource src, long long n, long long n_shards, const long long* __restrict__ shard_off,
    const long long* __restrict__ shard_budget, int cap, const long long* __restrict__ prefix, int depth, int usable,
    ShardTableKey* __restrict__ key, double* __restrict__ gain_table, double* __restrict__ surv_table,
    unsigned long long* __restrict__ level_bits, unsigned short* __restrict__ level_kge, int* __restrict__ todo,
    int32_t* __restrict__ delta, double* __restrict__ util, void* __restrict__ group_off,
    hora_alloc_summary* __restrict__ summary, int32_t* dev_status) {
    constexpr int kPerWave = kWave / L;                  // shards per wavefront
    constexpr int kPerBlock = kShardWaves * kPerWave;    // shards per workgroup
    // (16 lanes are chosen for at most 16 classes: their rows have 16 entries)
    constexpr int kCoarseStride = L == 16 ? 16 : 64;
    // Levels per block.  A 16-lane group looks at a block's levels L at a time, and the kernel is
    // bound by its vector instructions: blocks of 32 levels (two rounds instead of four) for twice
    // the rows in LDS, which 32-byte rows can afford; of 16 levels (one round) where a call has few
    // shards and LDS does not limit how many wavefronts are resident (measured: 22.7 -> 20.9 us for
    // 65536 shards with 32, 21.5 us with 16; 5.7 -> 5.3 / 4.5 us for four shards).
    constexpr int kBlock = L == 16 ? (kFused ? 16 : 32) : kLevelBlock;
    constexpr int kRowsMax = kShardTableCap / kBlock;
    __shared__ __align__(16) unsigned short s_coarse[kRowsMax * kCoarseStride];
    __shared__ GroupScratch<L> s_group[kPerBlock];
    __shared__ int s_left[kPerBlock];
    __shared__ int s_left_n, s_tables;
    const int g0 = src.g0;
    const int nc = g0 + 1;                               // (the host picks L >= nc)
    const int stride = L == 16 ? 16 : level_stride(nc);
    const int levels = nc * usable;
    const int n_coarse = (levels + kBlock - 1) / kBlock;
    const int lane = lane_id();
    const int sub = lane / L, sl = lane % L;             // the shard's slot in the wavefront, the lane in the group
    const long long first_shard = (long long)blockIdx.x * kPerBlock;
    const int slot = wave_id() * kPerWave + sub;
    const long long shard = first_shard + slot;
    const bool live = shard < n_shards;
    // the shard's bounds and budget are requested first, so that they travel while the coarse
    // rows are staged (coarse row q = the last level of block q)
    const long long lo_i = live ? shard_off[shard] : 0, hi_i = live ? shard_off[shard + 1] : 0;
    const long long budget = live ? shard_budget[shard] : 0;
    long long before = 0;                                // units of the shards before this one
    if (kOff != 0 && live) {
        if (prefix) {
            before = prefix[shard];
        } else {
            for (long long t = sl; t < shard; t += L) {
                const long long v = shard_budget[t];
                before += v > 0 ? v : 0;
            }
        }
    }
    if (kOff != 0 && !prefix) before = group_sum<long long, L>(before);
    if (threadIdx.x == 0) {
        s_left_n = 0;
        s_tables = shard_tables_match(key, g0, src.alpha0, src.beta0, depth, usable) ? 1 : 0;
    }
    // The coarse rows are requested before it is known whether the workspace holds the tables
    // (rows of 16 classes, two 16-byte pieces each, kEarly pieces per thread): the answer and the
    // rows travel together, and rows of a workspace without tables are dropped.
    constexpr int kEarly = (kRowsMax * 2 + kShardThreads - 1) / kShardThreads;
    const bool early_rows = stride == 16;
    uint4 early[kEarly];
#pragma unroll
    for (int i = 0; i < kEarly; ++i) {
        const int piece = i * kShardThreads + (int)threadIdx.x;
        early[i] = uint4{0u, 0u, 0u, 0u};
        if (early_rows && piece < n_coarse * 2) {
            int p = (piece >> 1) * kBlock + kBlock - 1;
            if (p > levels - 1) p = levels - 1;
            early[i] = reinterpret_cast<const uint4*>(level_kge + (long long)p * 16)[piece & 1];
        }
    }
    __syncthreads();
    const bool tables = s_tables != 0;
    if (tables && early_rows) {
#pragma unroll
        for (int i = 0; i < kEarly; ++i) {
            const int piece = i * kShardThreads + (int)threadIdx.x;
            if (piece < n_coarse * 2) reinterpret_cast<uint4*>(s_coarse)[piece] = early[i];
        }
    } else if (tables) {
        for (int idx = (int)threadIdx.x; idx < n_coarse * stride; idx += kShardThreads) {
            const int q = idx / stride, k = idx - q * stride;
            int p = q * kBlock + kBlock - 1;
            if (p > levels - 1) p = levels - 1;
            s_coarse[idx] = level_kge[(long long)p * stride + k];
        }
    }
    __syncthreads();
    GroupScratch<L>& gs = s_group[slot];
    // a ballot restricted to the group's lanes, from bit 0 (32 bits wide for the narrow groups)
    auto group_ballot = [&](bool p) {
        if constexpr (L == kWave) return (unsigned long long)__ballot(p);
        else return group_bits<L>(__ballot(p), sub);
    };
    bool defer = false;        // the workgroup-per-shard code has to take the shard
    if (live) {
        const int wrong = check_shard(shard, n_shards, n, lo_i, hi_i, budget, cap);
        const long long size = hi_i - lo_i;
        if (wrong != HORA_OK) {
            if (sl == 0) report(dev_status, wrong);
        } else if (!tables || size > kWaveShardMax) {
            defer = true;
        } else {
            const long long limit = cap > 0 ? (budget < cap ? budget : (long long)cap) : budget;   // (the tables are far shallower than the depth bound)
            // ---- 1. histogram: lane k of the group ends up with the number of prompts of class k;
            // groups narrower than a wavefront also keep all of their counts in every lane's
            // registers (at most L of them), which saves the shuffles below
            constexpr int kRegs = L < kWave ? L : 1;
            int n_mine = 0;
            int n_all[kRegs];
#pragma unroll
            for (int k = 0; k < kRegs; ++k) n_all[k] = 0;
            bool data_bad = false;
            int x_first = 0;   // this lane's prompt of the shard's first L prompts (read once, used again for the outputs)
            for (long long i0 = lo_i; i0 < hi_i; i0 += L) {
                const long long i = i0 + sl;
                int x = -1;
                if (i < hi_i) {
                    x = src.c[i];
                    if (x < 0 || x > g0) { data_bad = true; x = x < 0 ? 0 : g0; }
                }
                if (i0 == lo_i) x_first = x < 0 ? 0 : x;
                if constexpr (L < kWave) {
#pragma unroll
                    for (int k = 0; k < L; ++k)
                        if (k < nc) {   // uniform
                            const int cnt = count_bits(group_ballot(x == k));
                            n_all[k] += cnt;
                            if (sl == k) n_mine += cnt;
                        }
                } else {
                    for (int k = 0; k < nc; ++k) {
                        const int cnt = __popcll(__ballot(x == k));
                        if (sl == k) n_mine += cnt;
                    }
                }
            }
            if (data_bad) report(dev_status, HORA_ERR_RANGE);
            // the group's count of class k: a register, or lane k's value (a whole wavefront: scalar read)
            auto count_of = [&](int k) -> unsigned {
                if constexpr (L < kWave) return (unsigned)n_all[k];
                else return (unsigned)__builtin_amdgcn_readlane(n_mine, k);
            };
            // count_ge of a level from its row of per-class counts.  A shard here has at most 2^10
            // prompts and a class at most 2^9 gains in the tables: a count fits 32 bits, and a
            // class costs one 24-bit multiply-add.  A row of 16 classes comes as two 16-byte pieces.
            auto count_row16 = [&](const uint4& r0, const uint4& r1) -> int {
                const unsigned w[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
                unsigned sum = 0u;
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const unsigned kge = (k & 1) ? (w[k >> 1] >> 16) : (w[k >> 1] & 0xffffu);
                    if ((L == kWave || k < L) && k < nc) sum = __umul24(count_of(L == kWave || k < L ? k : 0), kge) + sum;   // uniform
                }
                return (int)sum;
            };
            auto count_row = [&](const unsigned short* row) -> int {
                unsigned sum = 0u;
                if constexpr (L < kWave) {
#pragma unroll
                    for (int k = 0; k < L; ++k)
                        if (k < nc) sum = __umul24(count_of(k), (unsigned)row[k]) + sum;   // uniform
                } else {
                    for (int k = 0; k < nc; ++k) sum = __umul24(count_of(k), (unsigned)row[k]) + sum;
                }
                return (int)sum;
            };

            // ---- 2. threshold
            int k_mine = 0, tied_mine = 0;            // lane c of the group: gains of class c above tau; its next gain equals tau
            double e_mine = 1.0;                      // E_c(k_c)
            int count_gt = 0, tie_prompts = 0;
            unsigned long long tau_bits = 0;
            bool ok = true;
            const int want = budget < (long long)INT_MAX ? (int)budget : INT_MAX;   // the budget as far as a count can reach
            if (budget > 0) {
                // coarse: the group's lanes share the blocks; the first block whose last level reaches the budget
                int block = INT_MAX;
                int below = 0;                        // largest coarse count that stays under the budget
                for (int q0 = 0; q0 < n_coarse; q0 += L) {
                    const int q = q0 + sl;
                    const bool in = q < n_coarse;
                    int cq = 0;
                    if (stride == 16) {
                        // (lanes past the last block read its row and drop the result)
                        const int qr = in ? q : n_coarse - 1;
                        cq = count_row16(*reinterpret_cast<const uint4*>(s_coarse + qr * 16),
                                         *reinterpret_cast<const uint4*>(s_coarse + qr * 16 + 8));
                    } else if (in) {
                        cq = count_row(s_coarse + q * stride);
                    }
                    const bool reached = in && cq >= want;
                    if (reached) block = q < block ? q : block;
                    if (in && cq < want) below = cq > below ? cq : below;
                    // the counts grow with the level: once every group of the wavefront has a block
                    // that reaches its budget, the blocks further down cannot be the first
                    if (__ballot(group_ballot(reached) == 0) == 0ull) break;
                }
                block = -group_max<L>(-block);                        // the smallest over the group
                const int before_block = group_max<L>(below);         // the counts grow with the level: this is block - 1's
                if (block == INT_MAX) {
                    ok = false;                       // the tables do not reach the budget
                } else {
                    // fine: the levels of the block, kBlock / L per lane
                    int under = 0;                    // levels of the block whose count stays under the budget
                    int best = before_block;          // ... and the largest such count
                    for (int t0 = 0; t0 < kBlock; t0 += L) {
                        const int lvl = block * kBlock + t0 + sl;
                        const bool in = lvl < levels;
                        // (lanes past the last level read its row and drop the result)
                        const unsigned short* row = level_kge + (long long)(in ? lvl : levels - 1) * stride;
                        int ct;
                        if (stride == 16)
                            ct = count_row16(*reinterpret_cast<const uint4*>(row), *reinterpret_cast<const uint4*>(row + 8));
                        else
                            ct = count_row(row);
                        if (in && ct < want) { under += 1; best = ct > best ? ct : best; }
                    }
                    const int t = group_sum<int, L>(under);                // the first level that reaches the budget
                    const int j = block * kBlock + t;                      // tau = level j
                    count_gt = group_max<L>(best);
                    tau_bits = level_bits[j];
                    if (sl < nc) {
                        const int ge = level_kge[(long long)j * stride + sl];
                        const int gt = j > 0 ? level_kge[(long long)(j - 1) * stride + sl] : 0;
                        k_mine = gt;
                        tied_mine = ge - gt;
                        // every usable gain of a class the shard holds is above tau and the sequence
                        // goes on beyond the tables: gains are missing from the counts
                        if (n_mine > 0 && gt == usable && (long long)usable < limit) ok = false;
                        const double a = src.alpha0 + (double)sl, b = src.beta0 + (double)(g0 - sl);
                        double e = surv_table[sl * depth + (gt < depth ? gt : depth - 1)];
                        if (gt == depth) e = surv_next(e, b, a + b, (double)(depth - 1));
                        e_mine = e;
                    }
                    ok = group_ballot(!ok) == 0;
                    tie_prompts = group_sum<int, L>(tied_mine ? n_mine : 0);
                }
            }
            if (!ok) {
                defer = true;
            } else {
                const long long r64 = budget - (long long)count_gt;
                const int r = r64 < (long long)INT_MAX ? (int)r64 : INT_MAX;   // tied prompts that get a unit (ranks are below 2^10)
                if (summary && sl == 0) {
                    summary[shard].tau = budget > 0 ? __longlong_as_double((long long)tau_bits) : 0.0;
                    summary[shard].count_gt = count_gt;
                    summary[shard].tie_units = r64;
                    summary[shard].tie_prompts = tie_prompts;
                }
                gs.k[sl] = k_mine;
                gs.tied[sl] = tied_mine;
                gs.e[sl] = e_mine;
                // (the group's own lanes read them back below: a wavefront's LDS operations complete in order)

                // ---- 3. outputs
                const long long off_base = kOff != 0 ? (long long)g0 * lo_i + before : 0;
                int rank_base = 0, given = 0;             // tied prompts / units handed out before this tile (32 bits: see above)
                for (long long i0 = lo_i; i0 < hi_i; i0 += L) {
                    const long long i = i0 + sl;
                    const bool in = i < hi_i;
                    int x = 0;
                    if (i0 == lo_i) {
                        x = x_first;
                    } else if (in) {
                        x = src.c[i];
                        x = x < 0 ? 0 : (x > g0 ? g0 : x);
                    }
                    const int kk = in ? gs.k[x] : 0;
                    const bool td = in && gs.tied[x] != 0;
                    const auto tied_mask = group_ballot(td);
                    const int rank = rank_base + count_below(tied_mask, sl);
                    const bool win = td && rank < r;
                    const int dd = kk + (win ? 1 : 0);
                    const int units = in ? g0 + dd : 0;
                    const int incl = group_incl_scan<L>(units, sl);
                    if (in) {
                        delta[i] = dd;
                        if (util) {
                            double e = gs.e[x];
                            if (win) {
                                const double a = src.alpha0 + (double)x, b = src.beta0 + (double)(g0 - x);
                                e = surv_next(e, b, a + b, (double)kk);
                            }
                            util[i] = 1.0 - e;
                        }
                        if (kOff != 0) {
                            const long long off = off_base + (long long)(given + incl - units);
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
                    rank_base += count_bits(tied_mask);
                    given += group_last<L>(incl);
                }
            }
        }
    }
    if constexpr (!kFused) {
        if (defer && sl == 0) todo[1 + atomicAdd(&todo[0], 1)] = (int)shard;
    } else {
        // ---- the shards that are left: one after the other, the whole workgroup on each
        if (defer && sl == 0) s_left[atomicAdd(&s_left_n, 1)] = slot;
        __syncthreads();
        const int left = s_left_n;
        for (int idx = 0; idx < left; ++idx) {
            shard_by_workgroup<CountsSource, kOff>(src, first_shard + s_left[idx], n, g0, n_shards, shard_off,
                                                   shard_budget, cap, prefix, tables ? depth : 0, gain_table,
                                                   surv_table, delta, util, group_off, summary, dev_status);
            __syncthreads();   // the LDS state is reused by the next shard
        }
        // ---- no tables yet: workgroup 0 leaves them for the next call
        if (!tables && blockIdx.x == 0 && depth > 0)
            build_shard_tables(g0, src.alpha0, src.beta0, depth, usable, key, gain_table, surv_table, level_bits,
                               level_kge, nullptr);
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
    if (group_off && n == 0) hipLaunchKernelGGL(k_store_zero_offset, 1, 1, 0, s, group_off, off_t == HORA_I64 ? 1 : 0);
    CountsSource src{c, g0, alpha0, beta0};
    const int cap = delta_max > 0 ? delta_max : 0;
    const int mode = group_off ? (off_t == HORA_I32 ? 1 : 2) : 0;
    const int nc = g0 + 1;
    // small shards: L lanes per shard; what the tables cannot settle is taken by the same
    // workgroup with the workgroup-per-shard code
    const bool waves = depth > 0 && n <= (long long)n_shards * kWaveShardMeanMax;
    // few shards: no set-up launch (the groups add up the earlier budgets themselves; tables that
    // are missing are built at the end of the call, for the next one)
    const bool inline_setup = waves && n_shards <= kInlineShards;
    if (!inline_setup) {
        // shards per prefix-sum workgroup: a multiple of the workgroup size, at most kPrefixGroups workgroups
        long long chunk = (n_shards + kPrefixGroups - 1) / kPrefixGroups;
        chunk = (chunk + kPrefixThreads - 1) / kPrefixThreads * kPrefixThreads;
        const unsigned setup_blocks = 2 + (group_off ? (unsigned)((n_shards + chunk - 1) / chunk) : 0u);
        hipLaunchKernelGGL(k_shard_setup, dim3(setup_blocks), dim3(kPrefixThreads), 0, s, (long long)n_shards, chunk,
                           (const long long*)shard_budget, prefix, (int)g0, alpha0, beta0, depth, usable, w.key,
                           w.gain_table, w.surv_table, w.level_bits, w.level_kge, w.todo);
    } else {
        prefix = nullptr;
    }
    if (waves) {
        const long long mean = n_shards > 0 ? (n + n_shards - 1) / n_shards : 0;
        const int lanes = (nc <= 16 && mean <= 16) ? 16 : (nc <= 32 && mean <= 32) ? 32 : 64;
#define HORA_LAUNCH_WAVES(M, LL, FUSED)                                                                          \
    do {                                                                                                          \
        const long long per_block = (long long)kShardWaves * (kWave / LL);                                        \
        const unsigned blocks = (unsigned)((n_shards + per_block - 1) / per_block);                               \
        hipLaunchKernelGGL((k_shard_allocate_waves<M, LL, FUSED>), dim3(blocks), dim3(kShardThreads), 0, s, src,   \
                           (long long)n, (long long)n_shards, (const long long*)shard_off,                        \
                           (const long long*)shard_budget, cap, (const long long*)prefix, depth, usable, w.key,   \
                           w.gain_table, w.surv_table, w.level_bits, w.level_kge, w.todo, delta, util, group_off, \
                           summary, dev_status);                                                                  \
    } while (0)
#define HORA_LAUNCH_WAVES_L(M, FUSED)                               \
    do {                                                            \
        if (lanes == 16) HORA_LAUNCH_WAVES(M, 16, FUSED);           \
        else if (lanes == 32) HORA_LAUNCH_WAVES(M, 32, FUSED);      \
        else HORA_LAUNCH_WAVES(M, 64, FUSED);                       \
    } while (0)
#define HORA_LAUNCH_WAVES_F(M)                                      \
    do {                                                            \
        if (inline_setup) HORA_LAUNCH_WAVES_L(M, true);             \
        else HORA_LAUNCH_WAVES_L(M, false);                         \
    } while (0)
        if (mode == 0) HORA_LAUNCH_WAVES_F(0);
        else if (mode == 1) HORA_LAUNCH_WAVES_F(1);
        else HORA_LAUNCH_WAVES_F(2);
#undef HORA_LAUNCH_WAVES_F
#undef HORA_LAUNCH_WAVES_L
#undef HORA_LAUNCH_WAVES
        if (!inline_setup) {   // the shards the groups could not settle (usually none)
            const unsigned todo_blocks = (unsigned)(n_shards < 1024 ? n_shards : 1024);
#define HORA_LAUNCH_TODO(M)                                                                                         \
    hipLaunchKernelGGL((k_shard_allocate_todo<CountsSource, M>), dim3(todo_blocks), dim3(kShardThreads), 0, s, src, \
                       (long long)n, (int)g0, (long long)n_shards, (const long long*)shard_off,                    \
                       (const long long*)shard_budget, cap, (const long long*)prefix, depth,                       \
                       (const double*)w.gain_table, (const double*)w.surv_table, delta, util, group_off, summary,  \
                       (const int*)w.todo, dev_status)
            if (mode == 0) HORA_LAUNCH_TODO(0);
            else if (mode == 1) HORA_LAUNCH_TODO(1);
            else HORA_LAUNCH_TODO(2);
#undef HORA_LAUNCH_TODO
        }
    } else {
#define HORA_LAUNCH_SHARDS(M)                                                                                   \
    hipLaunchKernelGGL((k_shard_allocate<CountsSource, M>), dim3((unsigned)n_shards), dim3(kShardThreads), 0, s, \
                       src, (long long)n, (int)g0, (long long)n_shards, (const long long*)shard_off,            \
                       (const long long*)shard_budget, cap, (const long long*)prefix, depth,                    \
                       (const double*)w.gain_table, (const double*)w.surv_table, delta, util, group_off,        \
                       summary, dev_status)
        if (mode == 0) HORA_LAUNCH_SHARDS(0);
        else if (mode == 1) HORA_LAUNCH_SHARDS(1);
        else HORA_LAUNCH_SHARDS(2);
#undef HORA_LAUNCH_SHARDS
    }
    return hipGetLastError() == hipSuccess ? HORA_OK : HORA_ERR_HIP;
}
