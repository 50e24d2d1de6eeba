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
#include "hora_alloc_emit.h"

namespace hora {

// (table entry, class) pairs ranked one per thread when a round or two of the workgroup cover them
// (G0 = 4 with rows of 32: 800 pairs, 13.8 us against 14.4 us); beyond that a thread per entry
// that searches four rows at a time is faster (G0 = 8 with rows of 128: 10 368 pairs, 22 us
// against 26 us)
constexpr int kPairCap = 2048;

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
// CLASS pass 1: per-workgroup histogram of c (lane k of every wavefront accumulates the
// count of class k from wavefront ballots), and, in one extra workgroup, the gain and
// survival tables of the G0+1 classes.
// ----------------------------------------------------------------------------------
__global__ __launch_bounds__(kBig) void k_class_hist(const int32_t* __restrict__ c, long long n, int g0,
                                                     double alpha0, double beta0, long long chunk, int nb, int row,
                                                     int* __restrict__ class_hist, double* __restrict__ gain_table,
                                                     double* __restrict__ surv_table, int32_t* dev_status) {
    __shared__ int s_cnt[kBigWaves][kWave];
    const int lane = lane_id();
    if ((int)blockIdx.x == nb) {
        // the extra workgroup: tables, one lane per class and sequence (a row is one chain of
        // divisions: the gains on the first wavefront, the survival products on the second, so
        // that the two chains of a class run side by side on two vector units)
        static_assert(kMaxClasses <= kWave, "a wavefront holds a lane per class");
        if (wave_id() < 2 && lane <= g0) {
            const double a = alpha0 + (double)lane;
            const double b = beta0 + (double)(g0 - lane);
            const double s = a + b;
            double lf = 0.0;
            if (wave_id() == 0) {   // uniform per wavefront
                double m = gain_first(a, s);
                double* grow = gain_table + (long long)lane * row;
                for (int l = 0; l < row; ++l) {
                    grow[l] = m;
                    m = gain_next(m, b, s, lf);
                    lf += 1.0;
                }
            } else {
                double e = 1.0;
                double* srow = surv_table + (long long)lane * row;
                for (int l = 0; l < row; ++l) {
                    srow[l] = e;
                    e = surv_next(e, b, s, lf);
                    lf += 1.0;
                }
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
    unsigned kt[kMaxClasses];  // gains of the class above tau, with kTiedBit when its next gain equals tau
    double u0[kMaxClasses];   // U_c(k_c)
    double u1[kMaxClasses];   // U_c(k_c + 1)
    long long tied_before;    // tied prompts in the workgroups before this one
    long long units_before;   // sum of k over the prompts of the workgroups before this one
};

// What the workgroups before this one hold, from the per-class counts of their prompts: run by
// the first wavefront (lane c: class c with its k and tied flag; other lanes pass zeros) at the
// end of a solver, so that the sixteen wavefronts do not each add up the same numbers.
__device__ __forceinline__ void sums_before(ClassSolution* sol, const long long* s_before, bool has, int k, bool tied) {
    const long long bef = has ? s_before[lane_id()] : 0;
    const long long tb = wave_total_i64(tied ? bef : 0);
    const long long ub = (long long)wave_total_u64((unsigned long long)(bef * k));   // (up to the budget: beyond the two-piece sums)
    if (lane_id() == 0) { sol->tied_before = tb; sol->units_before = ub; }
}

// #{l : row[l] > v} for a decreasing row of `row_len` (power of two) entries whose last
// entry is not above v.
__device__ __forceinline__ int row_count_above(const double* row, int row_len, unsigned long long v) {
    int pos = 0;
    for (int step = row_len >> 1; step > 0; step >>= 1)
        if (gain_bits(row[pos + step - 1]) > v) pos += step;
    return pos;
}

__device__ void solve_by_table(int nc, int row_len, int len, bool rows_end_at_cap, long long budget,
                               const long long* s_n, const long long* s_before, const double* s_gain,
                               const double* s_surv, unsigned short* s_pair, ClassSolution* sol) {
    // (sol->found is cleared by the caller before the barrier that precedes this call)
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
        if (wave_id() == 0) {
            const int cls = lane_id();
            const bool has = sol->found && cls < nc;
            int pos = 0;
            bool tied = false;
            if (has) {
                const int pr = s_pair[sol->win * nc + cls];
                pos = pr & 0x7fff;
                tied = (pr & 0x8000) != 0;
                sol->kt[cls] = (unsigned)pos | (tied ? kTiedBit : 0u);
                sol->u0[cls] = 1.0 - s_surv[cls * row_len + pos];
                sol->u1[cls] = 1.0 - s_surv[cls * row_len + (pos + 1 < row_len ? pos + 1 : pos)];
            }
            sums_before(sol, s_before, has, pos, tied);
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
    if (wave_id() == 0) {
        const int c = lane_id();
        const bool has = sol->found && c < nc;
        int cnt = 0;
        bool tied = false;
        if (has) {
            const double* row = s_gain + c * row_len;
            cnt = row_count_above(row, row_len, sol->tau_bits);
            tied = gain_bits(row[cnt]) == sol->tau_bits;
            sol->kt[c] = (unsigned)cnt | (tied ? kTiedBit : 0u);
            sol->u0[c] = 1.0 - s_surv[c * row_len + cnt];
            sol->u1[c] = 1.0 - s_surv[c * row_len + (cnt + 1 < row_len ? cnt + 1 : cnt)];
        }
        sums_before(sol, s_before, has, cnt, tied);
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
                                long long budget, const long long* s_n, const long long* s_before,
                                ClassSolution* sol, int32_t* dev_status) {
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
        sol->kt[lane] = has ? ((unsigned)k | (tied ? kTiedBit : 0u)) : 0u;
        sol->u0[lane] = 1.0 - e;
        sol->u1[lane] = 1.0 - surv_next(e, b, s, lf);
        sums_before(sol, s_before, has, has ? (int)k : 0, has && tied);
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
                              long long budget, const long long* s_n, const long long* s_before, ClassSolution* sol,
                              int32_t* dev_status) {
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
        sol->kt[lane] = (unsigned)k | (mine ? kTiedBit : 0u);
        sol->u0[lane] = 1.0 - e;
        sol->u1[lane] = 1.0 - surv_next(e, b, s, lf);
        sums_before(sol, s_before, has, (int)k, mine);
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
// kCap: doubles of LDS per table, kTableCap or half of it (the host's choice by the tables'
// size: the common small tables do not pay for the room of the large ones).
template <int kOff, int kCap>
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
    static_assert(kCap == kTableCap || kCap == kTableCap / 2, "table room");
    __shared__ double s_gain[kCap];
    __shared__ double s_surv[kCap];
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
    constexpr int kTableLoads = kCap / kBig;                        // table entries per thread
    constexpr int kClassRounds = kMaxClasses / kBigWaves;           // classes per wavefront: a class's counts are one 1 KB row
    static_assert(kMaxBlocks == 4 * kWave && kMaxClasses % kBigWaves == 0, "a wavefront reads a class's row as 16-byte pieces");
    const int table_len = nc * row_len;
    double tg[kTableLoads], ts[kTableLoads];
    v4i hh[kClassRounds];
#pragma unroll
    for (int q = 0; q < kTableLoads; ++q) {
        const int i = q * kBig + (int)threadIdx.x;
        tg[q] = 0.0; ts[q] = 0.0;
        if (q * kBig < table_len) {   // uniform: small tables skip the later rounds
            tg[q] = i < table_len ? gain_table[i] : 0.0;
            ts[q] = i < table_len ? surv_table[i] : 0.0;
        }
    }
#pragma unroll
    for (int q = 0; q < kClassRounds; ++q) {
        const int cls = wave_id() + kBigWaves * q;
        v4i v = {0, 0, 0, 0};
        if (cls < nc) v = *reinterpret_cast<const v4i*>(class_hist + cls * kMaxBlocks + lane * 4);   // uniform per wavefront
        hh[q] = v;
    }
    int first_tile[kItems];
    load_items_i32(c, base + (long long)threadIdx.x * kItems, end, c_vec, -1, first_tile);

    // tables into LDS, gains beyond `len` replaced by zeros
#pragma unroll
    for (int q = 0; q < kTableLoads; ++q) {
        const int i = q * kBig + (int)threadIdx.x;
        if (q * kBig < table_len && i < table_len) {
            s_gain[i] = (i & (row_len - 1)) < len ? tg[q] : 0.0;
            s_surv[i] = ts[q];
        }
    }

    // class totals and the part that lies before this workgroup: a wavefront adds up the
    // kMaxBlocks counts of its class, four per lane (entries of workgroups that do not exist
    // are whatever an earlier call left there: masked)
#pragma unroll
    for (int q = 0; q < kClassRounds; ++q) {
        const int cls = wave_id() + kBigWaves * q;
        if (cls < nc) {   // uniform per wavefront
            const int e[4] = {hh[q].x, hh[q].y, hh[q].z, hh[q].w};
            long long tot = 0, bef = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int b = lane * 4 + i;
                tot += b < nb ? (long long)e[i] : 0ll;
                bef += b < (int)blockIdx.x ? (long long)e[i] : 0ll;   // (blockIdx.x < nb)
            }
            tot = wave_total_i64(tot);
            bef = wave_total_i64(bef);
            if (lane == 0) { s_n[cls] = tot; s_before[cls] = bef; }
        }
    }
    if (threadIdx.x == 0) s_sol.found = 0;   // (for solve_by_table)
    __syncthreads();

    if (budget > 0 && rule != 0) {
        solve_by_rule(rule, g0, alpha0, beta0, cap_eff, depth_capped, budget, s_n, s_before, &s_sol, dev_status);
    } else if (budget > 0) {
        solve_by_table(nc, row_len, len, rows_end_at_cap, budget, s_n, s_before, s_gain, s_surv, s_pair, &s_sol);
        if (!s_sol.found)
            solve_by_greedy(g0, alpha0, beta0, cap_eff, depth_capped, budget, s_n, s_before, &s_sol, dev_status);
    } else {
        if (threadIdx.x < kMaxClasses) {
            s_sol.kt[threadIdx.x] = 0u;
            s_sol.u0[threadIdx.x] = 0.0;
            s_sol.u1[threadIdx.x] = 0.0;
        }
        if (threadIdx.x == 0) {
            s_sol.tau_bits = 0; s_sol.r = 0; s_sol.tie_prompts = 0; s_sol.found = 1;
            s_sol.tied_before = 0; s_sol.units_before = 0;
        }
        __syncthreads();
    }
    const long long r = s_sol.r;
    if (summary && blockIdx.x == 0 && threadIdx.x == 0) {
        summary->tau = __longlong_as_double((long long)s_sol.tau_bits);
        summary->count_gt = budget - r;
        summary->tie_units = r;
        summary->tie_prompts = s_sol.tie_prompts;
    }

    EmitCarry carry = {s_sol.tied_before, s_sol.units_before};   // what the workgroups before this one hold

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
                const unsigned kt = s_sol.kt[x];
                kk[j] = (int)(kt & ~kTiedBit);
                td[j] = (kt & kTiedBit) ? 1 : 0;
            } else {
                cls[j] = 0; kk[j] = 0; td[j] = 0;
            }
        }
        emit_tile<kOff>(parity, pos, end, n, g0, r, kk, td, carry, dd, win, delta, group_off, d_vec, o_vec,
                        &s_emit);
        if (util) {
            double uu[kItems];
#pragma unroll
            for (int j = 0; j < kItems; ++j) uu[j] = (win[j] ? s_sol.u1 : s_sol.u0)[cls[j]];   // (one LDS read)
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
#define HORA_LAUNCH_CLASS_WRITE(M, CAP)                                                                         \
    hipLaunchKernelGGL((k_class_write<M, CAP>), dim3(p.nb), dim3(kBig), 0, a.stream, c, (long long)a.n,     \
                       (int)a.g0, alpha0, beta0, (long long)a.budget, cap, p.chunk, p.nb, row, w.class_hist,   \
                       w.gain_table, w.surv_table, a.delta, a.util, a.group_off, a.summary, a.dev_status, rule)
#define HORA_LAUNCH_CLASS_WRITE_BY_SIZE(M)                               \
    do {                                                                 \
        if (nc * row <= kTableCap / 2) HORA_LAUNCH_CLASS_WRITE(M, kTableCap / 2); \
        else HORA_LAUNCH_CLASS_WRITE(M, kTableCap);                      \
    } while (0)
    if (mode == 0) HORA_LAUNCH_CLASS_WRITE_BY_SIZE(0);
    else if (mode == 1) HORA_LAUNCH_CLASS_WRITE_BY_SIZE(1);
    else HORA_LAUNCH_CLASS_WRITE_BY_SIZE(2);
#undef HORA_LAUNCH_CLASS_WRITE_BY_SIZE
#undef HORA_LAUNCH_CLASS_WRITE
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
    Workspace w = carve(nullptr, n);
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
    if (n >= 0 && g0 >= 0 && carve(nullptr, n).bytes > kStaticScratchBytes) return HORA_ERR_UNSUPPORTED;
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
    Workspace w = carve(workspace, n);
    if (workspace_bytes < w.bytes) return HORA_ERR_WORKSPACE;
    const Plan p = make_plan(n);
    if (method == HORA_ALLOC_BISECT) {
        CountsSource src{c, g0, alpha0, beta0};
        return run_bisect_counts(src, a, p, w);
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
    Workspace w = carve(workspace, n);
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
    Workspace w = carve(workspace, n);
    if (workspace_bytes < w.bytes) return HORA_ERR_WORKSPACE;
    const Plan p = make_plan(n);
    PosteriorSource src{alpha, beta};
    return run_bisect_posterior(src, a, p, w);
}

}  // extern "C"
