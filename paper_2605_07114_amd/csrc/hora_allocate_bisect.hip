// Phase-B allocation by threshold search, for any posterior (Sec. 3.2 Eq. 4, Alg. 1 Phase B,
// Prop. 1; App. D for per-prompt posteriors).
//
// By Prop. 1 the allocation is the set of the `budget` largest marginal gains over all
// (prompt, l) pairs; every prompt's gains decrease strictly, so the set is described by a
// threshold tau, the budget-th largest gain.  tau is found by a bisection on its bit pattern
// (positive binary64 values order like their patterns) in which every prompt does a monotone
// search along its own gain sequence.  Six launches do it for any input, and a prompt's
// sequence is walked once: each kernel leaves the state of every walk (a gain and its index l)
// for the next one to go on from.
//
//  1. coarse count (k_bisect_coarse): a sample of the batch says roughly how deep tau lies
//     (estimate_depth; it steers the work, nothing relies on it).  Every tile of 4096 prompts
//     walks its prompts' gains down to that depth in one go, counting them per quarter octave
//     (an octave = one exponent step of the pattern), and goes on octave by octave until the
//     tile has seen its share of the budget.  If every tile selected its share on its own, the
//     union would hold at least `budget` gains, all of them above the lowest tile's stopping
//     point: that point is a lower bound for tau, whatever the data, and no prompt walks much
//     deeper than tau.  A wavefront walks four prompts per lane in lockstep and regroups the
//     walks that are still active as the others end (regroup_plan), or, for deep budgets with
//     a few very deep prompts, hands its prompts to its lanes one by one (pooled_walk).
//  2. first narrowing pass (k_bisect_pass<0>): every workgroup adds the tiles' counts up for
//     itself and takes the quarter octave in which the running count reaches the budget as the
//     first bracket (lo, hi] of tau; the bracket is cut into 256 intervals, the gains inside are
//     tallied per interval (count, largest, smallest) and set aside, one list per workgroup.
//  3. k_bisect_reduce adds the workgroups' tallies up; the bracket shrinks to the gains seen in
//     the interval where the running count reaches the budget.
//  4. k_bisect_pass<1> keeps what the lists hold of the narrower bracket.
//  5. k_bisect_finalize: every workgroup finishes the search from the lists (usually a few
//     thousand gains), then k_i = #{l : M_i(l) > tau} and U_i = 1 - E_i(k_i) per prompt, E from
//     the gain the walk ends with (E(l) = M(l) (alpha + beta + l) / alpha, App. A), final for
//     every prompt that gets no unit at tau; a tied prompt is flagged and leaves the utility
//     of one more unit aside; k_bisect_write: ties at tau by prompt index (tied prompts rewritten),
//     group offsets.
//
// Under a shared prior the gains of a bracket are few distinct values, each repeated: step 3
// already closes the bracket and steps 4 and the finisher return at once.
// The steps are device functions with a kernel around each; a batch of one tile runs all of
// them in one launch (k_bisect_tile), and up to a few hundred prompts one workgroup searches
// alone with other code (k_whole_batch, with the sharded kernels).
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "hora.h"
#include "hora_device.h"
#include "hora_alloc_common.h"
#include "hora_alloc_emit.h"

namespace hora {

// Up to here one workgroup searches alone, in one launch, by walks: its first 512 prompts (two
// per thread) keep their walk states from pass to pass, the ones after them would walk from
// l = 0 in every pass, so the six steps below take over there (measured, learned-prior
// posteriors, 8 units per prompt: 21 us at 60 prompts, 23 at 256, 39 at 512; 47 us for one
// tile in one launch; counts through this method: 29 / 56 us at 60 / 512 prompts, and 87 us
// at 513 while this bound was 2048).
constexpr int kSoloMaxPrompts = 512;
constexpr unsigned long long kOne = 0x3ff0000000000000ull;  // pattern of 1.0: no gain exceeds it
constexpr unsigned long long kOctave = 1ull << 52;          // one exponent step of the pattern
constexpr int kMaxOctave = 1022;                            // octave o holds (2^-(o+1), 2^-o]; the last one ends at 0
constexpr int kRing = 2 * kWinOct;                          // octaves of counts a tile keeps in LDS while walking
constexpr unsigned long long kWindowStep = 4ull << 52;      // fallback windows: a factor 16 in value
constexpr long long kDeepRatio = 24;                            // budgets above this many units per prompt: kernels that can pool walks
constexpr int kFinalMaxPasses = 600;                        // one-workgroup finisher: windows down to zero plus narrowing passes
static_assert(kListCap % kBig == 0, "a thread holds a fixed number of list entries");
static_assert((kWinOct & (kWinOct - 1)) == 0 && kSubBins == 4, "octave window");

__device__ __forceinline__ unsigned long long octave_top(int o) { return kOne - (unsigned long long)o * kOctave; }

// ----------------------------------------------------------------------------------
// kItems consecutive posteriors per thread (one 16-byte load of c, or four of alpha / beta),
// in two steps: `fetch` only issues the loads, `unpack` checks and converts what came back.
// A kernel fetches its first tile before the prologue that every workgroup runs for itself
// (the depth estimate, the sums of the coarse counts, the end of the search), so that the
// latency of the loads is spent there.  Invalid entries are replaced by (1, 1) so that
// every walk is well defined.
// ----------------------------------------------------------------------------------
template <class Src> struct Fetched;
template <> struct Fetched<CountsSource> { int cls[kItems]; };
template <> struct Fetched<PosteriorSource> { double a[kItems], b[kItems]; };

__device__ __forceinline__ void fetch(const CountsSource& src, long long pos, long long end,
                                      Fetched<CountsSource>& f) {
    load_items_i32(src.c, pos, end, (reinterpret_cast<uintptr_t>(src.c) & 15) == 0, 0, f.cls);
}

__device__ __forceinline__ bool unpack(const CountsSource& src, const Fetched<CountsSource>& f,
                                       double (&a)[kItems], double (&b)[kItems]) {
    bool ok = true;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        int x = f.cls[j];
        ok &= (x >= 0) && (x <= src.g0);
        x = x < 0 ? 0 : (x > src.g0 ? src.g0 : x);
        a[j] = src.alpha0 + (double)x;
        b[j] = src.beta0 + (double)(src.g0 - x);
    }
    return ok;
}

__device__ __forceinline__ void fetch(const PosteriorSource& src, long long pos, long long end,
                                      Fetched<PosteriorSource>& f) {
    const bool vec = ((reinterpret_cast<uintptr_t>(src.alpha) | reinterpret_cast<uintptr_t>(src.beta)) & 15) == 0;
    if (vec && pos + kItems <= end) {
#pragma unroll
        for (int q = 0; q < kItems / 2; ++q) {
            const v2d x = *reinterpret_cast<const v2d*>(src.alpha + pos + 2 * q);
            const v2d y = *reinterpret_cast<const v2d*>(src.beta + pos + 2 * q);
            f.a[2 * q] = x.x; f.a[2 * q + 1] = x.y;
            f.b[2 * q] = y.x; f.b[2 * q + 1] = y.y;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            f.a[j] = pos + j < end ? src.alpha[pos + j] : 1.0;
            f.b[j] = pos + j < end ? src.beta[pos + j] : 1.0;
        }
    }
}

__device__ __forceinline__ bool unpack(const PosteriorSource&, const Fetched<PosteriorSource>& f,
                                       double (&a)[kItems], double (&b)[kItems]) {
    bool ok = true;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        a[j] = f.a[j];
        b[j] = f.b[j];
        const bool good = (a[j] > 0.0) && (b[j] > 0.0) && (a[j] < INFINITY) && (b[j] < INFINITY);
        if (!good) { a[j] = 1.0; b[j] = 1.0; }
        ok &= good;
    }
    return ok;
}

template <class Src>
__device__ __forceinline__ bool load_posteriors(const Src& src, long long pos, long long end,
                                                double (&a)[kItems], double (&b)[kItems]) {
    Fetched<Src> f;
    fetch(src, pos, end, f);
    return unpack(src, f, a, b);
}

// ----------------------------------------------------------------------------------
// Walk states between the kernels (one gain and its index l per prompt; kItems per thread).
// ----------------------------------------------------------------------------------
struct WalkStates { double g[kItems]; int l[kItems]; };

__device__ __forceinline__ void fetch_states(const double* __restrict__ ck_g, const int32_t* __restrict__ ck_l,
                                             long long pos, long long end, WalkStates& st) {
    if (pos + kItems <= end) {   // (the arrays are 256-byte aligned and pos is a multiple of kItems)
#pragma unroll
        for (int q = 0; q < kItems / 2; ++q) {
            const v2d x = *reinterpret_cast<const v2d*>(ck_g + pos + 2 * q);
            st.g[2 * q] = x.x; st.g[2 * q + 1] = x.y;
        }
        const v4i l = *reinterpret_cast<const v4i*>(ck_l + pos);
        st.l[0] = l.x; st.l[1] = l.y; st.l[2] = l.z; st.l[3] = l.w;
    } else {
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            st.g[j] = pos + j < end ? ck_g[pos + j] : 0.0;
            st.l[j] = pos + j < end ? ck_l[pos + j] : 0;
        }
    }
}

__device__ __forceinline__ void store_states(double* __restrict__ ck_g, int32_t* __restrict__ ck_l, long long pos,
                                             long long end, const double (&g)[kItems], const double (&lf)[kItems]) {
    int l[kItems];
#pragma unroll
    for (int j = 0; j < kItems; ++j) l[j] = (int)lf[j];
    store_items<v2d, double>(ck_g, pos, end, true, g);
    store_items<v4i, int32_t>(ck_l, pos, end, true, l);
}

// ----------------------------------------------------------------------------------
// 1a. How deep to walk: an estimate from a sample.  kEstSamples prompts spread evenly over the
// batch are walked octave by octave by the first kEstWaves wavefronts of every workgroup (the
// same prompts and the same arithmetic everywhere, so all workgroups agree) until the sample
// has seen its share of the budget and a margin.  The estimate decides only how much work
// the coarse count does in one go and where the walk states are kept; what the coarse count
// guarantees does not depend on it, so the sample's gains are only approximated (a reciprocal
// approximation and a multiplication per step: a quarter of the instructions of a division).
//   est : the octave in which the sample's count reached its share (walk to its bottom)
//   ck  : the octave at whose top the walk states are kept: est, or est - 1 when the sample's
//         count at the bottom of est - 1 was already close to the share
// Octaves whose gains all exceed n / budget are walked in one go: a prompt has fewer than
// 1 / x gains above x (they decrease and sum to at most 1), so fewer than `budget` gains
// exceed n / budget and tau lies below.
// ----------------------------------------------------------------------------------
// Shares of the budget, worked out by the host: a 64-bit division in a kernel is a long sequence
// of vector instructions, run by every wavefront of every workgroup.
struct BudgetShares {
    unsigned long long sample;      // of the depth estimate's sample, rounded up
    unsigned long long per_prompt;  // budget / n, rounded down
    unsigned long long tile;        // of a full tile, rounded up
    unsigned long long last_tile;   // of the batch's last tile (n - its start prompts), rounded up
};

// (eight wavefronts with one sample per lane: two walkers per vector unit fill each other's
// waits; four with two samples per lane took 3 % longer per call, sixteen with one, i.e. twice
// the sample, were no faster than four)
constexpr int kEstWaves = 8;
constexpr int kEstItems = 1;
constexpr int kEstSamples = kEstWaves * kWave * kEstItems;   // 512

struct EstimateShared {
    // [octave & 3]; a wavefront may be an octave ahead of another that still reads the last
    // octave's entries, so every octave has entries of its own, cleared two octaves ahead
    unsigned long long count[4];   // gains of the sample in that octave
    int alive[4];                  // a sample prompt has gains left below that octave
    int deepest;                   // most gains of one sample prompt above the estimated depth
};

template <class Src>
__device__ __forceinline__ void estimate_depth(const Src& src, long long n, const BudgetShares& shares, long long limit,
                                               EstimateShared& es, int& est, int& ck, bool& uneven,
                                               bool& very_uneven, int& deepest) {
    const bool walker = threadIdx.x < kEstWaves * kWave;
    const double limit_d = (double)limit;
    double b[kEstItems], s[kEstItems], g[kEstItems], lf[kEstItems];
    unsigned long long gb[kEstItems];
    bool alive[kEstItems];
#pragma unroll
    for (int j = 0; j < kEstItems; ++j) {
        double a = 1.0;
        b[j] = 1.0;
        if (walker) {
            const long long q = (long long)threadIdx.x * kEstItems + j;
            src.load((long long)(((unsigned long long)q * (unsigned long long)n) / kEstSamples), a, b[j]);
        }
        s[j] = a + b[j];
        g[j] = gain_first(a, s[j]);
        lf[j] = 0.0;
        gb[j] = gain_bits(g[j]);
        alive[j] = walker && limit > 0 && gb[j] != 0ull;
    }
    if (threadIdx.x < 4) {
        es.count[threadIdx.x] = 0ull;
        es.alive[threadIdx.x] = 0;
    }
    if (threadIdx.x == 0) es.deepest = 0;
    __syncthreads();
    const unsigned long long want = shares.sample;
    const unsigned long long need = want + (want >> 3) + 16ull;
    const unsigned long long sure = want - (want >> 3);
    const unsigned long long ratio = shares.per_prompt;
    // A prompt's gains add up to less than 1, so fewer than 1 / t of them exceed t, and tau <= n / budget
    // <= 2^-lumped: octaves 0 .. lumped - 1 lie above tau and are counted together with octave `lumped`.
    const int lumped = ratio >= 2ull ? 63 - __clzll((long long)ratio) : 0;
    int o = lumped;
    const int first = o;
    unsigned long long cum = 0ull;      // the sample's count at the bottom of octave o (the same in every thread)
    unsigned long long before = 0ull;   // ... and of the octave above it
    for (;; ++o) {
        if (walker) {
            const unsigned long long bottom = octave_top(o) - kOctave;
            int cnt = 0;
            bool any;
            do {
                any = false;
#pragma unroll
                for (int j = 0; j < kEstItems; ++j) {
                    const bool act = alive[j] && gb[j] > bottom;
                    if (act) {
                        // (an estimate: the hardware's reciprocal approximation instead of the division)
                        g[j] = (g[j] * (b[j] + lf[j])) * __builtin_amdgcn_rcp(s[j] + (lf[j] + 1.0));
                        lf[j] += 1.0;
                        gb[j] = gain_bits(g[j]);
                        alive[j] = lf[j] < limit_d && gb[j] != 0ull;
                        ++cnt;
                    }
                    any |= act;
                }
            } while (any);
            bool mine_alive = false;
#pragma unroll
            for (int j = 0; j < kEstItems; ++j) mine_alive |= alive[j];
            const bool wave_alive = __ballot(mine_alive) != 0ull;
            cnt = wave_last_i32(wave_incl_scan_i32(cnt));
            if (lane_id() == 0) {
                if (cnt) atomicAdd(&es.count[o & 3], (unsigned long long)(unsigned)cnt);
                if (wave_alive) es.alive[o & 3] = 1;
            }
        }
        __syncthreads();
        before = cum;
        cum += es.count[o & 3];
        if (cum >= need || es.alive[o & 3] == 0 || o == kMaxOctave) break;   // uniform
        if (threadIdx.x == 0) {   // (nobody reads or sets these now)
            es.count[(o + 2) & 3] = 0ull;
            es.alive[(o + 2) & 3] = 0;
        }
    }
    est = o;
    ck = (o > first && before > sure) ? o - 1 : o;   // (before: the count at the bottom of octave o - 1)
    // how uneven the walks are: the deepest one against the mean (lf is a walk's length by now)
    if (walker) {
        double deep = 0.0;
#pragma unroll
        for (int j = 0; j < kEstItems; ++j) deep = lf[j] > deep ? lf[j] : deep;
        int d = (int)(deep < 1.0e9 ? deep : 1.0e9);
#pragma unroll
        for (int k = kWave / 2; k > 0; k >>= 1) {
            const int other = __shfl_xor(d, k, kWave);
            d = other > d ? other : d;
        }
        if (lane_id() == 0 && d > 0) atomicMax(&es.deepest, d);
    }
    __syncthreads();
    // lockstep walks take as many rounds as the deepest prompt of a wavefront, pooled ones
    // (pooled_walk) as many as its mean, at a higher cost per round: measured, pooling pays for
    // deep budgets (deepest 592 against a mean of 200: 1.3 times faster; 3266 against 200: 2.7
    // times) and not for shallow ones whatever their spread (a deepest of 30 against a mean of 8:
    // no gain in the coarse count, a loss in the output kernel: staging, barriers and scattered
    // stores weigh more than the idle lanes).  Pooled above a mean of 32 and deepest > 2 mean + 8.
    uneven = cum > 32ull * kEstSamples &&
             (unsigned long long)es.deepest * kEstSamples > 2ull * cum + 8ull * kEstSamples;
    // The coarse count's lockstep walks regroup as they thin out (regroup_plan), which beats its pooled
    // walks up to a deepest walk of several times the mean (measured at a mean of 200: deepest 592,
    // lockstep 746 us against 828 us pooled; deepest 3266, 3031 us against 2721 us).
    very_uneven = uneven && (unsigned long long)es.deepest * kEstSamples > 6ull * cum;
    deepest = es.deepest;
}

// ----------------------------------------------------------------------------------
// 1b. Coarse count.  One tile of kTile prompts at a time, kItems per thread, walked in
// lockstep so that their divisions overlap.  Every gain down to the bottom of the estimated
// octave is counted in one go, per quarter octave of the last kWinOct octaves (a counter per
// thread and quarter octave in LDS: no conflicts, no reductions per gain), and the first state
// of every walk at or below the top of octave `ck` is kept for the kernels that follow.  A
// tile that has not seen its share of the budget by then goes on octave by octave (counts by
// wavefront ballots), comparing its running total with what it needs after every octave: its
// share plus a margin (any stopping rule that waits for the share is correct; the margin only
// makes it likely that the octave in which the global count reaches the budget has been
// walked completely by every tile).  LDS keeps a ring of kRing octaves of counts; the slot
// keeps the last kWinOct.
// ----------------------------------------------------------------------------------
// ----------------------------------------------------------------------------------
// The first go of the coarse count for prompts of very different depth.  In lockstep a
// wavefront walks as many rounds as its deepest prompt needs; here the 256 prompts of a
// wavefront are a pool: a lane takes a prompt, produces its gains one per round (one
// division per round, the first gain a / s included: the same operations in the same order
// as gain_first / gain_next), counts them as the lockstep walk does, leaves the prompt's
// walk state when the prompt is through, and takes the next prompt of the pool.  The
// posteriors come from LDS (pool_a, pool_b: the wavefront's 256 entries).
// ----------------------------------------------------------------------------------
__device__ __forceinline__ void pooled_walk(const double* __restrict__ pool_a, const double* __restrict__ pool_b,
                                            int items, long long first_pos, double limit_d,
                                            unsigned long long est_bottom, unsigned long long fine_top,
                                            unsigned long long top_ck, unsigned (*fine)[kBig], unsigned& higher,
                                            bool& left_alive, double* __restrict__ ck_g,
                                            int32_t* __restrict__ ck_l) {
    int next = kWave;                       // the pool's next prompt (the same in every lane)
    int t = lane_id();                      // this lane's prompt
    bool have = t < items;
    double a = have ? pool_a[t] : 1.0, b = have ? pool_b[t] : 1.0;
    double s = a + b, g = 0.0, l = 0.0;     // l: the index of the gain produced next
    double keep_g = 0.0, keep_l = 0.0;
    bool fresh = true, kept = false;
    while (__ballot(have)) {
        const double num = fresh ? a : g * (b + (l - 1.0));
        const double den = fresh ? s : s + l;
        g = num / den;
        fresh = false;
        const unsigned long long gb = gain_bits(g);
        const bool valid = l < limit_d && gb != 0ull;
        const bool count = have && valid && gb > est_bottom;
        if (count) {
            if (gb > fine_top) ++higher;
            else atomicAdd(&fine[(unsigned)((fine_top - gb) >> 50)][threadIdx.x], 1u);
        }
        // the first state at or below the top of the kept octave, or the one the walk ends in
        if (have && !kept && (!valid || gb <= top_ck)) { keep_g = g; keep_l = l; kept = true; }
        const bool through = have && !count;
        if (count) l += 1.0;
        const unsigned long long m = __ballot(through);
        if (m) {                            // uniform
            if (through) {
                left_alive |= valid;
                ck_g[first_pos + t] = keep_g;
                ck_l[first_pos + t] = (int)keep_l;
                t = next + lanes_below(m);
                have = t < items;
                if (have) { a = pool_a[t]; b = pool_b[t]; s = a + b; }
                l = 0.0;
                fresh = true;
                kept = false;
            }
            next += __popcll(m);
        }
    }
}

// ----------------------------------------------------------------------------------
// Regrouping the walks of a wavefront.  A wavefront holds kItems walks per lane and steps
// item j of its lanes as long as any lane's item j is active, so walks of different length
// leave most lanes idle towards the end.  When the active walks would fit fewer items per
// lane, the wavefront's 64 * kItems walks are permuted (a stable partition: the active ones
// first, item-major) so that the active ones fill the lanes of the first items: a field at a
// time through 2 KB of LDS per wavefront.  Nothing leaves the wavefront, whose LDS operations
// complete in order: no workgroup barrier is needed.  Position p = j * 64 + lane stands for
// item j of lane `lane`.
// ----------------------------------------------------------------------------------
struct WaveStage { double v[kWave * kItems]; };

__device__ __forceinline__ void wave_phase() {   // orders the wavefront's LDS phases for the compiler (emits nothing)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Where every walk goes (whole wavefronts call this); `total` = the number of active walks.
__device__ __forceinline__ void regroup_plan(const bool (&act)[kItems], int total, int (&dest)[kItems]) {
    int act_before = 0, idle_before = 0;
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
        const unsigned long long m = __ballot(act[j]);
        const int below = lanes_below(m);
        dest[j] = act[j] ? act_before + below : total + idle_before + (lane_id() - below);
        act_before += __popcll(m);
        idle_before += kWave - __popcll(m);
    }
}

__device__ __forceinline__ void regroup(WaveStage& st, const int (&dest)[kItems], double (&x)[kItems]) {
#pragma unroll
    for (int j = 0; j < kItems; ++j) st.v[dest[j]] = x[j];
    wave_phase();
#pragma unroll
    for (int j = 0; j < kItems; ++j) x[j] = st.v[j * kWave + lane_id()];
    wave_phase();
}
__device__ __forceinline__ void regroup(WaveStage& st, const int (&dest)[kItems], int (&x)[kItems]) {
    int* v = reinterpret_cast<int*>(st.v);
#pragma unroll
    for (int j = 0; j < kItems; ++j) v[dest[j]] = x[j];
    wave_phase();
#pragma unroll
    for (int j = 0; j < kItems; ++j) x[j] = v[j * kWave + lane_id()];
    wave_phase();
}

constexpr int kRegroupGain = 6;             // items saved x rounds left from which a regrouping pays (a gain step: ~55 instructions)
constexpr int kFine = kWinOct * kSubBins;   // quarter octaves counted per thread in the first go
static_assert(kFine == kBigWaves, "one wavefront adds up one quarter octave");

// kDeep: the variant for deep budgets (the host's choice, budget > kDeepRatio * n), which
// can pool its walks; the other one does without that code, its registers and its LDS.
template <class Src, bool kDeep>
__device__ __forceinline__ void bisect_coarse(Src src, long long n, BudgetShares shares, long long limit,
                                                        long long chunk, CoarseSlot* __restrict__ slots,
                                                        AllocHeader* __restrict__ hdr, double* __restrict__ ck_g,
                                                        int32_t* __restrict__ ck_l, int32_t* dev_status) {
    __shared__ unsigned s_fine[kFine][kBig];
    // the tile's posteriors for pooled_walk (kDeep), and later, or otherwise, the wavefronts' stages for regroup
    __shared__ double s_f64[kDeep ? 2 * kTile : kBigWaves * kWave * kItems];
    static_assert(sizeof(WaveStage) * kBigWaves <= sizeof(double) * 2 * kTile, "the stages fit the pool's arrays");
    WaveStage* const s_stage = reinterpret_cast<WaveStage*>(s_f64);
    __shared__ unsigned long long s_cnt[kRing][kSubBins];
    __shared__ unsigned long long s_total;       // gains counted in the first go
    __shared__ unsigned long long s_octave[4];   // [octave & 3] gains counted in an octave after it (see EstimateShared)
    __shared__ int s_alive[4];
    __shared__ EstimateShared s_est;
    const long long base = (long long)blockIdx.x * chunk;
    const long long end = base + chunk < n ? base + chunk : n;
    Fetched<Src> first_tile;
    fetch(src, base + (long long)threadIdx.x * kItems, base + kTile < end ? base + kTile : end, first_tile);
    int est, ck, deepest;
    bool uneven, very_uneven;
    estimate_depth(src, n, shares, limit, s_est, est, ck, uneven, very_uneven, deepest);
    const unsigned long long top_ck = octave_top(ck);
    if (blockIdx.x == 0 && threadIdx.x == 0) hdr->ck_top = top_ck;
    const unsigned long long est_bottom = octave_top(est) - kOctave;
    const unsigned long long fine_top = octave_top(est - (kWinOct - 1));   // (above 1.0 when est < kWinOct - 1: no gain lies there)
    const int lane = lane_id();
    const double limit_d = (double)limit;
    bool bad = false;
    for (long long t0 = base; t0 < end; t0 += kTile) {
        const long long tile_end = t0 + kTile < end ? t0 + kTile : end;
        // the tile's share of the budget (only the batch's last tile can be short)
        const unsigned long long share = t0 + kTile <= n ? shares.tile : shares.last_tile;
        const unsigned long long need = share + (share >> 5) + 64ull;
        const long long pos = t0 + (long long)threadIdx.x * kItems;
        double a[kItems], b[kItems], s[kItems], g[kItems], lf[kItems], keep_g[kItems], keep_l[kItems];
        unsigned long long gb[kItems];
        bool alive[kItems];
        if (t0 != base) fetch(src, pos, tile_end, first_tile);
        bad |= !unpack(src, first_tile, a, b) && pos < tile_end;
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            s[j] = a[j] + b[j];
            g[j] = gain_first(a[j], s[j]);
            lf[j] = 0.0;
            gb[j] = gain_bits(g[j]);
            alive[j] = pos + j < tile_end && limit > 0 && gb[j] != 0ull;
            keep_g[j] = g[j];
            keep_l[j] = 0.0;
        }
        if (threadIdx.x < kRing * kSubBins) (&s_cnt[0][0])[threadIdx.x] = 0ull;
        if (threadIdx.x < 4) { s_alive[threadIdx.x] = 0; s_octave[threadIdx.x] = 0ull; }
        if (threadIdx.x == 0) s_total = 0ull;
#pragma unroll
        for (int f = 0; f < kFine; ++f) s_fine[f][threadIdx.x] = 0u;
        __syncthreads();
        // everything down to the bottom of octave `est` in one go
        unsigned higher = 0u;   // gains above the counted octaves (a lane sees at most kItems * limit <= 2^22)
        bool pooled = kDeep && very_uneven;
        if constexpr (kDeep) if (pooled) {
            double (&s_pool)[2][kTile] = *reinterpret_cast<double (*)[2][kTile]>(s_f64);
#pragma unroll
            for (int j = 0; j < kItems; ++j) {
                s_pool[0][threadIdx.x * kItems + j] = a[j];
                s_pool[1][threadIdx.x * kItems + j] = b[j];
            }
            __syncthreads();   // (a wavefront reads what its own lanes wrote; the barrier also keeps the order)
            const long long first_pos = t0 + (long long)wave_id() * (kWave * kItems);
            const long long left = tile_end - first_pos;
            bool left_alive = false;
            pooled_walk(s_pool[0] + wave_id() * (kWave * kItems), s_pool[1] + wave_id() * (kWave * kItems),
                        (int)(left < kWave * kItems ? (left > 0 ? left : 0) : kWave * kItems), first_pos, limit_d,
                        est_bottom, fine_top, top_ck, s_fine, higher, left_alive, ck_g, ck_l);
            const bool wave_alive = __ballot(left_alive) != 0ull;
            const long long higher_all = wave_total_i64((long long)higher);
            if (lane == 0) {
                if (higher_all) atomicAdd(&s_total, (unsigned long long)higher_all);
                if (wave_alive) s_alive[est & 3] = 1;
            }
            __syncthreads();   // the counters of all threads are complete
            {
                // (a pooled walk cannot go on octave by octave, its walks are not in registers any more:
                // a tile that is short of its share is walked again, in lockstep)
                long long acc = 0;
#pragma unroll
                for (int i = 0; i < kBig / kWave; ++i) acc += (long long)s_fine[wave_id()][lane + kWave * i];
                acc = wave_total_i64(acc);
                if (lane == 0 && acc) atomicAdd(&s_octave[0], (unsigned long long)acc);   // (s_octave[0] is free until then)
            }
            __syncthreads();
            const bool short_of_share = s_total + s_octave[0] < need && s_alive[est & 3] != 0 && est < kMaxOctave;
            __syncthreads();
            if (short_of_share) {   // uniform
                pooled = false;
                higher = 0u;
                if (threadIdx.x == 0) { s_total = 0ull; s_alive[est & 3] = 0; }
#pragma unroll
                for (int f = 0; f < kFine; ++f) s_fine[f][threadIdx.x] = 0u;
            }
            if (threadIdx.x == 0) s_octave[0] = 0ull;
            __syncthreads();
        }
        if (!pooled) {
            // (the counters are per thread, not per prompt: a walk may change lanes on its way)
            WaveStage& stage = s_stage[wave_id()];
            int home[kItems];          // where in the wavefront's 256 prompts the walk in item j came from
#pragma unroll
            for (int j = 0; j < kItems; ++j) home[j] = j * kWave + lane;
            int in_use = kItems;       // items per lane that may hold an active walk
            // A regrouping costs about as much as five steps of one item (seven fields through LDS): it is
            // worth it when items saved x rounds left exceeds that, the rounds left taken from the deepest
            // walk of the estimate's sample.
            for (int round = 0;; ++round) {
                bool act[kItems];
                int total = 0;
#pragma unroll
                for (int j = 0; j < kItems; ++j) {
                    act[j] = alive[j] && gb[j] > est_bottom;
                    total += __popcll(__ballot(act[j]));
                }
                if (total == 0) break;                      // uniform over the wavefront
                const int fewer = in_use - (total + kWave - 1) / kWave;
                if (fewer > 0 && fewer * (deepest - round) >= kRegroupGain) {   // uniform
                    int dest[kItems], flags[kItems];
                    regroup_plan(act, total, dest);
#pragma unroll
                    for (int j = 0; j < kItems; ++j) flags[j] = home[j] | (alive[j] ? 0x10000 : 0);
                    regroup(stage, dest, b);
                    regroup(stage, dest, s);
                    regroup(stage, dest, g);
                    regroup(stage, dest, lf);
                    regroup(stage, dest, keep_g);
                    regroup(stage, dest, keep_l);
                    regroup(stage, dest, flags);
                    in_use = (total + kWave - 1) / kWave;
#pragma unroll
                    for (int j = 0; j < kItems; ++j) {
                        home[j] = flags[j] & 0xffff;
                        alive[j] = (flags[j] & 0x10000) != 0;
                        gb[j] = gain_bits(g[j]);
                        act[j] = j * kWave + lane < total;
                    }
                }
#pragma unroll
                for (int j = 0; j < kItems; ++j) {
                    if (act[j]) {
                        if (gb[j] > fine_top) ++higher;
                        else atomicAdd(&s_fine[(unsigned)((fine_top - gb[j]) >> 50)][threadIdx.x], 1u);
                        const bool above_ck = gb[j] > top_ck;
                        g[j] = gain_next(g[j], b[j], s[j], lf[j]);
                        lf[j] += 1.0;
                        gb[j] = gain_bits(g[j]);
                        alive[j] = lf[j] < limit_d && gb[j] != 0ull;
                        if (above_ck) { keep_g[j] = g[j]; keep_l[j] = lf[j]; }
                    }
                }
            }
            {   // the kept states go back to where their prompts are in memory (item j of lane L: prompt pos + j)
                double kg[kItems], kl[kItems];
#pragma unroll
                for (int j = 0; j < kItems; ++j) { kg[j] = keep_g[j]; kl[j] = keep_l[j]; }
                if (in_use != kItems) {   // uniform over the wavefront: walks have moved
                    regroup(stage, home, kg);
                    regroup(stage, home, kl);
                }
                store_states(ck_g, ck_l, pos, tile_end, kg, kl);
            }
            bool mine_alive = false;
#pragma unroll
            for (int j = 0; j < kItems; ++j) mine_alive |= alive[j];
            const bool wave_alive = __ballot(mine_alive) != 0ull;
            const long long higher_all = wave_total_i64((long long)higher);
            if (lane == 0) {
                if (higher_all) atomicAdd(&s_total, (unsigned long long)higher_all);
                if (wave_alive) s_alive[est & 3] = 1;
            }
        }
        __syncthreads();   // the counters of all threads are complete
        {
            const int f = wave_id();   // this wavefront adds up quarter octave f of the counted octaves
            long long acc = 0;
#pragma unroll
            for (int i = 0; i < kBig / kWave; ++i) acc += (long long)s_fine[f][lane + kWave * i];
            acc = wave_total_i64(acc);
            if (lane == 0 && acc) {
                const int oct = est - (kWinOct - 1) + f / kSubBins;   // (a count can only be non-zero for oct >= 0)
                s_cnt[oct & (kRing - 1)][f % kSubBins] = (unsigned long long)acc;
                atomicAdd(&s_total, (unsigned long long)acc);
            }
        }
        __syncthreads();
        int o = est;
        bool any_alive = s_alive[o & 3] != 0;
        unsigned long long total = s_total;   // the tile's running count (the same in every thread)
        if (total < need && any_alive && o < kMaxOctave) {
            // short of its share: the tile goes on octave by octave (the ring's rows for the next
            // two octaves are still zero)
            for (o = est + 1;; ++o) {
                const unsigned long long top = octave_top(o);
                const unsigned long long bottom = top - kOctave;
                // this lane's counts of the four quarter octaves: 8 bits each in one register, moved
                // to the wide counters before a field can overflow
                int c0 = 0, c1 = 0, c2 = 0, c3 = 0;
                unsigned packed = 0u;
                int rounds = 0;
                bool any;
                do {
                    any = false;
#pragma unroll
                    for (int j = 0; j < kItems; ++j) {
                        const bool act = alive[j] && gb[j] > bottom;
                        // 8 * quarter octave of the gain: bits 50 and 51 of (top - pattern)
                        const unsigned shift8 = ((unsigned)((top - gb[j]) >> 32) >> 15) & 0x18u;
                        packed += act ? (1u << shift8) : 0u;
                        if (act) {
                            g[j] = gain_next(g[j], b[j], s[j], lf[j]);
                            lf[j] += 1.0;
                            gb[j] = gain_bits(g[j]);
                            alive[j] = lf[j] < limit_d && gb[j] != 0ull;
                        }
                        any |= act;
                    }
                    if (++rounds == 255 / kItems) {   // uniform
                        c0 += (int)(packed & 0xffu); c1 += (int)((packed >> 8) & 0xffu);
                        c2 += (int)((packed >> 16) & 0xffu); c3 += (int)(packed >> 24);
                        packed = 0u;
                        rounds = 0;
                    }
                } while (__ballot(any));
                c0 += (int)(packed & 0xffu); c1 += (int)((packed >> 8) & 0xffu);
                c2 += (int)((packed >> 16) & 0xffu); c3 += (int)(packed >> 24);
                bool mine_alive = false;
#pragma unroll
                for (int j = 0; j < kItems; ++j) mine_alive |= alive[j];
                const bool wave_alive = __ballot(mine_alive) != 0ull;
                // (a lane counts at most kItems * limit <= 2^22 gains per octave: the sums fit 32 bits)
                c0 = wave_last_i32(wave_incl_scan_i32(c0));
                c1 = wave_last_i32(wave_incl_scan_i32(c1));
                c2 = wave_last_i32(wave_incl_scan_i32(c2));
                c3 = wave_last_i32(wave_incl_scan_i32(c3));
                if (lane == 0) {
                    unsigned long long* row = s_cnt[o & (kRing - 1)];
                    if (c0) atomicAdd(&row[0], (unsigned long long)(unsigned)c0);
                    if (c1) atomicAdd(&row[1], (unsigned long long)(unsigned)c1);
                    if (c2) atomicAdd(&row[2], (unsigned long long)(unsigned)c2);
                    if (c3) atomicAdd(&row[3], (unsigned long long)(unsigned)c3);
                    const unsigned long long all = (unsigned long long)(unsigned)c0 + (unsigned)c1 + (unsigned)c2 + (unsigned)c3;
                    if (all) atomicAdd(&s_octave[o & 3], all);
                    if (wave_alive) s_alive[o & 3] = 1;
                }
                __syncthreads();
                any_alive = s_alive[o & 3] != 0;
                total += s_octave[o & 3];
                if (total >= need || !any_alive || o == kMaxOctave) break;   // uniform
                // room for the octave after the next one (nobody reads or adds to these now)
                if (threadIdx.x < kSubBins) s_cnt[(o + 2) & (kRing - 1)][threadIdx.x] = 0ull;
                if (threadIdx.x == 0) { s_alive[(o + 2) & 3] = 0; s_octave[(o + 2) & 3] = 0ull; }
            }
        }
        // the tile's slot: the last kWinOct octaves in detail, everything above them as one number
        if (threadIdx.x < kWave) {
            const int w = lane / kSubBins, sub = lane % kSubBins;
            unsigned long long v = 0ull;
            if (lane < kWinOct * kSubBins) {
                const int oct = o - ((o - w) & (kWinOct - 1));   // the octave in [o - kWinOct + 1, o] that is w modulo kWinOct
                if (oct >= 0) v = s_cnt[oct & (kRing - 1)][sub];
            }
            const long long in_window = wave_total_i64((long long)v);
            CoarseSlot* slot = slots + t0 / kTile;
            if (lane < kWinOct * kSubBins) slot->cnt[w][sub] = v;
            if (lane == 0) {
                slot->cum_top = total - (unsigned long long)in_window;
                slot->stop = o;
                slot->exhausted = any_alive ? 0 : 1;
            }
        }
        __syncthreads();   // the counters are reused by the next tile
    }
    if (bad) report(dev_status, HORA_ERR_RANGE);
}
template <class Src, bool kDeep>
__global__ __launch_bounds__(kBig) void k_bisect_coarse(Src src, long long n, BudgetShares shares, long long limit,
    long long chunk, CoarseSlot* __restrict__ slots, AllocHeader* __restrict__ hdr, double* __restrict__ ck_g,
    int32_t* __restrict__ ck_l, int32_t* dev_status) {
    bisect_coarse<Src, kDeep>(src, n, shares, limit, chunk, slots, hdr, ck_g, ck_l, dev_status);
}

// ----------------------------------------------------------------------------------
// 3. Narrowing pass.  Invariant: exactly `above` pairs have a gain > hi, above < budget, and
// count_gt(lo) >= budget.  The gains inside (lo, hi] are tallied per interval; if the running
// count from the top interval down reaches the budget in interval j, the bracket shrinks to
// the gains that occur there, (min - 1, max], and closes when min == max (tau is that gain):
// each pass cuts the bracket at least 128-fold; with real-valued posteriors it keeps ~1/256
// of the gains of the pass before, with a shared prior it closes at once.  Every workgroup
// tallies its share into a slot of its own; k_bisect_reduce adds the slots up, and every
// workgroup of the next kernel moves the bracket by those totals for itself (the same
// arithmetic on the same numbers everywhere).  The bracket is kept twice: pass p reads slot
// p & 1, which nobody writes meanwhile, and its first workgroup stores the moved bracket in
// the other slot.
// ----------------------------------------------------------------------------------
struct SelectShared {
    TallyBins bins;
    long long red[kBigWaves];
    unsigned long long lo, hi;
    long long above;
    long long inside;   // pairs in the bracket (-1: not known)
    int done;
    int hit;            // the last step narrowed the bracket (it did not move to another window)
    int list_n;         // gains this workgroup has set aside in this pass
};

// The step that ends a pass, run by a whole workgroup: thread t < kBins holds the tally
// (cj, mx, mn) of interval kBins - 1 - t (thread 0 the top one), the other threads zeros.
// Finds the interval in which the running count from the top reaches the budget and shrinks
// the bracket to the gains seen there; when the whole bracket lies above tau (possible only
// for the wide brackets that the coarse count falls back to), takes the window below it.
__device__ __forceinline__ void move_bracket(SelectShared& sh, unsigned long long cj, unsigned long long mx,
                                             unsigned long long mn, long long budget) {
    static_assert(kBins % kWave == 0 && kBins / kWave <= kBigWaves, "the tallies fill whole wavefronts");
    constexpr int kTallyWaves = kBins / kWave;
    // (the caller's barrier lies between the last change of the bracket and these reads; the
    // barrier below between them and the next change)
    const unsigned long long lo = sh.lo;
    const long long start = sh.above;   // pairs above the bracket
    if (cj > (unsigned long long)budget) cj = (unsigned long long)budget;
    long long incl = 0;
    if (wave_id() < kTallyWaves) {       // uniform per wavefront: the others hold zeros
        incl = (long long)wave_incl_scan_u64(cj);
        if (lane_id() == kWave - 1) sh.red[wave_id()] = incl;
    }
    __syncthreads();
    long long before = start + incl - (long long)cj;     // pairs in higher intervals
    long long total = 0;
#pragma unroll
    for (int i = 0; i < kTallyWaves; ++i) {
        if (i < wave_id()) before += sh.red[i];
        total += sh.red[i];
    }
    if (start + total < budget) {                       // uniform: the whole bracket is above tau
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

// Loads the bracket of pass `pass` and, if the pass before tallied, moves it by the totals.
__device__ __forceinline__ void enter_pass(SelectShared& sh, const AllocHeader* hdr, const SelectBins* bins, int pass,
                                           long long budget) {
    const Bracket* in = &hdr->slot[pass & 1];
    const bool pending = (in->flags & kFlagPending) != 0 && in->done == 0;   // uniform
    const SelectBins* totals = bins + kMaxBlocks;
    const int j = kBins - 1 - (int)threadIdx.x;   // thread 0 owns the top interval
    unsigned long long cj = 0, mx = 0, mn = 0;
    if (pending && threadIdx.x < kBins) {
        cj = totals->cnt[j];
        mx = totals->vmax[j];
        mn = ~totals->vmin_inv[j];
    }
    if (threadIdx.x == 0) {
        sh.lo = in->lo; sh.hi = in->hi; sh.above = (long long)in->above; sh.done = (int)in->done;
        sh.hit = 0;
        sh.inside = -1;
        sh.list_n = 0;
    }
    __syncthreads();
    if (pending) move_bracket(sh, cj, mx, mn, budget);
}

// Appends the gains that `keep` marks to the workgroup's list (whole wavefronts call this).
__device__ __forceinline__ void list_append(SelectShared& sh, unsigned long long* __restrict__ list, bool keep,
                                            unsigned long long gb) {
    const unsigned long long m = __ballot(keep);
    if (m == 0ull) return;
    int at = 0;
    if (lane_id() == 0) at = atomicAdd(&sh.list_n, __popcll(m));
    at = __builtin_amdgcn_readfirstlane(at) + lanes_below(m);
    if (keep && at < kListCap) list[at] = gb;
}

// ----------------------------------------------------------------------------------
// 2. The tiles' coarse counts added up, and the first bracket; run by every workgroup of the
// first narrowing pass for itself (the slots are 144 bytes per 4096 prompts: reading them all
// costs less than a launch in between).  Octave o can be resolved when every tile still has it
// in detail (o >= stop - 7 for all tiles) and every tile that has gains left walked it
// completely (o <= stop for those).  Inside that range the quarter octave in which the
// running count reaches the budget becomes the bracket.  Otherwise (tiles of very different
// prompts, caps that leave tiles short of their share) a wider bracket that is still correct
// is taken and the narrowing passes do the rest.
// ----------------------------------------------------------------------------------
// One entry of the sums below: of the counts seen so far, t belongs to the lowest octave among
// them (o; octaves are numbered downwards, so the largest number) and r to the octaves above it.
struct LowestOctave { int o; long long t, r; };
__device__ __forceinline__ LowestOctave join(const LowestOctave& x, const LowestOctave& y) {
    LowestOctave z;
    z.o = x.o > y.o ? x.o : y.o;
    z.t = (x.o == z.o ? x.t : 0) + (y.o == z.o ? y.t : 0);
    z.r = x.r + y.r + (x.o == z.o ? 0 : x.t) + (y.o == z.o ? 0 : y.t);
    return z;
}

struct CoarseShared {   // what each wavefront found in its slots
    int o[kBigWaves][kWinOct * kSubBins];
    long long t[kBigWaves][kWinOct * kSubBins], r[kBigWaves][kWinOct * kSubBins];
    long long tops[kWave];   // per row of 16 lanes of every wavefront
    int smax[kWave], smin[kWave];
};

// The largest value of a wavefront, in every lane: rotations inside the rows of 16 lanes, then
// the four rows' results as scalars.
__device__ __forceinline__ int wave_max_i32(int v) {
    int o = dpp_take<0x128, 0xf, 0xf>(v); v = o > v ? o : v;   // row_ror:8
    o = dpp_take<0x124, 0xf, 0xf>(v); v = o > v ? o : v;       // row_ror:4
    o = dpp_take<0x122, 0xf, 0xf>(v); v = o > v ? o : v;       // row_ror:2
    o = dpp_take<0x121, 0xf, 0xf>(v); v = o > v ? o : v;       // row_ror:1
    const int a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    const int c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    const int ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

// Every thread takes one count of one slot at a time (a slot's counts are consecutive: coalesced
// loads), always the same ring row w and interval q of the slots it visits, all loads of the
// first kKeep rounds (everything up to 2^20 prompts) under way together.  Which octave a ring
// row holds depends on where its tile stopped, and which octaves form the range depends on all
// tiles: so a thread sums its counts per "lowest octave seen so far" (join), a wavefront joins
// the four lanes that share (w, q) and leaves 16 such entries in LDS.  After a barrier the first
// wavefront joins the 16 wavefronts' entries in the order of the range (lane j of each row of
// 16: octave first + j / 4, interval j % 4) and finds the bracket by a prefix sum over 16 lanes.
// One wavefront, because its fifteen neighbours would share its four vector units: the same
// instructions sixteen times take four times as long as once, and a second barrier costs less.
__device__ __forceinline__ void first_bracket(SelectShared& sh, CoarseShared& cs, long long tiles, long long budget,
                                              const CoarseSlot* __restrict__ slots) {
    static_assert(kBig % (kWinOct * kSubBins) == 0 && kWave == 4 * kWinOct * kSubBins, "lanes that share an interval");
    static_assert(kWinOct == 4 && kBigWaves == kWinOct * kSubBins, "one lane per wavefront's entry, ring of four octaves");
    constexpr int kKeep = 4;
    constexpr int kPerSlot = kWinOct * kSubBins;
    const long long counts = tiles * kPerSlot;
    const int e = (int)threadIdx.x % kPerSlot, w = e / kSubBins, q = e % kSubBins;
    long long kept_v[kKeep], kept_top[kKeep];
    int kept_stop[kKeep];
    bool kept_done[kKeep];
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        const long long idx = (long long)i * kBig + threadIdx.x;
        kept_v[i] = 0; kept_top[i] = 0; kept_stop[i] = -1; kept_done[i] = true;   // (no slot)
        if (idx < counts) {
            const CoarseSlot* slot = slots + idx / kPerSlot;
            kept_v[i] = (long long)slot->cnt[w][q];
            kept_stop[i] = slot->stop;
            kept_done[i] = slot->exhausted != 0;
            if (e == 0) kept_top[i] = (long long)slot->cum_top;
        }
    }
    LowestOctave acc{-1, 0, 0};
    long long tops = 0;
    int smax = 0, smin = INT_MAX;
    auto take = [&](long long v, long long top, int stop, bool exhausted) {
        if (stop < 0) return;
        smax = stop > smax ? stop : smax;
        if (!exhausted) smin = stop < smin ? stop : smin;
        tops += top;
        const int oct = stop - ((stop - w) & (kWinOct - 1));   // the octave of the slot's row w
        if (oct >= 0) acc = join(acc, LowestOctave{oct, v, 0});
    };
#pragma unroll
    for (int i = 0; i < kKeep; ++i) take(kept_v[i], kept_top[i], kept_stop[i], kept_done[i]);
    for (long long idx = (long long)kKeep * kBig + threadIdx.x; idx < counts; idx += kBig) {   // larger batches
        const CoarseSlot* slot = slots + idx / kPerSlot;
        take((long long)slot->cnt[w][q], e == 0 ? (long long)slot->cum_top : 0, slot->stop, slot->exhausted != 0);
    }
#pragma unroll
    for (int d = kPerSlot; d < kWave; d <<= 1) {
        LowestOctave other;
        other.o = __shfl_xor(acc.o, d, kWave);
        other.t = __shfl_xor(acc.t, d, kWave);
        other.r = __shfl_xor(acc.r, d, kWave);
        acc = join(acc, other);
    }
    if (lane_id() < kPerSlot) {
        cs.o[wave_id()][e] = acc.o; cs.t[wave_id()][e] = acc.t; cs.r[wave_id()][e] = acc.r;
    }
    // the 16 lanes of a row see the same slots: the row's first lane has its sum of cum_top and
    // its extremes of the stopping octaves
    if (e == 0) {
        const int row = wave_id() * (kWave / kPerSlot) + lane_id() / kPerSlot;
        cs.tops[row] = tops; cs.smax[row] = smax; cs.smin[row] = smin;
    }
    __syncthreads();
    if (wave_id() == 0) {
        const int j = lane_id() & (kPerSlot - 1), part = lane_id() / kPerSlot;
        const int s_max = wave_max_i32(cs.smax[lane_id()]);
        const int min_seen = -wave_max_i32(-cs.smin[lane_id()]);
        const int s_min = min_seen == INT_MAX ? s_max : min_seen;   // no tile has gains left: everything is counted
        const int first = s_max - (kWinOct - 1) > 0 ? s_max - (kWinOct - 1) : 0;   // first octave of the range
        // (counts up to a few times the budget: sums over the full 64-bit range)
        const long long tops_all = (long long)wave_total_u64((unsigned long long)cs.tops[lane_id()]);
        const int oct_j = first + j / kSubBins;
        const int e_j = (oct_j & (kWinOct - 1)) * kSubBins + (j % kSubBins);   // the ring row that can hold that octave
        // each row of 16 lanes joins four wavefronts' entries, then the four rows are joined
        LowestOctave all{-1, 0, 0};
#pragma unroll
        for (int v = 0; v < kBigWaves / 4; ++v) {
            const int from = part * (kBigWaves / 4) + v;
            all = join(all, LowestOctave{cs.o[from][e_j], cs.t[from][e_j], cs.r[from][e_j]});
        }
#pragma unroll
        for (int d = kPerSlot; d < kWave; d <<= 1) {
            LowestOctave other;
            other.o = __shfl_xor(all.o, d, kWave);
            other.t = __shfl_xor(all.t, d, kWave);
            other.r = __shfl_xor(all.r, d, kWave);
            all = join(all, other);
        }
        const bool low = lane_id() < kPerSlot;             // one copy of the 16 entries
        // (an entry's lowest octave is the range's octave oct_j or lies a multiple of four above it)
        const bool in_range = all.o == oct_j;
        const long long c = (low && in_range) ? all.t : 0;
        const long long all_above =
            tops_all + (long long)wave_total_u64((unsigned long long)(low ? all.r + (in_range ? 0 : all.t) : 0));
        const long long known = all_above + (long long)wave_total_u64((unsigned long long)c);
        const long long incl = (long long)wave_incl_scan_u64((unsigned long long)c);
        unsigned long long lo = 0ull, hi = kOne;
        long long above = 0, inside = -1;
        if (all_above >= budget) {
            lo = octave_top(first);              // count_gt(lo) >= budget already: tau lies above the range
        } else {
            // octaves up to s_min were walked completely by every tile that has gains left
            const unsigned long long reach = __ballot(low && oct_j <= s_min && all_above + incl >= budget);
            if (reach) {
                const int f = __builtin_ctzll(reach);
                const long long cf = (long long)read_lane_u64((unsigned long long)c, f);
                const long long upto = (long long)read_lane_u64((unsigned long long)incl, f);
                hi = octave_top(first + f / kSubBins) - (unsigned long long)(f % kSubBins) * (kOctave / kSubBins);
                lo = hi - kOctave / kSubBins;
                above = all_above + upto - cf;
                inside = cf;
            } else {
                // The range ends above tau.  When it is not empty, the count above its lower end is
                // complete and the bracket starts there; when it is empty (some tile stopped more
                // than kWinOct octaves above another: very different prompts), nothing below 1 is.
                // Downwards the bracket reaches to where every tile has seen its share, or, when the
                // tiles' counts do not add up to the budget (caps), to zero.
                if (s_min >= first) {
                    hi = octave_top(s_min + 1);
                    above = all_above +
                            (long long)read_lane_u64((unsigned long long)incl, (s_min - first) * kSubBins + kSubBins - 1);
                }
                lo = known >= budget ? octave_top(s_max) - kOctave : 0ull;
            }
        }
        if (lane_id() == 0) {
            sh.lo = lo; sh.hi = hi; sh.above = above; sh.inside = inside;
            sh.done = 0; sh.hit = 0; sh.list_n = 0;
        }
    }
    __syncthreads();
}

// kPass = 0: the first bracket comes from the coarse count; the pass walks the prompts, tallies
//   the bracket's gains and sets them aside when they are few enough.
// kPass = 1: the bracket of pass 0 moved by its totals; no tallies, the pass only leaves the
//   gains of the narrower bracket in the lists for the finisher: from the lists of pass 0, or,
//   where those did not fit, by walking the prompts again.
template <class Src, int kPass>
__device__ __forceinline__ void bisect_pass(Src src, long long n, long long budget, long long limit,
                                                      long long chunk, long long tiles,
                                                      const CoarseSlot* __restrict__ slots,
                                                      AllocHeader* __restrict__ hdr, SelectBins* __restrict__ bins,
                                                      unsigned long long* __restrict__ lists,
                                                      int* __restrict__ list_count, double* __restrict__ ck_g,
                                                      int32_t* __restrict__ ck_l) {
    __shared__ SelectShared sh;
    bool from_lists = false;
    Fetched<Src> first_tile;
    WalkStates first_states;
    if constexpr (kPass == 0) {
        // (pass 0 always walks: the loads of its first tile are under way during the prologue)
        const long long base = (long long)blockIdx.x * chunk;
        const long long end = base + chunk < n ? base + chunk : n;
        fetch(src, base + (long long)threadIdx.x * kItems, end, first_tile);
        fetch_states(ck_g, ck_l, base + (long long)threadIdx.x * kItems, end, first_states);
        __shared__ CoarseShared cs;
        first_bracket(sh, cs, tiles, budget, slots);
    } else {
        enter_pass(sh, hdr, bins, kPass, budget);
        // the pass before set the gains of its (wider) bracket aside and all of them fitted
        from_lists = (hdr->slot[kPass & 1].flags & kFlagCollected) != 0 && hdr->lists_ok != 0;
    }
    const unsigned long long b_lo = sh.lo, b_hi = sh.hi;   // the pass's bracket, the pairs above it and inside it
    const long long b_above = sh.above, b_inside = sh.inside;
    const int b_done = sh.done;
    const bool collect = from_lists || (b_inside >= 0 && b_inside <= kCollectMax);
    const bool done = b_done != 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {   // for the next kernel
        Bracket* out = &hdr->slot[(kPass + 1) & 1];
        out->lo = b_lo; out->hi = b_hi; out->above = (unsigned long long)b_above;
        out->done = (unsigned)b_done;
        out->flags = done ? 0u : ((kPass == 0 ? kFlagPending : 0u) | (collect ? kFlagCollected : 0u));
    }
    if (done) return;   // uniform over the grid: every workgroup moved the same bracket
    constexpr bool kTally = kPass == 0;
    const unsigned long long lo = b_lo, hi = b_hi;
    const int shift = bracket_shift(lo, hi);
    if (kTally && threadIdx.x < kBins) { sh.bins.cnt[threadIdx.x] = 0; sh.bins.vmax[threadIdx.x] = 0; sh.bins.vmin_inv[threadIdx.x] = 0; }
    unsigned long long* mine = lists + (long long)blockIdx.x * kListCap;
    if (from_lists) {
        constexpr int kPer = kListCap / kBig;
        const int have = list_count[blockIdx.x];
        unsigned long long v[kPer];
#pragma unroll
        for (int q = 0; q < kPer; ++q) {
            const int e = q * kBig + (int)threadIdx.x;
            v[q] = e < have ? mine[e] : 0ull;
        }
        __syncthreads();   // the list has been read: it is rewritten below
#pragma unroll
        for (int q = 0; q < kPer; ++q) list_append(sh, mine, v[q] > lo && v[q] <= hi, v[q]);
    } else if (kTally || collect) {
        __syncthreads();
        const long long base = (long long)blockIdx.x * chunk;
        const long long end = base + chunk < n ? base + chunk : n;
        const double limit_d = (double)limit;
        // Where the walks start: pass 0 takes the states that the coarse count kept when they lie
        // above the bracket (else it starts from l = 0) and leaves every walk's first state at or
        // below hi in their place, for pass 1 and the output kernel: all later brackets, and tau,
        // lie at or below this hi.
        const bool resume = kPass != 0 || hi <= hdr->ck_top;   // uniform
        for (long long t0 = base; t0 < end; t0 += kTile) {
            const long long pos = t0 + (long long)threadIdx.x * kItems;
            double a[kItems], b[kItems], s[kItems], g[kItems], lf[kItems];
            unsigned long long gb[kItems];
            bool alive[kItems];
            if (kPass != 0 || t0 != base) {
                fetch(src, pos, end, first_tile);
                fetch_states(ck_g, ck_l, pos, end, first_states);
            }
            unpack(src, first_tile, a, b);
#pragma unroll
            for (int j = 0; j < kItems; ++j) {
                s[j] = a[j] + b[j];
                if (resume) { g[j] = first_states.g[j]; lf[j] = (double)first_states.l[j]; }
                else { g[j] = gain_first(a[j], s[j]); lf[j] = 0.0; }
                gb[j] = gain_bits(g[j]);
                alive[j] = pos + j < end && lf[j] < limit_d;
            }
            // down to the bracket: the kItems walks in lockstep
            bool any;
            do {
                any = false;
#pragma unroll
                for (int j = 0; j < kItems; ++j) {
                    const bool act = alive[j] && gb[j] > hi;
                    if (act) {
                        g[j] = gain_next(g[j], b[j], s[j], lf[j]);
                        lf[j] += 1.0;
                        gb[j] = gain_bits(g[j]);
                        alive[j] = lf[j] < limit_d;
                    }
                    any |= act;
                }
            } while (any);
            if (kPass == 0) store_states(ck_g, ck_l, pos, end, g, lf);
            // through the bracket: whole wavefronts, one prompt of every lane at a time
#pragma unroll
            for (int j = 0; j < kItems; ++j) {
                bool inside = alive[j] && gb[j] > lo;
                while (__ballot(inside)) {
                    if (kTally) tally_gains(sh.bins, inside, gb[j], lo, shift);
                    if (collect) list_append(sh, mine, inside, gb[j]);
                    if (inside) {
                        g[j] = gain_next(g[j], b[j], s[j], lf[j]);
                        lf[j] += 1.0;
                        gb[j] = gain_bits(g[j]);
                        inside = lf[j] < limit_d && gb[j] > lo;
                    }
                }
            }
        }
    }
    __syncthreads();   // the workgroup's tallies and its list are complete
    if (collect && threadIdx.x == 0) list_count[blockIdx.x] = sh.list_n <= kListCap ? sh.list_n : -1;
    if (kTally) {
        SelectBins* slot = bins + blockIdx.x;
        if (threadIdx.x < kBins) {
            const unsigned long long c0 = sh.bins.cnt[threadIdx.x];
            slot->cnt[threadIdx.x] = c0 > (unsigned long long)budget ? (unsigned long long)budget : c0;
            slot->vmax[threadIdx.x] = sh.bins.vmax[threadIdx.x];
            slot->vmin_inv[threadIdx.x] = sh.bins.vmin_inv[threadIdx.x];
        }
    }
}
template <class Src, int kPass>
__global__ __launch_bounds__(kBig) void k_bisect_pass(Src src, long long n, long long budget, long long limit,
    long long chunk, long long tiles, const CoarseSlot* __restrict__ slots, AllocHeader* __restrict__ hdr,
    SelectBins* __restrict__ bins, unsigned long long* __restrict__ lists, int* __restrict__ list_count,
    double* __restrict__ ck_g, int32_t* __restrict__ ck_l) {
    bisect_pass<Src, kPass>(src, n, budget, limit, chunk, tiles, slots, hdr, bins, lists, list_count, ck_g, ck_l);
}

// ----------------------------------------------------------------------------------
// Between two kernels of the search: the interval tallies of the workgroups are added up
// (counts) and combined (largest, smallest gain) into bins[kMaxBlocks].  kReduceBins
// intervals per workgroup, 32 lanes per interval striding over the slots.  A kernel of its
// own rather than "the workgroup that finishes last": the device-wide fences that pattern
// needs (write back and invalidate the L2 of every die) cost several times the pass itself
// on this part.
// ----------------------------------------------------------------------------------
constexpr int kReduceBins = kThreads / 32;   // 8 intervals per workgroup of 256 threads

__global__ __launch_bounds__(kThreads) void k_bisect_reduce(int nb, int pass, AllocHeader* __restrict__ hdr,
                                                            SelectBins* __restrict__ bins,
                                                            const int* __restrict__ list_count) {
    const unsigned flags = hdr->slot[(pass + 1) & 1].flags;
    if ((flags & kFlagPending) == 0) return;   // pass `pass` did not tally: the search has ended
    if (blockIdx.x == 0) {   // did every workgroup's list fit?
        static_assert(kMaxBlocks <= kThreads, "one thread per list");
        const int any_bad = __syncthreads_or((int)threadIdx.x < nb && list_count[threadIdx.x] < 0 ? 1 : 0);
        if (threadIdx.x == 0) hdr->lists_ok = ((flags & kFlagCollected) != 0 && !any_bad) ? 1u : 0u;
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
// 4. The end of the search, run by every workgroup of the output kernel for itself (the same
// arithmetic on the same numbers everywhere): if the bracket that pass 1 left is still open,
// narrowing passes are repeated until it closes, from the workgroups' lists (what a 256-fold
// cut leaves of a quarter octave: usually a few thousand gains in all).  Only when the lists
// could not hold the bracket (more gains within 2^-10 of one another than the lists have room
// for, twice in a row) does every workgroup walk all prompts itself, which is slow but correct.
// Returns tau's pattern; *ok says whether the search ended properly.
// ----------------------------------------------------------------------------------
template <class Src>
__device__ unsigned long long finish_search(SelectShared& sh, const Src& src, long long n, long long budget,
                                            long long limit, int nb, const AllocHeader* __restrict__ hdr,
                                            const unsigned long long* __restrict__ lists,
                                            const int* __restrict__ list_count, bool* ok) {
    const Bracket* in = &hdr->slot[0];   // written by pass 1
    // (the tallies start from zero; the barriers below lie between this and the first pass)
    if (threadIdx.x < kBins) { sh.bins.cnt[threadIdx.x] = 0; sh.bins.vmax[threadIdx.x] = 0; sh.bins.vmin_inv[threadIdx.x] = 0; }
    if (threadIdx.x == 0) {
        sh.lo = in->lo; sh.hi = in->hi; sh.above = (long long)in->above; sh.done = (int)in->done;
        sh.hit = 0; sh.inside = -1; sh.list_n = 0;
    }
    static_assert(kMaxBlocks <= kBig && kMaxBlocks == 4 * kWave, "one thread per list, four wavefronts of them");
    __shared__ int s_off[kMaxBlocks + 1];   // list b holds the entries s_off[b] .. s_off[b + 1] - 1 of all lists together
    __shared__ int s_part[4];
    const int have_mine = (int)threadIdx.x < nb ? list_count[threadIdx.x] : 0;
    const int overflow = __syncthreads_or(have_mine < 0 ? 1 : 0);
    const bool from_lists = (in->flags & kFlagCollected) != 0 && !overflow;
    int total_entries = 0;
    if (from_lists) {
        const int incl = wave_incl_scan_i32(have_mine);
        if (threadIdx.x < kMaxBlocks && lane_id() == kWave - 1) s_part[wave_id()] = incl;
        __syncthreads();
        if (threadIdx.x < kMaxBlocks) {
            int before = 0;
            for (int w = 0; w < wave_id(); ++w) before += s_part[w];
            s_off[threadIdx.x + 1] = before + incl;
            if (threadIdx.x == 0) s_off[0] = 0;
        }
        __syncthreads();
        total_entries = s_off[kMaxBlocks];
    }
    // Usually all lists together hold a few thousand gains: then every thread fetches its share
    // once (all loads under way together) and the passes below work on registers.
    constexpr int kHeld = 8;   // list entries a thread holds
    const bool held = from_lists && total_entries <= kHeld * kBig && sh.done == 0;   // uniform
    unsigned long long mine[kHeld];
#pragma unroll
    for (int q = 0; q < kHeld; ++q) mine[q] = 0ull;   // (no gain: outside every bracket)
    if (held) {
#pragma unroll
        for (int q = 0; q < kHeld; ++q) {
            const int e = q * kBig + (int)threadIdx.x;
            if (e < total_entries) {
                int b = 0;
#pragma unroll
                for (int step = kMaxBlocks / 2; step > 0; step >>= 1)
                    if (s_off[b + step] <= e) b += step;     // the last list that starts at or before e
                mine[q] = lists[(long long)b * kListCap + (e - s_off[b])];
            }
        }
    }
    for (int iter = 0; iter < kFinalMaxPasses; ++iter) {
        if (sh.done) break;   // uniform: written before the barrier that ends move_bracket
        const unsigned long long lo = sh.lo, hi = sh.hi;
        const int shift = bracket_shift(lo, hi);
        if (held) {
#pragma unroll
            for (int q = 0; q < kHeld; ++q)
                if (q * kBig < total_entries)   // uniform
                    tally_gains(sh.bins, mine[q] > lo && mine[q] <= hi, mine[q], lo, shift);
        } else if (from_lists) {
            // all entries of all lists as one sequence: every thread finds the list of its entry
            // by a search of the offsets (LDS), so that the loads are independent of one another
            for (int e0 = 0; e0 < total_entries; e0 += kBig) {
                const int e = e0 + (int)threadIdx.x;
                unsigned long long v = 0ull;
                if (e < total_entries) {
                    int b = 0;
#pragma unroll
                    for (int step = kMaxBlocks / 2; step > 0; step >>= 1)
                        if (s_off[b + step] <= e) b += step;     // the last list that starts at or before e
                    v = lists[(long long)b * kListCap + (e - s_off[b])];
                }
                tally_gains(sh.bins, v > lo && v <= hi, v, lo, shift);
            }
        } else {
            for (long long i0 = 0; i0 < n; i0 += kBig) {
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
                    tally_gains(sh.bins, active && gb <= hi, gb, lo, shift);
                    if (active) {
                        g = gain_next(g, b, s, lf);
                        lf += 1.0;
                        k += 1;
                        gb = gain_bits(g);
                        active = k < limit && gb > lo;
                    }
                }
            }
        }
        __syncthreads();
        const int j = kBins - 1 - (int)threadIdx.x;   // thread 0 owns the top interval
        unsigned long long cj = 0, mx = 0, mn = 0;
        if (threadIdx.x < kBins) {   // (and cleared for the next pass by the thread that read them)
            cj = sh.bins.cnt[j];
            mx = sh.bins.vmax[j];
            mn = ~sh.bins.vmin_inv[j];
            sh.bins.cnt[j] = 0; sh.bins.vmax[j] = 0; sh.bins.vmin_inv[j] = 0;
        }
        move_bracket(sh, cj, mx, mn, budget);
    }
    __syncthreads();
    *ok = sh.done == 1;
    return sh.hi;
}

// ----------------------------------------------------------------------------------
// 5a. The end of the search (4.), then with tau known: k_i = #{l : M_i(l) > tau} and the tied
// flag go to delta[i] (flag in bit 31); util[i] gets U_i = 1 - E_i(k_i), and a tied prompt's
// 1 - E_i(k_i + 1) goes where its walk state was; per-workgroup sums to block_ksum / block_tied.  kItems prompts per thread, their walks in lockstep.
// ----------------------------------------------------------------------------------
template <class Src>
__device__ __forceinline__ void bisect_finalize(Src src, long long n, long long chunk, long long budget,
                                                          long long limit, int depth_capped, int nb,
                                                          AllocHeader* __restrict__ hdr,
                                                          const unsigned long long* __restrict__ lists,
                                                          const int* __restrict__ list_count,
                                                          double* ck_g, const int32_t* __restrict__ ck_l,
                                                          int32_t* __restrict__ delta, double* __restrict__ util,
                                                          long long* __restrict__ block_ksum,
                                                          long long* __restrict__ block_tied, int32_t* dev_status) {
    __shared__ SelectShared sh;
    long long (&s_red)[2][kBigWaves] = *reinterpret_cast<long long (*)[2][kBigWaves]>(&sh.bins.cnt[0]);
    const long long base = (long long)blockIdx.x * chunk;
    const long long end = base + chunk < n ? base + chunk : n;
    // (the loads of the first tile are under way while the search is finished)
    Fetched<Src> first_tile;
    WalkStates first_states;
    fetch(src, base + (long long)threadIdx.x * kItems, end, first_tile);
    if (ck_g) fetch_states(ck_g, ck_l, base + (long long)threadIdx.x * kItems, end, first_states);
    unsigned long long tau_bits = ~0ull;   // budget 0: nothing is above tau
    if (budget > 0) {
        bool ok;
        tau_bits = finish_search(sh, src, n, budget, limit, nb, hdr, lists, list_count, &ok);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            hdr->tau = tau_bits;   // for the report of the output kernel
            // (cannot happen with valid posteriors and a budget that fits)
            if (!ok) report(dev_status, sh.done == 2 ? HORA_ERR_INFEASIBLE : HORA_ERR_RANGE);
        }
        __syncthreads();   // sh is reused below
    }
    const bool d_vec = (reinterpret_cast<uintptr_t>(delta) & 15) == 0;
    const bool u_vec = (reinterpret_cast<uintptr_t>(util) & 15) == 0;
    const double limit_d = (double)limit;
    long long ks = 0, ts = 0;
    bool too_deep = false;
    for (long long t0 = base; t0 < end; t0 += kTile) {
        const long long pos = t0 + (long long)threadIdx.x * kItems;
        double a[kItems], b[kItems], s[kItems], g[kItems], e[kItems], lf[kItems];
        bool alive[kItems];
        if (t0 != base) {
            fetch(src, pos, end, first_tile);
            if (ck_g) fetch_states(ck_g, ck_l, pos, end, first_states);
        }
        unpack(src, first_tile, a, b);
        // the gains go on from where the first narrowing pass left them (above tau) ...
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            s[j] = a[j] + b[j];
            if (ck_g) { g[j] = first_states.g[j]; lf[j] = (double)first_states.l[j]; }
            else { g[j] = gain_first(a[j], s[j]); lf[j] = 0.0; }
            e[j] = 1.0;
            alive[j] = pos + j < end;
        }
        bool any;
        do {
            any = false;
#pragma unroll
            for (int j = 0; j < kItems; ++j) {
                const bool act = alive[j] && lf[j] < limit_d && gain_bits(g[j]) > tau_bits;
                if (act) {
                    g[j] = gain_next(g[j], b[j], s[j], lf[j]);
                    lf[j] += 1.0;
                }
                any |= act;
            }
        } while (any);
        // ... and the survival product follows from the gain the walk ended with, without a walk of
        // its own: App. A gives E(l) = B(alpha, beta + l) / B(alpha, beta) and M(l) =
        // B(alpha + 1, beta + l) / B(alpha, beta), whose ratio is alpha / (alpha + beta + l), so
        // E(k) = M(k) (alpha + beta + k) / alpha.  Two roundings on top of the gain's own (a few
        // 1e-16 of E per step, like the product's); E(0) = 1 exactly.
        if (util) {
#pragma unroll
            for (int j = 0; j < kItems; ++j) e[j] = lf[j] > 0.0 ? (g[j] * (s[j] + lf[j])) / a[j] : 1.0;
        }
        // what is final already is stored as such: k and U = 1 - E(k); a tied prompt leaves k
        // with the flag, and what its utility becomes if the tie pass gives it a unit,
        // 1 - E(k + 1), where its walk state was (nobody reads that again)
        int packed[kItems];
        double uu[kItems];
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            const bool at_limit = !(lf[j] < limit_d);
            const bool tied = alive[j] && !at_limit && gain_bits(g[j]) == tau_bits;
            // stopped by the library's depth bound with gains above tau left
            too_deep |= alive[j] && at_limit && depth_capped != 0 && gain_bits(g[j]) > tau_bits;
            const int k = alive[j] ? (int)lf[j] : 0;
            packed[j] = (int)((unsigned)k | (tied ? kTiedBit : 0u));
            uu[j] = 1.0 - e[j];
            if (tied && util) ck_g[pos + j] = 1.0 - surv_next(e[j], b[j], s[j], lf[j]);   // (ties need a budget: ck_g is there)
            ks += k;
            ts += tied ? 1 : 0;
        }
        store_items<v4i, int32_t>(delta, pos, end, d_vec, packed);
        if (util) store_items<v2d, double>(util, pos, end, u_vec, uu);
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
    if (too_deep) report(dev_status, HORA_ERR_UNSUPPORTED);
}
template <class Src>
__global__ __launch_bounds__(kBig) void k_bisect_finalize(Src src, long long n, long long chunk, long long budget,
    long long limit, int depth_capped, int nb, AllocHeader* __restrict__ hdr,
    const unsigned long long* __restrict__ lists, const int* __restrict__ list_count, double* ck_g,
    const int32_t* __restrict__ ck_l, int32_t* __restrict__ delta, double* __restrict__ util,
    long long* __restrict__ block_ksum, long long* __restrict__ block_tied, int32_t* dev_status) {
    bisect_finalize<Src>(src, n, chunk, budget, limit, depth_capped, nb, hdr, lists, list_count, ck_g, ck_l, delta, util, block_ksum, block_tied, dev_status);
}

// ----------------------------------------------------------------------------------
// 5b. Outputs.  Every workgroup adds up the per-workgroup sums of 5a (what lies before it,
// and the totals, from which r = budget - sum k follows), then runs the tie pass over its
// chunk.  delta[i] holds k_i, with the tied flag in bit 31 for a tied prompt; util[i] holds
// U_i(k_i), and for a tied prompt win_util[i] what it becomes with one more unit: only tied
// prompts are written again, the utility only of those that get a unit.
// ----------------------------------------------------------------------------------
template <class Src, int kOff>
__device__ __forceinline__ void bisect_write(Src src, long long n, int g0, long long chunk, int nb,
                                                       long long budget, const AllocHeader* __restrict__ hdr,
                                                       const long long* __restrict__ block_ksum,
                                                       const long long* __restrict__ block_tied,
                                                       const double* __restrict__ win_util,
                                                       int32_t* __restrict__ delta, double* __restrict__ util,
                                                       void* __restrict__ group_off,
                                                       hora_alloc_summary* __restrict__ summary,
                                                       int32_t* dev_status) {
    __shared__ EmitShared s_emit;
    constexpr int kSumWaves = kMaxBlocks / kWave;   // the wavefronts that hold the workgroups' sums
    __shared__ long long s_pre[4][kSumWaves];
    if (wave_id() < kSumWaves) {   // (the other wavefronts would add up zeros on the same vector units)
        static_assert(kMaxBlocks <= kBig && kMaxBlocks % kWave == 0, "one thread per workgroup sum");
        const int t = (int)threadIdx.x;
        const long long kv = t < nb ? block_ksum[t] : 0, tv = t < nb ? block_tied[t] : 0;
        const long long k_all = (long long)wave_total_u64((unsigned long long)kv), t_all = wave_total_i64(tv);
        const long long k_bef = (long long)wave_total_u64((unsigned long long)(t < (int)blockIdx.x ? kv : 0));
        const long long t_bef = wave_total_i64(t < (int)blockIdx.x ? tv : 0);
        if (lane_id() == 0) {
            s_pre[0][wave_id()] = k_all; s_pre[1][wave_id()] = t_all;
            s_pre[2][wave_id()] = k_bef; s_pre[3][wave_id()] = t_bef;
        }
    }
    __syncthreads();
    long long k_all = 0, t_all = 0, k_bef = 0, t_bef = 0;
#pragma unroll
    for (int w = 0; w < kSumWaves; ++w) {
        k_all += s_pre[0][w]; t_all += s_pre[1][w]; k_bef += s_pre[2][w]; t_bef += s_pre[3][w];
    }
    const long long r = budget - k_all;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (r < 0 || r > t_all) report(dev_status, HORA_ERR_RANGE);   // invalid posteriors upstream
        if (summary) {
            summary->tau = budget > 0 ? __longlong_as_double((long long)hdr->tau) : 0.0;
            summary->count_gt = k_all;
            summary->tie_units = r;
            summary->tie_prompts = t_all;
        }
    }
    const long long base = (long long)blockIdx.x * chunk;
    const long long end = base + chunk < n ? base + chunk : n;
    const bool d_vec = (reinterpret_cast<uintptr_t>(delta) & 15) == 0;
    const bool o_vec = (reinterpret_cast<uintptr_t>(group_off) & 15) == 0;
    EmitCarry carry = {t_bef, k_bef};
    int parity = 0;
    for (long long t0 = base; t0 < end; t0 += kTile, parity ^= 1) {
        const long long pos = t0 + (long long)threadIdx.x * kItems;
        int raw[kItems];
        load_items_i32(delta, pos, end, d_vec, 0, raw);
        int kk[kItems], td[kItems], dd[kItems];
        bool win[kItems];
        double with_unit[kItems];   // a tied prompt's utility if it gets a unit: on its way during the tie pass
#pragma unroll
        for (int j = 0; j < kItems; ++j) {
            kk[j] = (int)((unsigned)raw[j] & ~kTiedBit);
            td[j] = ((unsigned)raw[j] & kTiedBit) ? 1 : 0;
            with_unit[j] = 0.0;
            if (util && td[j]) with_unit[j] = win_util[pos + j];   // (tied: a prompt below `end`)
        }
        emit_tile<kOff, true>(parity, pos, end, n, g0, r, kk, td, carry, dd, win, delta, group_off, d_vec, o_vec,
                              &s_emit);
        if (util) {
#pragma unroll
            for (int j = 0; j < kItems; ++j)
                if (win[j]) util[pos + j] = with_unit[j];   // (a tied prompt that gets a unit)
        }
    }
}
template <class Src, int kOff>
__global__ __launch_bounds__(kBig) void k_bisect_write(Src src, long long n, int g0, long long chunk, int nb,
    long long budget, const AllocHeader* __restrict__ hdr, const long long* __restrict__ block_ksum,
    const long long* __restrict__ block_tied, const double* __restrict__ win_util, int32_t* __restrict__ delta,
    double* __restrict__ util, void* __restrict__ group_off, hora_alloc_summary* __restrict__ summary,
    int32_t* dev_status) {
    bisect_write<Src, kOff>(src, n, g0, chunk, nb, budget, hdr, block_ksum, block_tied, win_util, delta, util, group_off, summary, dev_status);
}

// ----------------------------------------------------------------------------------
// A batch of at most one tile: the one workgroup there is runs the six steps above one after
// the other in a single launch.  The same code; where a launch was, a barrier, which inside a
// workgroup orders the steps' writes to the workspace before the next step's reads.  Five
// launches less, which is worth 5 us (learned-prior posteriors, 8 units per prompt: 57 -> 51 us
// at 1024 prompts, 75 -> 70 at 4096): with one tile the time is the tile's own critical path,
// the walks of its deepest prompts in the estimate, the coarse count and the passes.
// ----------------------------------------------------------------------------------
template <class Src, int kOff>
__global__ __launch_bounds__(kBig) void k_bisect_tile(Src src, long long n, int g0, BudgetShares shares,
                                                      long long budget, long long limit, int depth_capped,
                                                      long long chunk, CoarseSlot* slots, AllocHeader* hdr,
                                                      SelectBins* bins, unsigned long long* lists, int* list_count,
                                                      double* ck_g, int32_t* ck_l, long long* block_ksum,
                                                      long long* block_tied, int32_t* delta, double* util,
                                                      void* group_off, hora_alloc_summary* summary,
                                                      int32_t* dev_status) {
    if (budget > 0) {   // (without a budget there is no search and no walk state)
        bisect_coarse<Src, false>(src, n, shares, limit, chunk, slots, hdr, ck_g, ck_l, dev_status);
        __syncthreads();
        bisect_pass<Src, 0>(src, n, budget, limit, chunk, 1, slots, hdr, bins, lists, list_count, ck_g, ck_l);
        __syncthreads();
        {   // what k_bisect_reduce does, for one workgroup's tallies
            const unsigned flags = hdr->slot[1].flags;
            if ((flags & kFlagPending) != 0) {   // uniform
                if (threadIdx.x == 0) hdr->lists_ok = ((flags & kFlagCollected) != 0 && list_count[0] >= 0) ? 1u : 0u;
                if (threadIdx.x < kBins) {
                    SelectBins* totals = bins + kMaxBlocks;
                    totals->cnt[threadIdx.x] = bins[0].cnt[threadIdx.x];
                    totals->vmax[threadIdx.x] = bins[0].vmax[threadIdx.x];
                    totals->vmin_inv[threadIdx.x] = bins[0].vmin_inv[threadIdx.x];
                }
            }
        }
        __syncthreads();
        bisect_pass<Src, 1>(src, n, budget, limit, chunk, 1, slots, hdr, bins, lists, list_count, ck_g, ck_l);
        __syncthreads();
    }
    bisect_finalize<Src>(src, n, chunk, budget, limit, depth_capped, 1, hdr, lists, list_count,
                         budget > 0 ? ck_g : nullptr, budget > 0 ? ck_l : nullptr, delta, util, block_ksum, block_tied,
                         dev_status);
    __syncthreads();
    bisect_write<Src, kOff>(src, n, g0, chunk, 1, budget, hdr, block_ksum, block_tied, ck_g, delta, util, group_off,
                            summary, dev_status);
}

// ----------------------------------------------------------------------------------
// Host side
// ----------------------------------------------------------------------------------
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
    // gains one prompt may contribute: the caller's cap, the budget, the library's depth bound
    long long wanted = a.delta_max > 0 ? (long long)a.delta_max : a.budget;
    if (wanted > a.budget) wanted = a.budget;
    const int depth_capped = wanted > (long long)HORA_MAX_DEPTH ? 1 : 0;
    const long long limit = depth_capped ? (long long)HORA_MAX_DEPTH : wanted;
    const long long tiles = (n + kTile - 1) / kTile;
    // deep budgets get the kernels that can pool their walks (see estimate_depth: pooling needs a
    // mean walk of more than 32 steps; the mean is budget / n)
    const bool deep = a.budget > kDeepRatio * n;
    const int mode = a.group_off ? (a.off_t == HORA_I32 ? 1 : 2) : 0;
    if (tiles == 1 && !deep) {   // one workgroup, one launch
        BudgetShares shares{0ull, 0ull, 0ull, 0ull};
        if (a.budget > 0) {
            const unsigned long long b_u = (unsigned long long)a.budget, n_u = (unsigned long long)n;
            shares.sample = (b_u * kEstSamples + n_u - 1ull) / n_u;
            shares.per_prompt = b_u / n_u;
            shares.tile = (b_u * kTile + n_u - 1ull) / n_u;
            shares.last_tile = b_u;   // the only tile takes the whole budget
        }
#define HORA_LAUNCH_BISECT_TILE(M)                                                                                  \
    hipLaunchKernelGGL((k_bisect_tile<Src, M>), dim3(1), dim3(kBig), 0, a.stream, src, n, (int)a.g0, shares,       \
                       (long long)a.budget, limit, depth_capped, p.chunk, w.coarse, w.header, w.bins, w.lists,    \
                       w.list_count, w.ck_g, w.ck_l, w.block_ksum, w.block_tied, a.delta, a.util, a.group_off,    \
                       a.summary, a.dev_status)
        if (mode == 0) HORA_LAUNCH_BISECT_TILE(0);
        else if (mode == 1) HORA_LAUNCH_BISECT_TILE(1);
        else HORA_LAUNCH_BISECT_TILE(2);
#undef HORA_LAUNCH_BISECT_TILE
        return check_launch();
    }
    if (a.budget > 0) {
        // shares of the budget, rounded up (budget < 2^52, at most 2^12 prompts: no overflow)
        const unsigned long long b_u = (unsigned long long)a.budget, n_u = (unsigned long long)n;
        const unsigned long long n_last = n_u - (unsigned long long)(tiles - 1) * kTile;
        BudgetShares shares;
        shares.sample = (b_u * kEstSamples + n_u - 1ull) / n_u;
        shares.per_prompt = b_u / n_u;
        shares.tile = (b_u * kTile + n_u - 1ull) / n_u;
        shares.last_tile = (b_u * n_last + n_u - 1ull) / n_u;
        if (deep)
            hipLaunchKernelGGL((k_bisect_coarse<Src, true>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, shares,
                               limit, p.chunk, w.coarse, w.header, w.ck_g, w.ck_l, a.dev_status);
        else
            hipLaunchKernelGGL((k_bisect_coarse<Src, false>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, shares,
                               limit, p.chunk, w.coarse, w.header, w.ck_g, w.ck_l, a.dev_status);
        hipLaunchKernelGGL((k_bisect_pass<Src, 0>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, (long long)a.budget,
                           limit, p.chunk, tiles, (const CoarseSlot*)w.coarse, w.header, w.bins, w.lists,
                           w.list_count, w.ck_g, w.ck_l);
        hipLaunchKernelGGL(k_bisect_reduce, dim3(kBins / kReduceBins), dim3(kThreads), 0, a.stream, p.nb, 0,
                           w.header, w.bins, (const int*)w.list_count);
        hipLaunchKernelGGL((k_bisect_pass<Src, 1>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, (long long)a.budget,
                           limit, p.chunk, tiles, (const CoarseSlot*)w.coarse, w.header, w.bins, w.lists,
                           w.list_count, w.ck_g, w.ck_l);
    }
    // (without a budget there was no search and no walk state)
    double* state_g = a.budget > 0 ? w.ck_g : nullptr;
    const int32_t* state_l = a.budget > 0 ? w.ck_l : nullptr;
    hipLaunchKernelGGL((k_bisect_finalize<Src>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, p.chunk,
                       (long long)a.budget, limit, depth_capped, p.nb, w.header, (const unsigned long long*)w.lists,
                       (const int*)w.list_count, state_g, state_l, a.delta, a.util, w.block_ksum, w.block_tied,
                       a.dev_status);
#define HORA_LAUNCH_BISECT_WRITE(M)                                                                       \
    hipLaunchKernelGGL((k_bisect_write<Src, M>), dim3(p.nb), dim3(kBig), 0, a.stream, src, n, (int)a.g0,  \
                       p.chunk, p.nb, (long long)a.budget, (const AllocHeader*)w.header,                  \
                       (const long long*)w.block_ksum, (const long long*)w.block_tied,                    \
                       (const double*)w.ck_g, a.delta, a.util,                                            \
                       a.group_off, a.summary, a.dev_status)
    if (mode == 0) HORA_LAUNCH_BISECT_WRITE(0);
    else if (mode == 1) HORA_LAUNCH_BISECT_WRITE(1);
    else HORA_LAUNCH_BISECT_WRITE(2);
#undef HORA_LAUNCH_BISECT_WRITE
    return check_launch();
}

int run_bisect_counts(const CountsSource& src, const CommonArgs& a, const Plan& p, const Workspace& w) {
    return run_bisect(src, a, p, w);
}
int run_bisect_posterior(const PosteriorSource& src, const CommonArgs& a, const Plan& p, const Workspace& w) {
    return run_bisect(src, a, p, w);
}

}  // namespace hora
