/*
 * TEST ORACLE -- not part of the product.
 *
 * Plain, slow, single-threaded CPU statement of what HORA's rollout layer
 * computes, written from the paper (Sec. 3.1, Sec. 3.2, Alg. 1, App. A, App. E)
 * in IEEE-754 binary64.  It exists so that tests and the benchmark's CPU
 * baseline have something independent to compare the GPU library with.  It
 * shares no code, header, table or helper with the GPU library, and nothing
 * in the product may call it.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -shared -fPIC
 * (no FMA contraction and no reassociation: the order of every floating-point
 * operation below is part of the definition of the result, see "canonical
 * gain").
 *
 * Every pointer is host memory owned by the caller.
 *
 * Parity pins (tests/test_oracle_*.py): all functions here are pinned by
 * closed forms, exact rational arithmetic, numerical integration, brute
 * force or invariants; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define ORACLE_OK 0
#define ORACLE_ERR_INVALID (-1)
#define ORACLE_ERR_INFEASIBLE (-2)
#define ORACLE_ERR_NOMEM (-3)
#define ORACLE_ERR_RANGE (-4)

/* ---------------------------------------------------------------------------
 * Marginal hit utility (Sec. 3.2 "Greedy allocator", Eq. 5; App. A).
 *
 * M(l) = B(alpha+1, beta+l) / B(alpha, beta), evaluated by the paper's stable
 * update M(0) = alpha/(alpha+beta), M(l+1) = M(l) (beta+l) / (alpha+beta+l+1).
 *
 * Canonical gain: the binary64 value produced by exactly this sequence --
 * s = alpha+beta; M(0) = alpha/s; M(l+1) = (M(l) * (beta+l)) / (s + (l+1)) --
 * one multiply, then one divide, always walked from l = 0.  The paper's argmax
 * has no tie rule; ordering by (canonical gain, prompt index) is this library's
 * reading, so the rounding of this sequence is part of the result.
 * ------------------------------------------------------------------------- */
static inline double gain_first(double alpha, double beta) {
    return alpha / (alpha + beta);
}

static inline double gain_next(double m, double alpha, double beta, int64_t l) {
    /* M(l+1) from M(l) */
    double num = beta + (double)l;
    double den = (alpha + beta) + (double)(l + 1);
    return (m * num) / den;
}

void hora_oracle_marginal_gains(double alpha, double beta, int64_t count, double *out) {
    if (count <= 0) return;
    double m = gain_first(alpha, beta);
    out[0] = m;
    for (int64_t l = 0; l + 1 < count; ++l) {
        m = gain_next(m, alpha, beta, l);
        out[l + 1] = m;
    }
}

/* ---------------------------------------------------------------------------
 * Hit utility (Sec. 3.2 Eq. 3; App. A closed form U = 1 - B(a, b+D)/B(a, b)).
 * B(a, b+D)/B(a, b) = prod_{k<D} (b+k)/(a+b+k); evaluated as the product
 * recurrence E_0 = 1, E_{k+1} = (E_k * (b+k)) / (a+b+k), U = 1 - E_D.
 * ------------------------------------------------------------------------- */
double hora_oracle_hit_utility(double alpha, double beta, int64_t delta) {
    double e = 1.0;
    double s = alpha + beta;
    for (int64_t k = 0; k < delta; ++k) {
        e = (e * (beta + (double)k)) / (s + (double)k);
    }
    return 1.0 - e;
}

/* ---------------------------------------------------------------------------
 * Phase A posterior (Sec. 3.2 Eq. 2; Alg. 1 "Phase A"):
 * alpha_i = alpha0 + c_i, beta_i = beta0 + G0 - c_i.
 * ------------------------------------------------------------------------- */
int hora_oracle_posterior(int64_t n, int32_t g0, const int32_t *c, double alpha0, double beta0,
                          double *alpha, double *beta) {
    if (n < 0 || g0 < 0 || !(alpha0 > 0.0) || !(beta0 > 0.0)) return ORACLE_ERR_INVALID;
    for (int64_t i = 0; i < n; ++i) {
        if (c[i] < 0 || c[i] > g0) return ORACLE_ERR_RANGE;
        alpha[i] = alpha0 + (double)c[i];
        beta[i] = beta0 + (double)(g0 - c[i]);
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Phase B greedy allocation (Alg. 1 "Phase B"; Prop. 1).
 *
 * Literal form: B times, pick the prompt whose current marginal gain
 * M_i(Delta_i) is largest and give it one more rollout.  Ties go to the lower
 * prompt index.  A prompt that has reached delta_max (> 0) leaves the
 * competition.  This version finds the argmax by a linear scan: O(B*N), for
 * small inputs and for checking the heap version below.
 * ------------------------------------------------------------------------- */
int hora_oracle_allocate_scan(int64_t n, const double *alpha, const double *beta, int64_t budget,
                              int64_t delta_max, int64_t *delta) {
    if (n < 0 || budget < 0) return ORACLE_ERR_INVALID;
    if (budget > 0 && n == 0) return ORACLE_ERR_INFEASIBLE;
    if (delta_max > 0 && (budget + delta_max - 1) / delta_max > n) /* budget > n * delta_max */
        return ORACLE_ERR_INFEASIBLE;
    double *gain = (double *)malloc((size_t)(n > 0 ? n : 1) * sizeof(double));
    if (!gain) return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < n; ++i) {
        delta[i] = 0;
        gain[i] = gain_first(alpha[i], beta[i]);
    }
    for (int64_t b = 0; b < budget; ++b) {
        int64_t best = -1;
        for (int64_t i = 0; i < n; ++i) {
            if (delta_max > 0 && delta[i] >= delta_max) continue;
            if (best < 0 || gain[i] > gain[best]) best = i; /* strict: lower index wins ties */
        }
        if (best < 0) { free(gain); return ORACLE_ERR_INFEASIBLE; }
        gain[best] = gain_next(gain[best], alpha[best], beta[best], delta[best]);
        delta[best] += 1;
    }
    free(gain);
    return ORACLE_OK;
}

/* Same allocation with the argmax kept in a binary max-heap ordered by
 * (gain descending, prompt index ascending): O(B log N). */
typedef struct { double gain; int64_t idx; } heap_item;

static inline int item_before(const heap_item *x, const heap_item *y) {
    if (x->gain > y->gain) return 1;
    if (x->gain < y->gain) return 0;
    return x->idx < y->idx;
}

static void sift_down(heap_item *h, int64_t size, int64_t pos) {
    heap_item v = h[pos];
    for (;;) {
        int64_t child = 2 * pos + 1;
        if (child >= size) break;
        if (child + 1 < size && item_before(&h[child + 1], &h[child])) child += 1;
        if (!item_before(&h[child], &v)) break;
        h[pos] = h[child];
        pos = child;
    }
    h[pos] = v;
}

int hora_oracle_allocate(int64_t n, const double *alpha, const double *beta, int64_t budget,
                         int64_t delta_max, int64_t *delta) {
    if (n < 0 || budget < 0) return ORACLE_ERR_INVALID;
    if (budget > 0 && n == 0) return ORACLE_ERR_INFEASIBLE;
    if (delta_max > 0 && (budget + delta_max - 1) / delta_max > n) /* budget > n * delta_max */
        return ORACLE_ERR_INFEASIBLE;
    heap_item *h = (heap_item *)malloc((size_t)(n > 0 ? n : 1) * sizeof(heap_item));
    if (!h) return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < n; ++i) {
        delta[i] = 0;
        h[i].gain = gain_first(alpha[i], beta[i]);
        h[i].idx = i;
    }
    int64_t size = n;
    for (int64_t pos = size / 2 - 1; pos >= 0; --pos) sift_down(h, size, pos);
    for (int64_t b = 0; b < budget; ++b) {
        if (size == 0) { free(h); return ORACLE_ERR_INFEASIBLE; }
        int64_t i = h[0].idx;
        double next = gain_next(h[0].gain, alpha[i], beta[i], delta[i]);
        delta[i] += 1;
        if (delta_max > 0 && delta[i] >= delta_max) {
            h[0] = h[size - 1];
            size -= 1;
        } else {
            h[0].gain = next;
        }
        if (size > 0) sift_down(h, size, 0);
    }
    free(h);
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Sharded Phase B (App. C): the batch is cut into consecutive shards and the
 * greedy loop above is run on every shard by itself, with the shard's own
 * budget; the optimality statement then holds inside each shard.  Shard s holds
 * prompts shard_off[s] .. shard_off[s+1]-1.
 * ------------------------------------------------------------------------- */
int hora_oracle_allocate_sharded(int64_t n, const double *alpha, const double *beta, int64_t n_shards,
                                 const int64_t *shard_off, const int64_t *shard_budget,
                                 int64_t delta_max, int64_t *delta) {
    if (n < 0 || n_shards < 0) return ORACLE_ERR_INVALID;
    if (n_shards == 0) return n == 0 ? ORACLE_OK : ORACLE_ERR_INVALID;
    if (shard_off[0] != 0 || shard_off[n_shards] != n) return ORACLE_ERR_RANGE;
    for (int64_t s = 0; s < n_shards; ++s) {
        int64_t lo = shard_off[s], hi = shard_off[s + 1];
        if (hi < lo) return ORACLE_ERR_RANGE;
        int rc = hora_oracle_allocate(hi - lo, alpha + lo, beta + lo, shard_budget[s], delta_max, delta + lo);
        if (rc != ORACLE_OK) return rc;
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Group assembly (Alg. 1 "group assembly"; Sec. 3.2): G_i = G0 + Delta_i,
 * responses of prompt i stored contiguously, pre-rollouts first.
 * off[0] = 0, off[i+1] = off[i] + G_i.
 * ------------------------------------------------------------------------- */
void hora_oracle_group_offsets(int64_t n, int32_t g0, const int64_t *delta, int64_t *off) {
    off[0] = 0;
    for (int64_t i = 0; i < n; ++i) off[i + 1] = off[i] + (int64_t)g0 + delta[i];
}

/* ---------------------------------------------------------------------------
 * Group-relative advantages on variable-size groups.
 *
 * mode 0, GRPO (Sec. 3.1): A_j = (R_j - mean(R)) / (std(R) + eps) over the G_i
 * rewards of the group; std is the population one (ddof = 0) unless ddof = 1.
 * When the empirical standard deviation is zero the advantage is zero: a group
 * whose rewards are all equal gets exactly 0 (eps plays no part).  A group with
 * G_i - ddof <= 0 gets 0 as well.
 *
 * mode 1, RLOO (Sec. 4 "compatible with GRPO-family objectives"; App. E):
 * leave-one-out baseline, A_j = R_j - (sum_{k != j} R_k) / (G_i - 1), evaluated
 * as R_j - (S - R_j)/(G_i - 1) with S the group sum; G_i = 1 gives 0.
 *
 * mode 2, centred only: A_j = R_j - mean(R), the GRPO advantage without the
 * division by the standard deviation (the variant that objectives of the
 * Dr. GRPO kind use; the paper's runs keep the normalised form of Sec. 3.1).
 * A group whose rewards are all equal gets exactly 0 here too.
 * ------------------------------------------------------------------------- */
int hora_oracle_group_advantage(int64_t n_groups, const int64_t *off, const double *reward,
                                double *adv, int32_t mode, double eps, int32_t ddof) {
    if (n_groups < 0 || mode < 0 || mode > 2 || (ddof != 0 && ddof != 1) || eps < 0.0)
        return ORACLE_ERR_INVALID;
    for (int64_t g = 0; g < n_groups; ++g) {
        int64_t lo = off[g], hi = off[g + 1];
        if (hi < lo) return ORACLE_ERR_RANGE;
        int64_t size = hi - lo;
        if (size == 0) continue;
        double sum = 0.0;
        for (int64_t j = lo; j < hi; ++j) sum += reward[j];
        if (mode == 1) {
            for (int64_t j = lo; j < hi; ++j) {
                if (size == 1) adv[j] = 0.0;
                else adv[j] = reward[j] - (sum - reward[j]) / (double)(size - 1);
            }
            continue;
        }
        int all_equal = 1;
        for (int64_t j = lo + 1; j < hi; ++j)
            if (reward[j] != reward[lo]) { all_equal = 0; break; }
        if (all_equal || (mode == 0 && size - ddof <= 0)) {
            for (int64_t j = lo; j < hi; ++j) adv[j] = 0.0;
            continue;
        }
        double mean = sum / (double)size;
        if (mode == 2) {
            for (int64_t j = lo; j < hi; ++j) adv[j] = reward[j] - mean;
            continue;
        }
        double ss = 0.0;
        for (int64_t j = lo; j < hi; ++j) {
            double d = reward[j] - mean;
            ss += d * d;
        }
        double sd = sqrt(ss / (double)(size - ddof));
        for (int64_t j = lo; j < hi; ++j) adv[j] = (reward[j] - mean) / (sd + eps);
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Per-token advantage (Sec. 3.1, objective and advantage definition): the
 * advantage of a response does not depend on the token position, so every
 * token t of response j, tok_off[j] <= t < tok_off[j+1], carries adv[j].
 * ------------------------------------------------------------------------- */
int hora_oracle_token_broadcast(int64_t n_resp, const double *adv, const int64_t *tok_off,
                                double *tok_adv) {
    if (n_resp < 0) return ORACLE_ERR_INVALID;
    if (n_resp > 0 && tok_off[0] != 0) return ORACLE_ERR_RANGE;
    for (int64_t j = 0; j < n_resp; ++j) {
        if (tok_off[j + 1] < tok_off[j]) return ORACLE_ERR_RANGE;
        for (int64_t t = tok_off[j]; t < tok_off[j + 1]; ++t) tok_adv[t] = adv[j];
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Loss weight of every token of a response (Sec. 3.1 objective; Sec. 3.2
 * "Training objective with variable-size groups"): the objective averages over
 * the tokens of a response (1/|o_j|) and over the responses of a prompt, and
 * with variable-size groups the 1/G in front becomes 1/G_i, so that every
 * prompt weighs the same however many additional rollouts it received.
 *   length_const <= 0:  w_j = 1 / (G_i * |o_j|)
 *   length_const  > 0:  w_j = 1 / (G_i * length_const)   (a constant in place of
 *                       |o_j|: length normalisation of the Dr. GRPO kind, which
 *                       the paper's runs use; the constant is the caller's)
 * A response without tokens gets weight 0.  One multiply, then one divide.
 * ------------------------------------------------------------------------- */
int hora_oracle_response_weights(int64_t n_groups, const int64_t *group_off, const int64_t *tok_off,
                                 double length_const, double *weight) {
    if (n_groups < 0) return ORACLE_ERR_INVALID;
    for (int64_t g = 0; g < n_groups; ++g) {
        int64_t lo = group_off[g], hi = group_off[g + 1];
        if (hi < lo) return ORACLE_ERR_RANGE;
        double size = (double)(hi - lo);
        for (int64_t j = lo; j < hi; ++j) {
            int64_t len = tok_off[j + 1] - tok_off[j];
            if (len < 0) return ORACLE_ERR_RANGE;
            if (len == 0) { weight[j] = 0.0; continue; }
            double norm = length_const > 0.0 ? length_const : (double)len;
            weight[j] = 1.0 / (size * norm);
        }
    }
    return ORACLE_OK;
}

/* ---------------------------------------------------------------------------
 * Baseline allocation rules the paper compares with (Sec. 5, Table 2; Sec. 4).
 *   rule 0, uniform: the fixed-group baseline; every prompt gets the same
 *           number of additional rollouts.
 *   rule 1, hard-first: the Phase-B budget goes only to prompts with c_i = 0.
 * The paper does not say how the budget is split inside the eligible set, nor
 * what happens when no prompt has c_i = 0.  Reading taken: the eligible prompts
 * share the budget evenly, the remainder going one unit each to the lowest
 * indices; with no eligible prompt the rule falls back to uniform.
 * ------------------------------------------------------------------------- */
int hora_oracle_allocate_baseline(int64_t n, const int32_t *c, int64_t budget, int64_t delta_max,
                                  int32_t rule, int64_t *delta) {
    if (n < 0 || budget < 0 || (rule != 0 && rule != 1)) return ORACLE_ERR_INVALID;
    if (budget > 0 && n == 0) return ORACLE_ERR_INFEASIBLE;
    int64_t eligible = 0;
    if (rule == 1)
        for (int64_t i = 0; i < n; ++i) eligible += c[i] == 0;
    int all = (rule == 0) || eligible == 0;
    if (all) eligible = n;
    int64_t each = eligible > 0 ? budget / eligible : 0;
    int64_t rest = eligible > 0 ? budget - each * eligible : 0;
    if (delta_max > 0 && each + (rest > 0) > delta_max) return ORACLE_ERR_INFEASIBLE;
    int64_t rank = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (all || c[i] == 0) {
            delta[i] = each + (rank < rest);
            rank += 1;
        } else {
            delta[i] = 0;
        }
    }
    return ORACLE_OK;
}
