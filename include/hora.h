/*
 * hora.h -- C ABI of the HORA rollout-layer library for AMD MI355X (gfx950).
 *
 * HORA (Hit-Utility Optimal Rollout Allocation) splits the rollouts of one
 * RLVR training step into G0 pre-rollouts per prompt (Phase A) and a budget of
 * additional rollouts (Phase B) that is distributed over the prompts so as to
 * maximise the total posterior "hit utility".  This library holds the
 * data-parallel part between rollout generation and the policy loss:
 *
 *   Phase-A counts c_i -> Beta posterior -> marginal gains -> optimal budgeted
 *   allocation Delta_i -> variable-size groups G_i = G0 + Delta_i ->
 *   group-relative advantages (GRPO or RLOO) -> per-token advantages.
 *
 * Conventions that hold for every entry point unless it says otherwise:
 *  - Pointers marked "device" are GPU global memory owned by the caller and
 *    must stay valid until the work enqueued on `stream` has finished.  The
 *    library allocates nothing and copies nothing between host and device.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls validate their host-visible arguments, enqueue kernels on `stream`
 *    and return without synchronising.
 *  - The return value reports argument / launch errors.  Errors that depend on
 *    device data (a count outside [0, G0], offsets that decrease, ...) are
 *    reported through `dev_status`, a device int32 that the library only ever
 *    writes when it finds such an error (it then holds the hora_status code).
 *    The caller zeroes it once and reads it after synchronising; it is sticky
 *    across calls.  After a data error the outputs of that call are
 *    unspecified, but no access leaves the caller's buffers.
 *  - n = 0 and budget = 0 are valid and give empty / all-zero outputs.
 */
#ifndef HORA_H
#define HORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HORA_OK = 0,
    HORA_ERR_INVALID_ARG = -1, /* null pointer, negative size, unknown enum, misaligned buffer */
    HORA_ERR_INFEASIBLE = -2,  /* budget cannot be placed: n == 0, or budget > n * delta_max   */
    HORA_ERR_WORKSPACE = -3,   /* workspace missing or smaller than *_workspace_bytes()        */
    HORA_ERR_RANGE = -4,       /* device data out of range (via dev_status)                    */
    HORA_ERR_HIP = -5,         /* a HIP runtime call or kernel launch failed                   */
    HORA_ERR_UNSUPPORTED = -6  /* size outside what this entry point / method handles          */
} hora_status;

typedef enum { HORA_ADV_GRPO = 0, HORA_ADV_RLOO = 1, HORA_ADV_CENTER = 2 } hora_adv_mode;
typedef enum { HORA_F32 = 0, HORA_F64 = 1 } hora_ftype;
typedef enum { HORA_I32 = 0, HORA_I64 = 1 } hora_itype;

/* How hora_allocate finds the allocation.  All methods return bit-identical results. */
typedef enum {
    HORA_ALLOC_AUTO = 0,   /* the library picks (CLASS when g0 allows it, else BISECT)             */
    HORA_ALLOC_CLASS = 1,  /* shared prior only: histogram of c, threshold solved per class       */
    HORA_ALLOC_BISECT = 2  /* bisection on the gain threshold with per-prompt monotone searches   */
} hora_alloc_method;

/* Baseline allocation rules (hora_allocate_baseline). */
typedef enum {
    HORA_RULE_UNIFORM = 0,    /* the same number of additional rollouts for every prompt        */
    HORA_RULE_HARD_FIRST = 1  /* the budget goes only to prompts with c_i = 0 (Sec. 5, Table 2) */
} hora_baseline_rule;

/* Largest G0 the CLASS method handles (one wavefront lane per class c = 0..G0). */
#define HORA_CLASS_MAX_G0 63

/*
 * Largest number of additional rollouts one prompt may receive in one call.  A prompt's
 * marginal gains are evaluated one after the other (each from the one before), so this
 * bounds the longest serial chain a kernel can run.  A budget above n * HORA_MAX_DEPTH is
 * refused on the host (HORA_ERR_UNSUPPORTED); an allocation in which the data would send
 * more than this to a single prompt is reported through dev_status (HORA_ERR_UNSUPPORTED).
 * A call whose deepest prompt comes near the bound runs for about a second on the GPU,
 * whatever the method: the chain is serial.
 */
#define HORA_MAX_DEPTH (1 << 20)

/* Optional device-side report of one allocation (all fields written by the call). */
typedef struct {
    double tau;           /* threshold gain: the budget-th largest marginal gain (0 if budget = 0) */
    int64_t count_gt;     /* number of (prompt, l) pairs whose gain is > tau                       */
    int64_t tie_units;    /* budget - count_gt: units handed to prompts tied at tau, by index      */
    int64_t tie_prompts;  /* prompts whose next gain equals tau                                    */
} hora_alloc_summary;

const char *hora_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int hora_version(void);

/*
 * Marginal hit utility and hit utility tables (Sec. 3.2, Eq. 3 and Eq. 5; App. A).
 *
 * For every posterior (alpha[i], beta[i]), i < n, evaluates
 *   M_i(l) = B(alpha+1, beta+l) / B(alpha, beta),      l = 0 .. count-1
 *   U_i(l) = 1 - B(alpha, beta+l) / B(alpha, beta),    l = 0 .. count-1
 * in binary64 by the paper's recurrences, each step one multiply then one
 * divide, walked from l = 0:
 *   s = alpha+beta;  M(0) = alpha/s;  M(l+1) = (M(l) * (beta+l)) / (s + (l+1));
 *   E(0) = 1;  E(l+1) = (E(l) * (beta+l)) / (s + l);  U(l) = 1 - E(l).
 * These binary64 values are the "canonical gains" that order the allocation.
 *
 * alpha, beta : device, n doubles each, all > 0.
 * gains       : device out, count*n doubles, l-major: gains[l*n + i] = M_i(l).  Nullable.
 * util        : device out, count*n doubles, same layout: util[l*n + i] = U_i(l).  Nullable.
 */
int hora_marginal_gains(int64_t n, const double *alpha, const double *beta, int32_t count,
                        double *gains, double *util, void *stream);

/*
 * Bytes of workspace hora_allocate / hora_allocate_posterior / hora_allocate_baseline need
 * for n prompts (a workspace sized for n serves every smaller batch): about 10 MB plus 12
 * bytes per prompt (the threshold search keeps the state of every prompt's walk between its
 * kernels).  The workspace is device memory, 256-byte aligned, and needs no initialisation:
 * nothing is carried from one call to the next.  Two calls that may run concurrently need
 * separate workspaces.
 */
size_t hora_allocate_workspace_bytes(int64_t n, int32_t g0);

/*
 * Phase-B allocation under a shared prior (Sec. 3.2 Eq. 2-5, Alg. 1 Phase A/B, Prop. 1).
 *
 * Posterior of prompt i: alpha_i = alpha0 + c[i], beta_i = beta0 + g0 - c[i].
 * Result: delta maximises sum_i U_i(delta_i) subject to sum_i delta_i = budget,
 * 0 <= delta_i (<= delta_max if delta_max > 0).  By Prop. 1 this is the greedy
 * allocation, i.e. the `budget` largest elements of {M_i(l)} are selected and
 * delta_i counts those of prompt i.  The paper's argmax has no tie rule; here
 * elements are ordered by (canonical gain descending, prompt index ascending),
 * which makes delta unique and equal to a greedy run that prefers the lower
 * index among equal gains.
 *
 * The call evaluates the gain tables of the G0+1 classes afresh every time (its workspace
 * needs no preparation and keeps nothing).  For the batch of one training step (some
 * dozens to a thousand prompts) hora_allocate_sharded with a single shard returns the
 * same delta, util and offsets in one launch and keeps its tables between calls: 40 % of
 * the time at 60 prompts with 24 units each.
 *
 * n, g0     : number of prompts (>= 0) and pre-rollouts per prompt (>= 0).
 * c         : device, n int32, each in [0, g0] (else HORA_ERR_RANGE in dev_status).
 * alpha0, beta0 : prior, both > 0 and finite (the paper uses 1, 1).
 * budget    : Phase-B budget, >= 0; need not be a multiple of n.  HORA_ERR_UNSUPPORTED
 *             from 2^52 on, and above n * HORA_MAX_DEPTH (some prompt would have to receive
 *             more than HORA_MAX_DEPTH units).
 * delta_max : per-prompt cap; <= 0 means none (the paper states none).  A budget above
 *             n * delta_max gives HORA_ERR_INFEASIBLE.
 * method    : hora_alloc_method.
 * delta     : device out, n int32.
 * util      : device out, n doubles, U_i(delta_i) = 1 - E_i(delta_i) (App. A), U_i(0) = 0
 *             exactly.  HORA_ALLOC_CLASS takes E from the product recurrence; the bisection
 *             method takes it from the last gain of its search, E(k) = M(k) (alpha + beta + k)
 *             / alpha (the ratio of the two closed forms of App. A).  Both lie within a few
 *             1e-16 of E per step of the true value; U is a difference from 1, so its
 *             relative accuracy is that divided by U.  Nullable.
 * group_off : device out, n+1 offsets of type off_t: exclusive prefix sums of
 *             g0 + delta_i (group i holds responses group_off[i] .. group_off[i+1]-1,
 *             pre-rollouts first).  Nullable.  With HORA_I32 the total n*g0 + budget
 *             must be < 2^31 (else HORA_ERR_INVALID_ARG).
 * summary   : device out, one hora_alloc_summary.  Nullable.
 * dev_status: device, one int32, see the conventions above.  Required.
 * workspace : device, >= hora_allocate_workspace_bytes(n, g0).
 */
int hora_allocate(int64_t n, int32_t g0, const int32_t *c, double alpha0, double beta0,
                  int64_t budget, int32_t delta_max, int32_t method, int32_t *delta, double *util,
                  void *group_off, int32_t off_t, hora_alloc_summary *summary,
                  int32_t *dev_status, void *workspace, size_t workspace_bytes, void *stream);

/*
 * hora_allocate for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as hora_allocate, without the workspace: the kernels use a
 * buffer of HORA_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy on
 * every GPU the library runs on, held until the process ends).  The call allocates nothing.
 *
 *  - n above HORA_STATIC_MAX_PROMPTS gives HORA_ERR_UNSUPPORTED (use hora_allocate).
 *  - All calls on one GPU share that GPU's buffer: calls that may overlap on one GPU
 *    (different streams, different threads) race; serialise them or use hora_allocate with
 *    workspaces of their own.
 *  - The first call on a device looks up the buffer's address (hipGetSymbolAddress); make
 *    that call outside a stream capture.
 */
#define HORA_STATIC_MAX_PROMPTS (1 << 22)
#define HORA_STATIC_SCRATCH_BYTES (64u << 20)
int hora_allocate_static(int64_t n, int32_t g0, const int32_t *c, double alpha0, double beta0,
                         int64_t budget, int32_t delta_max, int32_t method, int32_t *delta, double *util,
                         void *group_off, int32_t off_t, hora_alloc_summary *summary,
                         int32_t *dev_status, void *stream);

/*
 * Phase-B allocation for per-prompt posteriors (App. D, prompt-conditioned prior:
 * alpha_i = s_i p_i + c_i, beta_i = s_i (1 - p_i) + G0 - c_i are formed by the caller).
 * Same result definition, outputs and conventions as hora_allocate; always uses the
 * bisection method.  g0 only enters group_off (pass 0 to get prefix sums of delta).
 *
 * alpha, beta : device, n doubles each, all > 0 and finite (else HORA_ERR_RANGE in dev_status).
 */
int hora_allocate_posterior(int64_t n, int32_t g0, const double *alpha, const double *beta,
                            int64_t budget, int32_t delta_max, int32_t *delta, double *util,
                            void *group_off, int32_t off_t, hora_alloc_summary *summary,
                            int32_t *dev_status, void *workspace, size_t workspace_bytes,
                            void *stream);

/*
 * The allocation rules the paper compares hit-utility allocation with, with the same
 * outputs as hora_allocate (util[i] is still the hit utility U_i(delta_i) of what the rule
 * hands out, so that rules can be compared on the paper's own objective, Eq. 4):
 *   HORA_RULE_UNIFORM    the fixed-group baseline (Sec. 4): every prompt gets
 *                        budget / n additional rollouts;
 *   HORA_RULE_HARD_FIRST the hard-first heuristic (Sec. 5, Table 2): the budget goes only
 *                        to the prompts with c_i = 0.
 * The paper does not say how the eligible prompts share the budget or what happens when
 * no prompt has c_i = 0: here they share it evenly, the remainder going one unit each to
 * the lowest prompt indices, and a batch without such a prompt is allocated uniformly.
 * A cap that the rule would exceed gives HORA_ERR_INFEASIBLE (return value where the
 * arguments alone show it, else dev_status).  g0 <= HORA_CLASS_MAX_G0.  summary: tau = 0,
 * count_gt = budget - tie_units, tie_units = the remainder, tie_prompts = eligible prompts.
 * Workspace and the other arguments: as for hora_allocate.
 */
int hora_allocate_baseline(int64_t n, int32_t g0, const int32_t *c, double alpha0, double beta0,
                           int64_t budget, int32_t delta_max, int32_t rule, int32_t *delta, double *util,
                           void *group_off, int32_t off_t, hora_alloc_summary *summary,
                           int32_t *dev_status, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Allocation statistics per Phase-A outcome (Sec. 4, "Allocation dynamics" and its figure: the
 * share of the prompts with c_i = k and the share of the Phase-B budget they received):
 *   class_count[k]  = #{i : c[i] = k},   class_budget[k] = sum of delta[i] over those prompts,
 * k = 0 .. g0.  Works on the result of any of the allocation calls.
 *
 * c, delta    : device, n int32 each (c[i] outside [0, g0] or delta[i] < 0: HORA_ERR_RANGE in
 *               dev_status, the prompt is left out).
 * class_count, class_budget : device out, g0 + 1 int64 each.  g0 <= HORA_CLASS_MAX_G0.
 */
int hora_allocation_shares(int64_t n, int32_t g0, const int32_t *c, const int32_t *delta,
                           int64_t *class_count, int64_t *class_budget, int32_t *dev_status, void *stream);

/*
 * Bytes of workspace hora_allocate_sharded needs for n_shards shards: the gain tables of
 * the G0+1 classes (kept from call to call and reused while the prior, G0 and the cap
 * stay the same) and the prefix sums of the shard budgets.  Device memory, 256-byte
 * aligned; it must be zero-filled once before its first use.  Two calls that may run
 * concurrently need separate workspaces.
 */
size_t hora_allocate_sharded_workspace_bytes(int64_t n_shards);

/*
 * Phase-B allocation run independently on shards of the batch (App. C: the paper runs
 * Phase B on four mini-batches of Gamma/4 prompts instead of the whole batch at once;
 * Prop. 1 then holds inside each shard and the total budget is unchanged).
 *
 * Shard s holds the prompts shard_off[s] .. shard_off[s+1]-1 and distributes
 * shard_budget[s] among them; its delta, util and summary are exactly those of
 * hora_allocate called on that slice of c with that budget (same prior, same cap, same
 * tie rule with the prompt index taken inside the batch).  group_off runs over the
 * whole batch: exclusive prefix sums of g0 + delta_i over all n prompts.
 *
 * shard_off    : device, n_shards+1 int64, shard_off[0] = 0, non-decreasing,
 *                shard_off[n_shards] = n (else HORA_ERR_RANGE in dev_status).  Empty
 *                shards are allowed.
 * shard_budget : device, n_shards int64, each >= 0, at most (shard size) * HORA_MAX_DEPTH, and at
 *                most (shard size) * delta_max with a cap; a positive budget needs a non-empty
 *                shard (else HORA_ERR_RANGE / HORA_ERR_INFEASIBLE / HORA_ERR_UNSUPPORTED in
 *                dev_status; the outputs of such a shard are unspecified).
 * group_off    : as for hora_allocate; with HORA_I32 a total n*g0 + sum of the budgets of
 *                2^31 or more gives HORA_ERR_RANGE in dev_status (HORA_ERR_INVALID_ARG
 *                where n*g0 alone shows it).
 * summary      : device out, n_shards entries.  Nullable.
 * workspace    : device, >= hora_allocate_sharded_workspace_bytes(n_shards).
 * The other arguments are those of hora_allocate.  One workgroup works on one shard:
 * meant for many small or medium shards; a single large batch belongs to hora_allocate.
 */
int hora_allocate_sharded(int64_t n, int32_t g0, const int32_t *c, double alpha0, double beta0,
                          int64_t n_shards, const int64_t *shard_off, const int64_t *shard_budget,
                          int32_t delta_max, int32_t *delta, double *util, void *group_off,
                          int32_t off_t, hora_alloc_summary *summary, int32_t *dev_status,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Group-relative advantages over variable-size groups (Sec. 3.1 for GRPO; Sec. 4
 * "compatible with GRPO-family objectives" and App. E for RLOO).
 *
 * Group g holds responses group_off[g] .. group_off[g+1]-1 (G_g of them).
 *   GRPO: adv_j = (R_j - mean) / (std + eps), mean and std over the group's rewards,
 *         std with divisor G_g - ddof.  A group whose rewards are all equal (zero
 *         empirical std) gets exactly 0, as does a group with G_g - ddof <= 0.
 *   RLOO: adv_j = R_j - (S - R_j) / (G_g - 1), S the group's reward sum; G_g = 1 gives 0, and so
 *         does a group whose rewards are all equal (every response equals its leave-one-out
 *         baseline; the product with the reciprocal of G_g - 1 would leave 1e-16 there).
 *   CENTER: adv_j = R_j - mean, the GRPO form without the division by the standard
 *         deviation (for objectives of the Dr. GRPO kind; the paper's runs use GRPO as
 *         written in Sec. 3.1).  A group whose rewards are all equal gets exactly 0.
 * Evaluated in binary64 (partial sums per lane, then combined); a quotient whose divisor
 * is the same for the whole group (G_g, G_g - 1, std + eps) is formed as a product with the
 * divisor's reciprocal (itself the rounded quotient 1 / divisor for normal numbers), and the
 * last step of GRPO is one fused multiply-add: a few units in the last place of binary64
 * away from the expression as written.  The result is rounded once when stored as float.
 *
 * group_off : device, n_groups+1 offsets of type off_t, group_off[0] = 0, non-decreasing
 *             (else HORA_ERR_RANGE in dev_status).
 * reward, adv : device, n_resp values of type ft (HORA_F32 or HORA_F64); n_resp must
 *             equal group_off[n_groups] (else HORA_ERR_RANGE in dev_status).
 * eps >= 0; ddof is 0 or 1 (both used by GRPO only).
 */
int hora_group_advantage(int64_t n_groups, const void *group_off, int32_t off_t, int64_t n_resp,
                         const void *reward, void *adv, int32_t ft, int32_t mode, double eps,
                         int32_t ddof, int32_t *dev_status, void *stream);

/*
 * Per-response loss weights for variable-size groups (Sec. 3.1, objective: mean over the
 * tokens of a response, then over the responses of a prompt; Sec. 3.2 "Training objective
 * with variable-size groups": 1/G becomes 1/G_i so that every prompt weighs the same
 * however many additional rollouts it received):
 *   length_const <= 0 : weight[j] = 1 / (G_g * len_j),  len_j = tok_off[j+1] - tok_off[j]
 *   length_const  > 0 : weight[j] = 1 / (G_g * length_const), a constant in place of the
 *                       response length (length normalisation of the Dr. GRPO kind)
 * for every response j of group g; 0 for a response without tokens.  Evaluated in binary64
 * (one multiply, then one divide) and rounded once when stored as float.  Feeding the
 * result to hora_token_broadcast gives the weight of every token.
 *
 * group_off : device, n_groups+1 offsets (as for hora_group_advantage).
 * tok_off   : device, n_resp+1 packed token offsets, non-decreasing (else HORA_ERR_RANGE
 *             in dev_status).
 * weight    : device out, n_resp values of type ft.
 */
int hora_response_weights(int64_t n_groups, const void *group_off, int32_t group_off_t, int64_t n_resp,
                          const void *tok_off, int32_t tok_off_t, double length_const, void *weight,
                          int32_t ft, int32_t *dev_status, void *stream);

/*
 * Bytes of workspace hora_token_broadcast needs for n_tokens tokens of type out_t
 * (per 8 KiB of output one short descriptor of 32 bytes for float, 64 for double output,
 * and room for a wide one of 64 / 128 bytes).  Device memory, 256-byte aligned, no
 * initialisation needed; two calls that may run concurrently need separate workspaces.
 */
size_t hora_token_broadcast_workspace_bytes(int64_t n_tokens, int32_t out_t);

/*
 * Per-token advantages (Sec. 3.1: the advantage in the objective carries a token
 * index but does not depend on it): tok_adv[t] = adv[j] for tok_off[j] <= t < tok_off[j+1].
 *
 * adv      : device, n_resp values of type adv_t (n_resp < 2^31).
 * tok_off  : device, n_resp+1 packed token offsets of type off_t, tok_off[0] = 0,
 *            non-decreasing, tok_off[n_resp] = n_tokens (else HORA_ERR_RANGE in
 *            dev_status).  Zero-length responses are allowed.
 * tok_adv  : device out, n_tokens values of type out_t (a binary64 advantage stored as
 *            float is rounded to nearest once).  Must be aligned to its element size;
 *            any such alignment runs at full speed.
 * workspace: device, >= hora_token_broadcast_workspace_bytes(n_tokens, out_t).
 */
int hora_token_broadcast(int64_t n_resp, const void *adv, int32_t adv_t, const void *tok_off,
                         int32_t off_t, void *tok_adv, int32_t out_t, int64_t n_tokens,
                         int32_t *dev_status, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Two per-token streams over the same packed offsets in one pass (Sec. 3.1 objective and
 * Sec. 3.2 "Training objective with variable-size groups": besides its advantage, every token
 * carries a loss weight that is constant over the response, e.g. the 1/(G_i |o_j|) of
 * hora_response_weights; or the advantages of two estimators, GRPO and RLOO, side by side):
 *   tok_a[t] = adv_a[j],  tok_b[t] = adv_b[j]   for tok_off[j] <= t < tok_off[j+1].
 * Results equal two calls of hora_token_broadcast; the offsets are checked and the row
 * descriptors are built once for both outputs, in one launch pair instead of two.
 *
 * adv_a, adv_b : device, n_resp values of type adv_t each.
 * tok_a, tok_b : device out, n_tokens values of type out_t each; both must have the same
 *                address modulo 16 (else HORA_ERR_INVALID_ARG: they share one row grid).
 * workspace    : device, >= hora_token_broadcast2_workspace_bytes(n_tokens, out_t), which is
 *                twice what the one-stream call needs.
 * The other arguments and the errors are those of hora_token_broadcast.
 */
size_t hora_token_broadcast2_workspace_bytes(int64_t n_tokens, int32_t out_t);
int hora_token_broadcast2(int64_t n_resp, const void *adv_a, const void *adv_b, int32_t adv_t,
                          const void *tok_off, int32_t off_t, void *tok_a, void *tok_b, int32_t out_t,
                          int64_t n_tokens, int32_t *dev_status, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * Bytes of workspace hora_pass_at_k needs (device memory, 8-byte aligned, no
 * initialisation needed).  n_k <= 64.
 */
size_t hora_pass_at_k_workspace_bytes(int64_t n_problems, int32_t n_k);

/*
 * Unbiased Pass@K estimator (Sec. 4, Eq. 6).  Problem q has a pool of n_samples[q]
 * samples of which correct[q] are correct; for every K in ks
 *   per_problem[a * n_problems + q] = 1 - C(n_samples[q] - correct[q], ks[a]) / C(n_samples[q], ks[a])
 *   mean[a] = the average of that over the problems (the benchmark's Pass@K).
 * Evaluated in binary64 as a product of quotients (no binomial coefficient is formed).
 *
 * n_samples, correct : device, n_problems int32 each; 0 <= correct <= n_samples, and
 *                      1 <= K <= n_samples for every K (else HORA_ERR_RANGE in dev_status
 *                      and the value counts as 0).
 * ks          : HOST, n_k int32 (n_k <= 64), read before the call returns.
 * per_problem : device out, n_k * n_problems doubles.  Nullable.
 * mean        : device out, n_k doubles.
 */
int hora_pass_at_k(int64_t n_problems, const int32_t *n_samples, const int32_t *correct, int32_t n_k,
                   const int32_t *ks, double *per_problem, double *mean, int32_t *dev_status,
                   void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HORA_H */
