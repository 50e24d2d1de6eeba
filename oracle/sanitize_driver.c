/*
 * TEST INFRASTRUCTURE -- driver for a sanitizer build of the test oracle.
 *
 * Built together with hora_oracle.c under -fsanitize=address,undefined (gcc) by
 * tests/test_oracle_sanitizers.py.  It runs every oracle function on small seeded inputs,
 * including the empty and degenerate cases, with every buffer allocated at its exact size
 * on the heap (so that an access one element too far is an error), and prints the results
 * as text; the test compares them with what the ordinary build of the oracle returns for
 * the same inputs.  The inputs come from a 64-bit linear congruential generator that the
 * test repeats in Python.
 */
#include <inttypes.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void hora_oracle_marginal_gains(double alpha, double beta, int64_t count, double *out);
double hora_oracle_hit_utility(double alpha, double beta, int64_t delta);
int hora_oracle_posterior(int64_t n, int32_t g0, const int32_t *c, double alpha0, double beta0, double *alpha,
                          double *beta);
int hora_oracle_allocate_scan(int64_t n, const double *alpha, const double *beta, int64_t budget, int64_t delta_max,
                              int64_t *delta);
int hora_oracle_allocate(int64_t n, const double *alpha, const double *beta, int64_t budget, int64_t delta_max,
                         int64_t *delta);
int hora_oracle_allocate_sharded(int64_t n, const double *alpha, const double *beta, int64_t n_shards,
                                 const int64_t *shard_off, const int64_t *shard_budget, int64_t delta_max,
                                 int64_t *delta);
void hora_oracle_group_offsets(int64_t n, int32_t g0, const int64_t *delta, int64_t *off);
int hora_oracle_group_advantage(int64_t n_groups, const int64_t *off, const double *reward, double *adv, int32_t mode,
                                double eps, int32_t ddof);
int hora_oracle_token_broadcast(int64_t n_resp, const double *adv, const int64_t *tok_off, double *tok_adv);
int hora_oracle_response_weights(int64_t n_groups, const int64_t *group_off, const int64_t *tok_off,
                                 double length_const, double *weight);
int hora_oracle_allocate_baseline(int64_t n, const int32_t *c, int64_t budget, int64_t delta_max, int32_t rule,
                                  int64_t *delta);

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint32_t next_u32(void) {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}

static void *exact(size_t count, size_t size) {   /* exactly count elements; one byte for count == 0 */
    void *p = malloc(count * size ? count * size : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    return p;
}

static void print_doubles(const char *tag, const double *x, int64_t n) {
    printf("%s", tag);
    for (int64_t i = 0; i < n; ++i) printf(" %a", x[i]);
    printf("\n");
}
static void print_ints(const char *tag, const int64_t *x, int64_t n) {
    printf("%s", tag);
    for (int64_t i = 0; i < n; ++i) printf(" %" PRId64, x[i]);
    printf("\n");
}

static void one_case(int64_t n, int32_t g0, int64_t budget, int64_t cap, double alpha0, double beta0) {
    int32_t *c = exact((size_t)n, sizeof *c);
    for (int64_t i = 0; i < n; ++i) c[i] = (int32_t)(next_u32() % (uint32_t)(g0 + 1));
    double *alpha = exact((size_t)n, sizeof *alpha), *beta = exact((size_t)n, sizeof *beta);
    int rc = hora_oracle_posterior(n, g0, c, alpha0, beta0, alpha, beta);
    printf("case n=%" PRId64 " g0=%d budget=%" PRId64 " cap=%" PRId64 " rc=%d\n", n, g0, budget, cap, rc);
    int64_t *delta = exact((size_t)n, sizeof *delta), *delta2 = exact((size_t)n, sizeof *delta2);
    rc = hora_oracle_allocate(n, alpha, beta, budget, cap, delta);
    int rc2 = hora_oracle_allocate_scan(n, alpha, beta, budget, cap, delta2);
    printf("allocate rc=%d scan rc=%d\n", rc, rc2);
    if (rc == 0) {
        print_ints("delta", delta, n);
        print_ints("delta_scan", delta2, n);
        double *u = exact((size_t)n, sizeof *u);
        for (int64_t i = 0; i < n; ++i) u[i] = hora_oracle_hit_utility(alpha[i], beta[i], delta[i]);
        print_doubles("util", u, n);
        free(u);
        /* two shards, the first of n/3 prompts */
        int64_t shard_off[3] = {0, n / 3, n};
        int64_t first = 0;
        for (int64_t i = 0; i < n / 3; ++i) first += delta[i];
        int64_t shard_budget[2] = {first, budget - first};
        rc = hora_oracle_allocate_sharded(n, alpha, beta, 2, shard_off, shard_budget, cap, delta2);
        printf("sharded rc=%d\n", rc);
        if (rc == 0) print_ints("delta_sharded", delta2, n);
        for (int rule = 0; rule < 2; ++rule) {
            rc = hora_oracle_allocate_baseline(n, c, budget, cap, rule, delta2);
            printf("baseline rule=%d rc=%d\n", rule, rc);
            if (rc == 0) print_ints("delta_rule", delta2, n);
        }
        /* groups, rewards, advantages, tokens */
        int64_t *goff = exact((size_t)n + 1, sizeof *goff);
        hora_oracle_group_offsets(n, g0, delta, goff);
        print_ints("group_off", goff, n + 1);
        int64_t r = goff[n];
        double *reward = exact((size_t)r, sizeof *reward), *adv = exact((size_t)r, sizeof *adv);
        for (int64_t j = 0; j < r; ++j) reward[j] = (double)(next_u32() % 3u) * 0.5;
        int64_t *toff = exact((size_t)r + 1, sizeof *toff);
        toff[0] = 0;
        for (int64_t j = 0; j < r; ++j) toff[j + 1] = toff[j] + (int64_t)(next_u32() % 5u);
        for (int mode = 0; mode < 3; ++mode) {
            for (int64_t j = 0; j < r; ++j) adv[j] = 0.0;
            rc = hora_oracle_group_advantage(n, goff, reward, adv, mode, mode == 0 ? 1e-6 : 0.0, 0);
            printf("advantage mode=%d rc=%d\n", mode, rc);
            print_doubles("adv", adv, r);
        }
        double *tok = exact((size_t)toff[r], sizeof *tok);
        rc = hora_oracle_token_broadcast(r, adv, toff, tok);
        printf("broadcast rc=%d\n", rc);
        print_doubles("tok", tok, toff[r]);
        double *w = exact((size_t)r, sizeof *w);
        for (int k = 0; k < 2; ++k) {
            rc = hora_oracle_response_weights(n, goff, toff, k ? 2048.0 : 0.0, w);
            printf("weights rc=%d\n", rc);
            print_doubles("w", w, r);
        }
        free(w); free(tok); free(toff); free(adv); free(reward); free(goff);
    }
    free(delta2); free(delta); free(beta); free(alpha); free(c);
}

int main(void) {
    double *g = exact(40, sizeof *g);
    hora_oracle_marginal_gains(0.75, 3.25, 40, g);
    print_doubles("gains", g, 40);
    hora_oracle_marginal_gains(2.0, 2.0, 0, g);   /* nothing to write */
    free(g);
    one_case(0, 4, 0, 0, 1.0, 1.0);
    one_case(1, 4, 0, 0, 1.0, 1.0);
    one_case(1, 4, 9, 0, 1.0, 1.0);
    one_case(7, 2, 30, 0, 0.5, 3.0);
    one_case(12, 8, 40, 4, 2.0, 3.25);
    one_case(12, 8, 48, 4, 1.0, 1.0);    /* every prompt at the cap */
    one_case(5, 4, 21, 4, 1.0, 1.0);     /* infeasible */
    one_case(33, 16, 100, 0, 1.0, 1.0);
    return 0;
}
