/*
 * Sanitizer driver for the CPU oracle (test infrastructure, like the oracle itself).
 *
 * tests/test_oracle_pins.py compiles this file together with colbandit_oracle.c under
 * -fsanitize=address,undefined and runs it: every entry point of the oracle is exercised on
 * small deterministic inputs with exactly sized buffers, so that any out-of-bounds access,
 * leak or undefined operation inside the oracle aborts the run.  A few cross-checks between
 * entry points (they must agree by the definitions of Sec. 2.1 / Algorithm 1) are asserted on
 * the way.  Exit status 0 = clean.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

double oracle_cell(const float *Q, int t, int d, const float *E, const int64_t *off, int64_t i);
int oracle_maxsim_cells(const float *Q, int T, int d, const float *E, const int64_t *off,
                        int64_t N, double *H);
int oracle_row_sums(const double *H, int64_t N, int T, double *S);
int oracle_topk(const double *S, const int64_t *ids, int64_t n, int K, int64_t *out_ids,
                double *out_scores);
double oracle_rho(int n, int T);
double oracle_radius(double alpha, int T, double sigma, int64_t N, double delta, int n);
int oracle_bounds(const double *vals, int n, int T, double a, double b, double alpha,
                  double delta, int64_t N, double *out);
uint64_t oracle_splitmix64_next(uint64_t *state);
int oracle_permutation(uint64_t seed, int64_t query_index, int T, int32_t *pi);
int oracle_colbandit_from_H(const double *H, int64_t N, int T, int K, int M, int B, double alpha,
                            double delta, double a, double b, const int32_t *pi,
                            int64_t *out_ids, double *out_scores, int64_t *final_ids,
                            int64_t *n_final, int64_t *counts, double *tau, double *tr_lcb,
                            double *tr_ucb, uint8_t *tr_alive, int64_t *cells);
int oracle_colbandit_resume(const double *H, const double *H_exact, int64_t N, int T, int K, int M,
                            int B, double alpha, double delta, double a, double b, const int32_t *pi,
                            const int64_t *A0, int64_t nA0, int r0, int64_t *out_ids,
                            double *out_scores, int64_t *final_ids, int64_t *n_final, int64_t *counts,
                            double *tau, double *tr_lcb, double *tr_ucb, uint8_t *tr_alive,
                            int64_t *cells);
int oracle_colbandit_coarse(const double *H_coarse, const double *H_exact, int64_t N, int T,
                            int K, int M, int B, double alpha, double delta, double a, double b,
                            const int32_t *pi, int64_t *out_ids, double *out_scores,
                            int64_t *final_ids, int64_t *n_final, int64_t *counts, double *tau,
                            double *tr_lcb, double *tr_ucb, uint8_t *tr_alive, int64_t *cells);
int oracle_abs_percentile(const float *x, int64_t n, int permille, float *clip);
int oracle_quantize_i8(const float *x, int64_t n, float clip, int8_t *out);
int oracle_maxsim_cells_i8(const int8_t *Q8, float sq, int T, int d, const int8_t *D8, float sd,
                           const int64_t *off, int64_t N, double *H, int32_t *Hint);
int oracle_colbandit_lazy(const float *Q, int T, int d, const float *E, const int64_t *off,
                          int64_t N, int K, int M, int B, double alpha, double delta, double a,
                          double b, const int32_t *pi, int64_t *out_ids, double *out_scores,
                          int64_t *final_ids, int64_t *n_final, int64_t *counts, double *tau,
                          int64_t *cells);
int oracle_num_threads(void);
uint64_t oracle_uniform_subset(uint64_t seed, int64_t q, int64_t i, int T, int m);
int oracle_doc_uniform_from_H(const double *H, int64_t N, int T, int m, uint64_t seed,
                              int64_t query_index, int K, uint64_t *masks, double *S,
                              int64_t *out_ids, double *out_scores);
float oracle_round_bf16(float x);
int oracle_ball_carving_clusters(const float *Q, int T, int d, float tau, int round_bf16,
                                 int32_t *labels, float *C);
int oracle_ball_carving(const float *Q, int T, int d, float tau, int round_bf16, const float *E,
                        const int64_t *off, int64_t N, int K, int32_t *labels, float *C,
                        double *S, int64_t *out_ids, double *out_scores);
int oracle_full_batch(const float *Q, int nq, int T, int d, const float *E, const int64_t *off,
                      int64_t N, int K, double *S, int64_t *out_ids, double *out_scores);
int oracle_colbandit_batch(const float *Q, int nq, int T, int d, const float *E,
                           const int64_t *off, int64_t N, int K, int M, int B, double alpha,
                           double delta, double a, double b, const int32_t *pi, int64_t *out_ids,
                           double *out_scores, int64_t *cells, int32_t *rounds);

#define CHECK(c)                                                              \
    do {                                                                      \
        if (!(c)) {                                                           \
            fprintf(stderr, "selftest: check failed at line %d: %s\n", __LINE__, #c); \
            exit(1);                                                          \
        }                                                                     \
    } while (0)

static uint64_t rng = 0x1234567ull;
static float unit_rand(void) /* in (-1, 1) */
{
    return (float)((double)(oracle_splitmix64_next(&rng) >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}

static void unit_rows(float *x, int rows, int d)
{
    for (int r = 0; r < rows; ++r) {
        double s = 0.0;
        for (int k = 0; k < d; ++k) {
            x[r * d + k] = unit_rand();
            s += (double)x[r * d + k] * x[r * d + k];
        }
        for (int k = 0; k < d; ++k) x[r * d + k] = (float)(x[r * d + k] / sqrt(s));
    }
}

int main(void)
{
    enum { NQ = 2, T = 7, D = 12, N = 37, K = 3, M = 2, B = 3 };
    const int Rmax = (T + B - 1) / B;
    int64_t off[N + 1];
    off[0] = 0;
    for (int i = 0; i < N; ++i) off[i + 1] = off[i] + 1 + (int64_t)(oracle_splitmix64_next(&rng) % 9);
    const int64_t total = off[N];
    float *Q = malloc(sizeof(float) * NQ * T * D);
    float *E = malloc(sizeof(float) * (size_t)total * D);
    CHECK(Q && E);
    unit_rows(Q, NQ * T, D);
    unit_rows(E, (int)total, D);

    /* definitions: cells, row sums, top-K */
    double *H = malloc(sizeof(double) * N * T);
    double *S = malloc(sizeof(double) * N);
    CHECK(H && S);
    CHECK(oracle_maxsim_cells(Q, T, D, E, off, N, H) == 0);
    CHECK(fabs(oracle_cell(Q, T - 1, D, E, off, N - 1) - H[(N - 1) * T + T - 1]) == 0.0);
    CHECK(oracle_row_sums(H, N, T, S) == 0);
    int64_t ids[K];
    double sc[K];
    CHECK(oracle_topk(S, NULL, N, K, ids, sc) >= 0);
    for (int k = 1; k < K; ++k) CHECK(sc[k - 1] >= sc[k]);

    /* closed forms */
    CHECK(oracle_rho(T, T) == 0.0 && oracle_rho(1, T) == 1.0);
    CHECK(oracle_radius(1.0, T, 0.3, N, 0.01, T) == 0.0);
    double o[7];
    CHECK(oracle_bounds(H, T, T, -1.0, 1.0, 0.2, 0.01, N, o) == 0);
    CHECK(o[0] == o[1]);                                /* all cells revealed: exact sum */
    CHECK(oracle_bounds(H, 1, T, -1.0, 1.0, 0.2, 0.01, N, o) == 0);
    CHECK(oracle_bounds(H, B, T, -1.0, 1.0, 0.2, 0.01, N, o) == 0 && o[0] <= o[1]);

    /* permutation */
    int32_t pi[NQ * T];
    for (int q = 0; q < NQ; ++q) {
        CHECK(oracle_permutation(99, q, T, pi + q * T) == 0);
        int seen = 0;
        for (int t = 0; t < T; ++t) seen |= 1 << pi[q * T + t];
        CHECK(seen == (1 << T) - 1);
    }

    /* Algorithm 1 over a matrix, with every trace buffer exactly sized */
    int64_t out_ids[K], final_ids[N], n_final = 0, counts[8], cells[3];
    double out_sc[K], tau[8];
    double *lcb = malloc(sizeof(double) * Rmax * N), *ucb = malloc(sizeof(double) * Rmax * N);
    uint8_t *alive = malloc((size_t)Rmax * N);
    CHECK(lcb && ucb && alive && Rmax + 1 <= 8);
    int r1 = oracle_colbandit_from_H(H, N, T, K, M, B, 0.2, 0.01, -1.0, 1.0, pi, out_ids, out_sc,
                                     final_ids, &n_final, counts, tau, lcb, ucb, alive, cells);
    CHECK(r1 >= 0 && r1 <= Rmax && n_final >= K && counts[0] == N);
    CHECK(cells[1] == (int64_t)T * n_final);
    /* the same, computing cells lazily from the embeddings: identical run */
    int64_t out_ids2[K], final2[N], n_final2 = 0, counts2[8], cells2[3];
    double out_sc2[K], tau2[8];
    int r2 = oracle_colbandit_lazy(Q, T, D, E, off, N, K, M, B, 0.2, 0.01, -1.0, 1.0, pi, out_ids2,
                                   out_sc2, final2, &n_final2, counts2, tau2, cells2);
    CHECK(r2 == r1 && n_final2 == n_final);
    for (int k = 0; k < K; ++k) CHECK(out_ids2[k] == out_ids[k]);
    /* re-entered at round 2 with the first round's survivors: the same final set and top-K */
    if (r1 >= 1) {
        int64_t A0[N], nA0 = 0;
        for (int i = 0; i < N; ++i)
            if (alive[i]) A0[nA0++] = i;
        CHECK(nA0 == counts[1]);
        int r5 = oracle_colbandit_resume(H, NULL, N, T, K, M, B, 0.2, 0.01, -1.0, 1.0, pi, A0, nA0, 2,
                                         out_ids2, out_sc2, final2, &n_final2, counts2, tau2, lcb,
                                         ucb, alive, cells2);
        CHECK(r5 == r1 && n_final2 == n_final);
        for (int k = 0; k < K; ++k) CHECK(out_ids2[k] == out_ids[k]);
    }
    /* alpha = 1 with every cell revealed (B = T, M = 0, K + M < N): the exhaustive top-K */
    int r3 = oracle_colbandit_from_H(H, N, T, K, 0, 1, 1.0, 0.01, -1.0, 1.0, pi, out_ids2, out_sc2,
                                     final2, &n_final2, NULL, NULL, NULL, NULL, NULL, cells2);
    CHECK(r3 >= 0);
    if (r3 == T)                                        /* loop ran to n = T: exact */
        for (int k = 0; k < K; ++k) CHECK(out_ids2[k] == ids[k]);

    /* int8 coarse pass */
    float cq = 0.f, cd = 0.f;
    CHECK(oracle_abs_percentile(Q, (int64_t)T * D, 999, &cq) == 0 && cq > 0.f);
    CHECK(oracle_abs_percentile(E, total * D, 999, &cd) == 0 && cd > 0.f);
    int8_t *Q8 = malloc((size_t)T * D), *D8 = malloc((size_t)total * D);
    CHECK(Q8 && D8);
    CHECK(oracle_quantize_i8(Q, (int64_t)T * D, cq, Q8) == 0);
    CHECK(oracle_quantize_i8(E, total * D, cd, D8) == 0);
    double *Hc = malloc(sizeof(double) * N * T);
    int32_t *Hi = malloc(sizeof(int32_t) * N * T);
    CHECK(Hc && Hi);
    CHECK(oracle_maxsim_cells_i8(Q8, cq / 127.0f, T, D, D8, cd / 127.0f, off, N, Hc, Hi) == 0);
    for (int x = 0; x < N * T; ++x) CHECK(fabs(Hc[x] - H[x]) < 0.2);
    int r4 = oracle_colbandit_coarse(Hc, H, N, T, K, M, B, 0.2, 0.01, -1.0, 1.0, pi, out_ids2, out_sc2,
                                     final2, &n_final2, counts2, tau2, lcb, ucb, alive, cells2);
    CHECK(r4 >= 0 && n_final2 >= K);
    for (int k = 0; k < K; ++k) CHECK(fabs(out_sc2[k] - S[out_ids2[k]]) < 1e-12);   /* exact rescore */

    /* the two non-adaptive baselines */
    uint64_t um[N];
    double us[N];
    CHECK(oracle_doc_uniform_from_H(H, N, T, T, 5, 1, K, um, us, out_ids2, out_sc2) == 0);
    for (int i = 0; i < N; ++i) CHECK(um[i] == (1u << T) - 1 && fabs(us[i] - S[i]) < 1e-12);
    for (int k = 0; k < K; ++k) CHECK(out_ids2[k] == ids[k]);      /* every cell: exhaustive */
    CHECK(oracle_doc_uniform_from_H(H, N, T, 3, 5, 1, K, um, NULL, out_ids2, out_sc2) == 0);
    for (int i = 0; i < N; ++i) CHECK(__builtin_popcountll(um[i]) == 3 && um[i] < (1u << T));
    CHECK(oracle_uniform_subset(5, 1, N - 1, T, 3) == um[N - 1]);
    CHECK(oracle_round_bf16(1.0f) == 1.0f && oracle_round_bf16(1.00390625f) == 1.0f);
    int32_t lab[T];
    float *C = malloc(sizeof(float) * T * D);
    CHECK(C);
    int kc = oracle_ball_carving(Q, T, D, 1.0f, 0, E, off, N, K, lab, C, us, out_ids2, out_sc2);
    CHECK(kc == T);                                     /* tau = 1: every token its own cluster */
    for (int i = 0; i < N; ++i) CHECK(fabs(us[i] - S[i]) < 1e-12);
    kc = oracle_ball_carving(Q, T, D, 0.05f, 1, E, off, N, K, lab, C, NULL, out_ids2, out_sc2);
    CHECK(kc >= 1 && kc <= T && lab[0] == 0);
    CHECK(oracle_ball_carving_clusters(Q, T, D, 0.5f, 0, lab, C) >= 1);
    free(C);

    /* batch entry points (OpenMP) */
    CHECK(oracle_num_threads() >= 1);
    double *Sb = malloc(sizeof(double) * NQ * N), bsc[NQ * K];
    int64_t bids[NQ * K], bcells[NQ * 3];
    int32_t brounds[NQ];
    CHECK(Sb);
    CHECK(oracle_full_batch(Q, NQ, T, D, E, off, N, K, Sb, bids, bsc) == 0);
    for (int i = 0; i < N; ++i) CHECK(Sb[i] == S[i]);
    CHECK(oracle_colbandit_batch(Q, NQ, T, D, E, off, N, K, M, B, 0.2, 0.01, -1.0, 1.0, pi, bids, bsc,
                                 bcells, brounds) == 0);
    CHECK(brounds[0] == r1);
    for (int k = 0; k < K; ++k) CHECK(bids[k] == out_ids[k]);

    free(Q); free(E); free(H); free(S); free(lcb); free(ucb); free(alive);
    free(Q8); free(D8); free(Hc); free(Hi); free(Sb);
    printf("oracle selftest ok\n");
    return 0;
}
