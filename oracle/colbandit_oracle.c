/*
 * Plain CPU oracle for the Col-Bandit query-time scoring path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or
 * import this file: it exists so that tests, the smoke check and the
 * benchmark's CPU-baseline leg have a slow, obviously correct statement of
 * what the method computes.  It shares no code with the HIP library.
 *
 * Everything is scalar C in double precision.  Inputs are float arrays that
 * already hold the storage-precision values (fp32, or bf16 values widened to
 * float), so the only rounding here is that of double arithmetic.
 *
 * What follows the paper:
 *   - MaxSim cell h(d,t) and score S(d;Q): Sec. 2.1, Eq. (1)-(2); matrix form
 *     H and row sum S_i: Sec. 3.1, Eq. (4)-(5).
 *   - exhaustive top-K: Sec. 2.1, Eq. (3).
 *   - hard bounds, Bernstein-Serfling radius, hybrid interval: Sec. 4.1,
 *     Eq. (7)-(8); empirical standard deviation, the n<=1 case, the
 *     finite-population correction rho_n and c=1: Appendix A.
 *   - batched progressive elimination, exact rescore of the survivors and
 *     final top-K: Sec. 4.2, Algorithm 1 and its detailed listing in
 *     Appendix "Detailed Algorithm Listing" with the walkthrough and the
 *     complexity paragraph (cells touched).
 *   - the two non-adaptive baselines, Doc-Uniform and Ball-carving: appendix
 *     "Compared Methods" and its two algorithm boxes.
 *
 * Readings taken where the paper is silent (each is listed in the design
 * notes of the repository):
 *   - log is the natural logarithm, c = 1, no O(1/n) term (Appendix A);
 *   - the N inside the logarithm is the size of the candidate set handed to
 *     the call and stays fixed over rounds;
 *   - a document survives a round iff UCB >= tau (non-strict);
 *   - the last batch holds the T mod B leftover tokens when B does not
 *     divide T;
 *   - every member of the final active set is rescored, however many;
 *   - final order is (score descending, document index ascending);
 *   - the reveal permutation comes from a SplitMix64-driven Fisher-Yates
 *     shuffle defined in oracle_permutation() below.  PARITY UNPINNED with
 *     respect to the authors' own generator: the paper fixes only that pi is
 *     a uniform permutation drawn with a fixed seed.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_EMPTY_DOC (-2)
#define ORACLE_ERR_NOMEM (-3)

/* ------------------------------------------------------------------ */
/* MaxSim cells and scores (Eq. (1)-(2), (4)-(5))                      */
/* ------------------------------------------------------------------ */

/* One cell: max over the document's tokens of <q_t, e_j>. */
double oracle_cell(const float *Q, int t, int d, const float *E,
                   const int64_t *off, int64_t i)
{
    const float *q = Q + (size_t)t * (size_t)d;
    double best = -INFINITY;
    for (int64_t j = off[i]; j < off[i + 1]; ++j) {
        const float *e = E + (size_t)j * (size_t)d;
        double dot = 0.0;
        for (int k = 0; k < d; ++k)
            dot += (double)q[k] * (double)e[k];
        if (dot > best)
            best = dot;
    }
    return best;
}

/* H[i*T+t] for all documents and query tokens. */
int oracle_maxsim_cells(const float *Q, int T, int d, const float *E,
                        const int64_t *off, int64_t N, double *H)
{
    if (!Q || !E || !off || !H || T < 1 || d < 1 || N < 0)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N; ++i) {
        if (off[i + 1] <= off[i])
            return ORACLE_ERR_EMPTY_DOC;
        for (int t = 0; t < T; ++t)
            H[(size_t)i * T + t] = oracle_cell(Q, t, d, E, off, i);
    }
    return ORACLE_OK;
}

/* S_i = sum_t H[i][t], t ascending. */
int oracle_row_sums(const double *H, int64_t N, int T, double *S)
{
    if (!H || !S || N < 0 || T < 1)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N; ++i) {
        double s = 0.0;
        for (int t = 0; t < T; ++t)
            s += H[(size_t)i * T + t];
        S[i] = s;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* exhaustive top-K (Eq. (3)): full sort by (score desc, id asc)       */
/* ------------------------------------------------------------------ */

typedef struct {
    double s;
    int64_t id;
} scored_t;

static int cmp_scored(const void *pa, const void *pb)
{
    const scored_t *a = (const scored_t *)pa, *b = (const scored_t *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

/* ids may be NULL (then candidate k has id k).  Writes min(K,n) entries. */
int oracle_topk(const double *S, const int64_t *ids, int64_t n, int K,
                int64_t *out_ids, double *out_scores)
{
    if (!S || !out_ids || n < 0 || K < 0)
        return ORACLE_ERR_ARG;
    scored_t *v = (scored_t *)malloc(sizeof(scored_t) * (size_t)(n > 0 ? n : 1));
    if (!v)
        return ORACLE_ERR_NOMEM;
    for (int64_t k = 0; k < n; ++k) {
        v[k].s = S[k];
        v[k].id = ids ? ids[k] : k;
    }
    qsort(v, (size_t)n, sizeof(scored_t), cmp_scored);
    int64_t m = K < n ? K : n;
    for (int64_t k = 0; k < m; ++k) {
        out_ids[k] = v[k].id;
        if (out_scores)
            out_scores[k] = v[k].s;
    }
    free(v);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* decision bounds (Sec. 4.1, Eq. (7)-(8); Appendix A)                 */
/* ------------------------------------------------------------------ */

/* Finite-population correction rho_n, piecewise in n <= T/2 (Appendix A). */
double oracle_rho(int n, int T)
{
    if (2 * n <= T)
        return 1.0 - (double)(n - 1) / (double)T;
    return (1.0 - (double)n / (double)T) * (1.0 + 1.0 / (double)n);
}

/* Effective radius, Eq. (7), with c = 1; +inf when n <= 1 (Appendix A). */
double oracle_radius(double alpha, int T, double sigma, int64_t N, double delta, int n)
{
    if (n <= 1)
        return INFINITY;
    double lg = log((double)N * (double)T / delta);
    return alpha * (double)T * sigma * sqrt(2.0 * lg / (double)n) * sqrt(oracle_rho(n, T));
}

/*
 * Interval of one document from its n revealed cell values (any order).
 * out[0]=LCB out[1]=UCB out[2]=mean out[3]=sigma_hat out[4]=radius
 * out[5]=LB_hard out[6]=UB_hard.  n == 0 gives the trivial [aT, bT].
 */
int oracle_bounds(const double *vals, int n, int T, double a, double b,
                  double alpha, double delta, int64_t N, double *out)
{
    if (!out || n < 0 || n > T || (n > 0 && !vals))
        return ORACLE_ERR_ARG;
    double sum = 0.0;
    for (int k = 0; k < n; ++k)
        sum += vals[k];
    double lbh = sum + (double)(T - n) * a;
    double ubh = sum + (double)(T - n) * b;
    if (n == 0) {
        out[0] = a * T; out[1] = b * T; out[2] = 0.0; out[3] = 0.0;
        out[4] = INFINITY; out[5] = lbh; out[6] = ubh;
        return ORACLE_OK;
    }
    double mu = sum / (double)n;
    double sigma = 0.0;
    if (n > 1) {
        double ss = 0.0;
        for (int k = 0; k < n; ++k) {
            double dv = vals[k] - mu;
            ss += dv * dv;
        }
        sigma = sqrt(ss / (double)(n - 1));
    }
    double r = oracle_radius(alpha, T, sigma, N, delta, n);
    /* n = T: the row is fully observed, the estimator IS the sum (Appendix A: the
     * radius collapses entirely); taking it from the sum keeps rounding of
     * T*(sum/T) from opening a one-ulp gap between LCB and UCB. */
    double shat = (n == T) ? sum : (double)T * mu;
    double lcb = shat - r, ucb = shat + r;
    if (lbh > lcb) lcb = lbh;      /* max(LB_hard, S_hat - r) */
    if (ubh < ucb) ucb = ubh;      /* min(UB_hard, S_hat + r) */
    out[0] = lcb; out[1] = ucb; out[2] = mu; out[3] = sigma;
    out[4] = r; out[5] = lbh; out[6] = ubh;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* reveal permutation                                                  */
/* ------------------------------------------------------------------ */

/* SplitMix64 step (Steele, Lea, Flood 2014; public-domain reference). */
uint64_t oracle_splitmix64_next(uint64_t *state)
{
    *state += 0x9E3779B97F4A7C15ULL;
    uint64_t z = *state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/*
 * Per-query permutation of [0,T): the generator state starts at
 * seed + (query_index + 1) * 0x9E3779B97F4A7C15 (mod 2^64); then a
 * Fisher-Yates shuffle walks i = T-1 .. 1 with j = next() mod (i+1).
 */
int oracle_permutation(uint64_t seed, int64_t query_index, int T, int32_t *pi)
{
    if (!pi || T < 1)
        return ORACLE_ERR_ARG;
    uint64_t st = seed + ((uint64_t)query_index + 1ULL) * 0x9E3779B97F4A7C15ULL;
    for (int t = 0; t < T; ++t)
        pi[t] = t;
    for (int i = T - 1; i >= 1; --i) {
        uint64_t j = oracle_splitmix64_next(&st) % (uint64_t)(i + 1);
        int32_t tmp = pi[i];
        pi[i] = pi[j];
        pi[j] = tmp;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Algorithm 1 (detailed listing)                                      */
/* ------------------------------------------------------------------ */

typedef struct {
    /* cell source: either a dense H (N x T) or the embeddings themselves */
    const double *H;
    const float *Q;
    const float *E;
    const int64_t *off;
    int T, d;
    /* exact cells for the rescore when H holds coarse (quantised) estimates;
       NULL: the rescore reads the same source as the reveals */
    const double *H_exact;
} cell_source_t;

static double reveal(const cell_source_t *src, int64_t i, int t)
{
    if (src->H)
        return src->H[(size_t)i * src->T + t];
    return oracle_cell(src->Q, t, src->d, src->E, src->off, i);
}

static double exact_cell(const cell_source_t *src, int64_t i, int t)
{
    if (src->H_exact)
        return src->H_exact[(size_t)i * src->T + t];
    return reveal(src, i, t);
}

static int cmp_desc(const void *pa, const void *pb)
{
    double a = *(const double *)pa, b = *(const double *)pb;
    return (a > b) ? -1 : (a < b) ? 1 : 0;
}

/*
 * The elimination loop, the rescore and the final top-K for one query.
 *
 * Outputs (any trace pointer may be NULL):
 *   out_ids/out_scores [K]        estimated top-K, exact scores
 *   final_ids [N], *n_final       final active set, index ascending
 *   counts [Rmax+1]               |A_r| entering round r (counts[0]=N), then
 *                                 the size after the last executed round
 *   tau [Rmax]                    threshold of each executed round
 *   tr_lcb, tr_ucb [Rmax x N]     interval of every document that was active
 *                                 in the round (NaN for the others)
 *   tr_alive [Rmax x N]           1 if the document is in A_{r+1}
 *   cells [3]                     cells_elim, cells_rescore, cells_unique
 * Rmax = ceil(T/B).  Returns the number of executed rounds (>= 0) or a
 * negative error.
 *
 * Resuming (A0 != NULL): the loop is entered at round r0 >= 1 with the active
 * set A0[0..nA0) (document indices, strictly ascending) instead of round 1
 * with all N documents.  Every member of A0 then already has the
 * (r0-1)*B cells pi[0 .. (r0-1)B) revealed, exactly as after r0-1 rounds of
 * an uninterrupted run (the shared reveal order makes that state a function
 * of the active set alone).  N inside the radius stays the candidate count
 * of the call.  counts[r0-1] = nA0; entries of counts, tau and the trace
 * below round r0 are left as initialised; cells_elim counts the resumed
 * rounds only.  The return value is still the index of the last executed
 * round (r0-1 if none ran).
 */
static int colbandit_core(const cell_source_t *src, int64_t N, int K, int M, int B,
                          double alpha, double delta, double a, double b,
                          const int32_t *pi,
                          const int64_t *A0, int64_t nA0, int r0,
                          int64_t *out_ids, double *out_scores,
                          int64_t *final_ids, int64_t *n_final,
                          int64_t *counts, double *tau,
                          double *tr_lcb, double *tr_ucb, uint8_t *tr_alive,
                          int64_t *cells)
{
    const int T = src->T;
    if (N < 1 || K < 1 || K > N || M < 0 || B < 1 || !pi || !(alpha > 0.0) ||
        !(delta > 0.0) || !(delta < 1.0) || !(a < b))
        return ORACLE_ERR_ARG;
    const int Rmax = (T + B - 1) / B;
    if (A0) {
        if (r0 < 1 || r0 > Rmax + 1 || nA0 < 1 || nA0 > N)
            return ORACLE_ERR_ARG;
        for (int64_t x = 0; x < nA0; ++x)
            if (A0[x] < 0 || A0[x] >= N || (x > 0 && A0[x] <= A0[x - 1]))
                return ORACLE_ERR_ARG;
    }

    int64_t *A = (int64_t *)malloc(sizeof(int64_t) * (size_t)N);      /* active set   */
    double *vals = (double *)malloc(sizeof(double) * (size_t)N * T);  /* revealed     */
    double *lcb = (double *)malloc(sizeof(double) * (size_t)N);
    double *ucb = (double *)malloc(sizeof(double) * (size_t)N);
    double *srt = (double *)malloc(sizeof(double) * (size_t)N);
    double *S = (double *)malloc(sizeof(double) * (size_t)N);
    if (!A || !vals || !lcb || !ucb || !srt || !S) {
        free(A); free(vals); free(lcb); free(ucb); free(srt); free(S);
        return ORACLE_ERR_NOMEM;
    }
    int64_t nA = N;
    for (int64_t i = 0; i < N; ++i) {
        A[i] = i;
        lcb[i] = a * T;     /* trivial initial interval */
        ucb[i] = b * T;
    }
    if (tr_lcb)
        for (size_t x = 0; x < (size_t)Rmax * N; ++x) tr_lcb[x] = NAN;
    if (tr_ucb)
        for (size_t x = 0; x < (size_t)Rmax * N; ++x) tr_ucb[x] = NAN;
    if (tr_alive)
        memset(tr_alive, 0, (size_t)Rmax * N);

    int n = 0;              /* revealed cells per active document (same for all) */
    int r = 1;
    int64_t cells_elim = 0;
    if (A0) {
        /* the state after r0-1 rounds: active set A0, first (r0-1)B cells of pi revealed */
        nA = nA0;
        r = r0;
        n = (r0 - 1) * B < T ? (r0 - 1) * B : T;
        for (int64_t x = 0; x < nA; ++x) {
            A[x] = A0[x];
            for (int p = 0; p < n; ++p)
                vals[(size_t)A0[x] * T + p] = reveal(src, A0[x], pi[p]);
        }
        if (counts) counts[r0 - 1] = nA0;
    } else if (counts) {
        counts[0] = N;
    }

    while (nA > (int64_t)K + M && (r - 1) * B < T) {
        int lo = (r - 1) * B;
        int hi = r * B < T ? r * B : T;            /* batch pi[lo..hi) */
        for (int64_t x = 0; x < nA; ++x) {
            int64_t i = A[x];
            for (int p = lo; p < hi; ++p)
                vals[(size_t)i * T + p] = reveal(src, i, pi[p]);
        }
        cells_elim += (int64_t)(hi - lo) * nA;
        n = hi;
        for (int64_t x = 0; x < nA; ++x) {
            int64_t i = A[x];
            double o[7];
            oracle_bounds(vals + (size_t)i * T, n, T, a, b, alpha, delta, N, o);
            lcb[i] = o[0];
            ucb[i] = o[1];
            srt[x] = o[0];
            if (tr_lcb) tr_lcb[(size_t)(r - 1) * N + i] = o[0];
            if (tr_ucb) tr_ucb[(size_t)(r - 1) * N + i] = o[1];
        }
        qsort(srt, (size_t)nA, sizeof(double), cmp_desc);
        double th = srt[K - 1];                     /* K-th largest LCB */
        if (tau) tau[r - 1] = th;
        int64_t m = 0;
        for (int64_t x = 0; x < nA; ++x) {
            int64_t i = A[x];
            if (ucb[i] >= th) {
                A[m++] = i;
                if (tr_alive) tr_alive[(size_t)(r - 1) * N + i] = 1;
            }
        }
        nA = m;
        if (counts) counts[r] = nA;
        ++r;
    }
    const int rounds = r - 1;

    /* exact rescore of every survivor on all T tokens */
    for (int64_t x = 0; x < nA; ++x) {
        int64_t i = A[x];
        double s = 0.0;
        for (int t = 0; t < T; ++t)
            s += exact_cell(src, i, t);
        S[x] = s;
    }
    int rc = oracle_topk(S, A, nA, K, out_ids, out_scores);

    if (final_ids)
        for (int64_t x = 0; x < nA; ++x) final_ids[x] = A[x];
    if (n_final) *n_final = nA;
    if (cells) {
        cells[0] = cells_elim;
        cells[1] = (int64_t)T * nA;
        cells[2] = cells_elim + (int64_t)(T - n) * nA;
    }
    free(A); free(vals); free(lcb); free(ucb); free(srt); free(S);
    return rc < 0 ? rc : rounds;
}

/* Col-Bandit over a given dense MaxSim matrix H (N x T). */
int oracle_colbandit_from_H(const double *H, int64_t N, int T, int K, int M, int B,
                            double alpha, double delta, double a, double b,
                            const int32_t *pi,
                            int64_t *out_ids, double *out_scores,
                            int64_t *final_ids, int64_t *n_final,
                            int64_t *counts, double *tau,
                            double *tr_lcb, double *tr_ucb, uint8_t *tr_alive,
                            int64_t *cells)
{
    if (!H || T < 1)
        return ORACLE_ERR_ARG;
    cell_source_t src = {H, NULL, NULL, NULL, T, 0, NULL};
    return colbandit_core(&src, N, K, M, B, alpha, delta, a, b, pi, NULL, 0, 1, out_ids,
                          out_scores, final_ids, n_final, counts, tau, tr_lcb, tr_ucb, tr_alive,
                          cells);
}

/*
 * The same loop entered at round r0 with the active set A0 (see colbandit_core): what
 * Algorithm 1 does from the state "A_{r0} = A0, (r0-1)B cells of the shared order revealed".
 * H_exact may be NULL (then the rescore reads H, as in oracle_colbandit_from_H).
 */
int oracle_colbandit_resume(const double *H, const double *H_exact, int64_t N, int T, int K,
                            int M, int B, double alpha, double delta, double a, double b,
                            const int32_t *pi, const int64_t *A0, int64_t nA0, int r0,
                            int64_t *out_ids, double *out_scores,
                            int64_t *final_ids, int64_t *n_final,
                            int64_t *counts, double *tau,
                            double *tr_lcb, double *tr_ucb, uint8_t *tr_alive,
                            int64_t *cells)
{
    if (!H || !A0 || T < 1)
        return ORACLE_ERR_ARG;
    cell_source_t src = {H, NULL, NULL, NULL, T, 0, H_exact};
    return colbandit_core(&src, N, K, M, B, alpha, delta, a, b, pi, A0, nA0, r0, out_ids,
                          out_scores, final_ids, n_final, counts, tau, tr_lcb, tr_ucb, tr_alive,
                          cells);
}

/*
 * Col-Bandit whose elimination loop sees coarse cells H_coarse while the survivors are
 * rescored from the exact cells H_exact (implementation appendix, "Cache-separated
 * quantized layout": decisions on the int8 estimates, exact rescore of the survivors).
 */
int oracle_colbandit_coarse(const double *H_coarse, const double *H_exact, int64_t N, int T,
                            int K, int M, int B, double alpha, double delta, double a,
                            double b, const int32_t *pi,
                            int64_t *out_ids, double *out_scores,
                            int64_t *final_ids, int64_t *n_final,
                            int64_t *counts, double *tau,
                            double *tr_lcb, double *tr_ucb, uint8_t *tr_alive,
                            int64_t *cells)
{
    if (!H_coarse || !H_exact || T < 1)
        return ORACLE_ERR_ARG;
    cell_source_t src = {H_coarse, NULL, NULL, NULL, T, 0, H_exact};
    return colbandit_core(&src, N, K, M, B, alpha, delta, a, b, pi, NULL, 0, 1, out_ids,
                          out_scores, final_ids, n_final, counts, tau, tr_lcb, tr_ucb, tr_alive,
                          cells);
}

/* ------------------------------------------------------------------ */
/* int8 coarse pass (implementation appendix, paragraph on the         */
/* quantized layout: magnitudes clipped at the 999th permille, the     */
/* clipped range coded linearly in 8 bits)                             */
/* ------------------------------------------------------------------ */

static int cmp_float_asc(const void *pa, const void *pb)
{
    float a = *(const float *)pa, b = *(const float *)pb;
    return (a < b) ? -1 : (a > b) ? 1 : 0;
}

/*
 * Clip value: the nearest-rank percentile of |x| -- the smallest v such that at
 * least permille/1000 of the n values satisfy |x| <= v, i.e. the element of rank
 * ceil(n * permille / 1000) (1-based) of the ascending sort.  Readings: the
 * paper does not say which percentile definition or which population; here the
 * population is whatever array is handed in (the whole corpus matrix, or one
 * query's T x d matrix) and the definition is nearest-rank, which needs no
 * interpolation and is therefore reproducible bit for bit.
 */
int oracle_abs_percentile(const float *x, int64_t n, int permille, float *clip)
{
    if (!x || !clip || n < 1 || permille < 1 || permille > 1000)
        return ORACLE_ERR_ARG;
    float *v = (float *)malloc(sizeof(float) * (size_t)n);
    if (!v)
        return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < n; ++i)
        v[i] = fabsf(x[i]);
    qsort(v, (size_t)n, sizeof(float), cmp_float_asc);
    /* ceil(n * permille / 1000) in integers; n * 1000 fits int64 for any array in memory */
    int64_t rank = (n * (int64_t)permille + 999) / 1000;
    if (rank < 1) rank = 1;
    *clip = v[rank - 1];
    free(v);
    return ORACLE_OK;
}

/*
 * Linear quantisation to int8 after clipping at +-clip: code = round-half-even(x * (127/clip))
 * saturated to [-127, 127]; the decoded value is code * (clip/127).  A floating-point value
 * decides an integer here, so the arithmetic is fixed: 127/clip and the product are single
 * precision operations (the precision of the kernels), rounding is to nearest even.
 * clip == 0 (an all-zero array) gives all-zero codes.
 */
int oracle_quantize_i8(const float *x, int64_t n, float clip, int8_t *out)
{
    if (!x || !out || n < 0 || !(clip >= 0.0f))
        return ORACLE_ERR_ARG;
    volatile float inv = clip > 0.0f ? 127.0f / clip : 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        volatile float y = x[i] * inv;       /* one single-precision rounding */
        float r = rintf(y);                  /* default mode: to nearest, ties to even */
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        out[i] = (int8_t)r;
    }
    return ORACLE_OK;
}

/*
 * Coarse MaxSim matrix from int8 codes: H[i][t] = sq * sd * max_j sum_k Q8[t][k] * D8[j][k],
 * the integer dot products exact, sq and sd the two decode scales (clip/127).
 * Also returns the integer maxima if Hint is non-NULL.
 */
int oracle_maxsim_cells_i8(const int8_t *Q8, float sq, int T, int d, const int8_t *D8, float sd,
                           const int64_t *off, int64_t N, double *H, int32_t *Hint)
{
    if (!Q8 || !D8 || !off || !H || T < 1 || d < 1 || N < 0)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N; ++i) {
        if (off[i + 1] <= off[i])
            return ORACLE_ERR_EMPTY_DOC;
        for (int t = 0; t < T; ++t) {
            int64_t best = 0;
            for (int64_t j = off[i]; j < off[i + 1]; ++j) {
                int64_t acc = 0;
                for (int k = 0; k < d; ++k)
                    acc += (int64_t)Q8[(size_t)t * d + k] * (int64_t)D8[(size_t)j * d + k];
                if (j == off[i] || acc > best)
                    best = acc;
            }
            H[(size_t)i * T + t] = (double)best * (double)sq * (double)sd;
            if (Hint)
                Hint[(size_t)i * T + t] = (int32_t)best;
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* non-adaptive baselines (appendix "Compared Methods")                 */
/* ------------------------------------------------------------------ */

/*
 * Doc-Uniform, the static random reveal (appendix "Compared Methods", Doc-Uniform paragraph
 * and its algorithm box): every document gets its own uniformly drawn subset R_i of m query
 * tokens, without replacement, and is ranked by the sum of those m cells.
 *
 * The subset of (query q, document i) as a bit mask over [0,T).  Readings (the paper fixes
 * only "uniformly, without replacement"): the draw is Floyd's subset sampling -- for
 * j = T-m .. T-1 take t = floor(next() * (j+1) / 2^64), a uniform index in [0, j], and insert
 * t, or j if t is already in -- fed by a SplitMix64 stream of its own per (q, i): one SplitMix64 step from the query's state
 * seed + (q+1)*0x9E3779B97F4A7C15 gives a query key, and the stream of document i starts at
 * state key + (i+1)*0xD1B54A32D192ED03.  PARITY UNPINNED with respect to the authors'
 * generator, as for the reveal permutation.
 */
/*
 * Budget of Doc-Uniform: "ceil(gamma T) cells per row" (first line of its algorithm box).
 * gamma is a decimal knob; the smallest integer m with m >= gamma*T is searched upwards, and a
 * product that exceeds an integer by less than 1e-9 (binary representation of the decimal)
 * counts as that integer.  Clamped to [1, T].  Negative on bad arguments.
 */
int oracle_cells_per_doc(double gamma, int T)
{
    if (T < 1 || !(gamma > 0.0) || !(gamma <= 1.0))
        return ORACLE_ERR_ARG;
    const double want = gamma * (double)T;
    for (int m = 1; m < T; ++m)
        if ((double)m + 1e-9 >= want)
            return m;
    return T;
}

uint64_t oracle_uniform_subset(uint64_t seed, int64_t q, int64_t i, int T, int m)
{
    if (T < 1 || T > 64 || m < 0 || m > T)
        return 0;
    uint64_t qs = seed + ((uint64_t)q + 1ULL) * 0x9E3779B97F4A7C15ULL;
    uint64_t key = oracle_splitmix64_next(&qs);
    uint64_t st = key + ((uint64_t)i + 1ULL) * 0xD1B54A32D192ED03ULL;
    uint64_t mask = 0;
    for (int j = T - m; j < T; ++j) {
        unsigned __int128 wide = (unsigned __int128)oracle_splitmix64_next(&st) * (uint64_t)(j + 1);
        int t = (int)(uint64_t)(wide >> 64);
        if ((mask >> t) & 1ULL)
            mask |= 1ULL << j;
        else
            mask |= 1ULL << t;
    }
    return mask;
}

/*
 * Doc-Uniform scores of one query over a given MaxSim matrix H (N x T):
 * S~_i = sum over t in R_i of H[i][t], t ascending; then the top-K by (S~ desc, id asc).
 * masks [N] and S [N] may be NULL; out_ids/out_scores may be NULL when K == 0.
 */
int oracle_doc_uniform_from_H(const double *H, int64_t N, int T, int m, uint64_t seed,
                              int64_t query_index, int K, uint64_t *masks, double *S,
                              int64_t *out_ids, double *out_scores)
{
    if (!H || N < 1 || T < 1 || T > 64 || m < 1 || m > T || K < 0 || K > N)
        return ORACLE_ERR_ARG;
    double *Sq = S ? S : (double *)malloc(sizeof(double) * (size_t)N);
    if (!Sq)
        return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < N; ++i) {
        uint64_t R = oracle_uniform_subset(seed, query_index, i, T, m);
        double s = 0.0;
        for (int t = 0; t < T; ++t)
            if ((R >> t) & 1ULL)
                s += H[(size_t)i * T + t];
        Sq[i] = s;
        if (masks)
            masks[i] = R;
    }
    if (K > 0 && out_ids)
        oracle_topk(Sq, NULL, N, K, out_ids, out_scores);
    if (!S)
        free(Sq);
    return ORACLE_OK;
}

/* Nearest-even rounding of a float to the bf16 grid (result widened back to float). */
float oracle_round_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) != 0x7F800000u) {          /* finite */
        u += 0x7FFFu + ((u >> 16) & 1u);
        u &= 0xFFFF0000u;
    }
    float y;
    memcpy(&y, &u, 4);
    return y;
}

/*
 * Ball-carving, step 1 (appendix "Compared Methods", Ball-carving paragraph and its algorithm
 * box): greedy clustering of the T query tokens.  The smallest remaining index is the pivot;
 * its cluster takes every remaining token whose cosine with the pivot is >= tau; the cluster
 * is replaced by the SUM of its (unnormalised) members; repeat until no token remains.
 *
 * labels [T]: cluster index of each token, clusters numbered in pivot order.
 * C [T x d]: row c holds centroid c for c < k, zeros beyond.  Returns k (>= 1) or an error.
 *
 * Readings:
 *   - a floating-point value decides a set here, so the test is fixed: with dot, |p|^2, |i|^2
 *     plain double sums over k ascending, token i joins pivot p iff dot > 0 and
 *     dot*dot >= ((tau*tau) * |p|^2) * |i|^2 in double -- the inequality cos >= tau (tau > 0)
 *     freed of the square root and the division;
 *   - the pivot always belongs to its own cluster, whatever rounding makes of its own cosine;
 *   - a centroid is accumulated in single precision, members in ascending index, and, when
 *     the embeddings are stored as bf16 (round_bf16 != 0), rounded to nearest-even bf16,
 *     because the scoring kernel takes query rows in the storage type.
 */
int oracle_ball_carving_clusters(const float *Q, int T, int d, float tau, int round_bf16,
                                 int32_t *labels, float *C)
{
    if (!Q || !labels || !C || T < 1 || d < 1 || !(tau > 0.0f) || !(tau <= 1.0f))
        return ORACLE_ERR_ARG;
    double *nn = (double *)malloc(sizeof(double) * (size_t)T);
    if (!nn)
        return ORACLE_ERR_NOMEM;
    for (int t = 0; t < T; ++t) {
        double s = 0.0;
        for (int k = 0; k < d; ++k)
            s += (double)Q[(size_t)t * d + k] * (double)Q[(size_t)t * d + k];
        nn[t] = s;
        labels[t] = -1;
    }
    memset(C, 0, sizeof(float) * (size_t)T * (size_t)d);
    const double tau2 = (double)tau * (double)tau;
    int k = 0;
    for (int p = 0; p < T; ++p) {
        if (labels[p] >= 0)
            continue;                       /* p is the smallest remaining index: the pivot */
        for (int i = p; i < T; ++i) {
            if (labels[i] >= 0)
                continue;
            int in = (i == p);
            if (!in) {
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += (double)Q[(size_t)p * d + c] * (double)Q[(size_t)i * d + c];
                in = dot > 0.0 && dot * dot >= (tau2 * nn[p]) * nn[i];
            }
            if (in) {
                labels[i] = k;
                for (int c = 0; c < d; ++c) {
                    volatile float acc = C[(size_t)k * d + c] + Q[(size_t)i * d + c];
                    C[(size_t)k * d + c] = acc;
                }
            }
        }
        if (round_bf16)
            for (int c = 0; c < d; ++c)
                C[(size_t)k * d + c] = oracle_round_bf16(C[(size_t)k * d + c]);
        ++k;
    }
    free(nn);
    return k;
}

/*
 * Ball-carving, step 2: Score(doc) = sum over the k centroids of max_j <c, e_j>, then the
 * top-K by (score desc, id asc).  S [N] may be NULL.  Returns k or an error.
 */
int oracle_ball_carving(const float *Q, int T, int d, float tau, int round_bf16, const float *E,
                        const int64_t *off, int64_t N, int K, int32_t *labels, float *C,
                        double *S, int64_t *out_ids, double *out_scores)
{
    if (!E || !off || N < 1 || K < 0 || K > N)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N; ++i)
        if (off[i + 1] <= off[i])
            return ORACLE_ERR_EMPTY_DOC;
    int k = oracle_ball_carving_clusters(Q, T, d, tau, round_bf16, labels, C);
    if (k < 0)
        return k;
    double *Sq = S ? S : (double *)malloc(sizeof(double) * (size_t)N);
    if (!Sq)
        return ORACLE_ERR_NOMEM;
    for (int64_t i = 0; i < N; ++i) {
        double s = 0.0;
        for (int c = 0; c < k; ++c)
            s += oracle_cell(C, c, d, E, off, i);
        Sq[i] = s;
    }
    if (K > 0 && out_ids)
        oracle_topk(Sq, NULL, N, K, out_ids, out_scores);
    if (!S)
        free(Sq);
    return k;
}

/* Col-Bandit that computes each revealed cell from the embeddings. */
int oracle_colbandit_lazy(const float *Q, int T, int d, const float *E,
                          const int64_t *off, int64_t N, int K, int M, int B,
                          double alpha, double delta, double a, double b,
                          const int32_t *pi,
                          int64_t *out_ids, double *out_scores,
                          int64_t *final_ids, int64_t *n_final,
                          int64_t *counts, double *tau, int64_t *cells)
{
    if (!Q || !E || !off || T < 1 || d < 1)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N; ++i)
        if (off[i + 1] <= off[i])
            return ORACLE_ERR_EMPTY_DOC;
    cell_source_t src = {NULL, Q, E, off, T, d, NULL};
    return colbandit_core(&src, N, K, M, B, alpha, delta, a, b, pi, NULL, 0, 1, out_ids,
                          out_scores, final_ids, n_final, counts, tau, NULL, NULL, NULL, cells);
}

/* ------------------------------------------------------------------ */
/* query batches: one thread per query, as in the paper's threading    */
/* model (Appendix "Multi-threading model")                            */
/* ------------------------------------------------------------------ */

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Exhaustive scores + top-K for nq queries.  S [nq x N] may be NULL. */
int oracle_full_batch(const float *Q, int nq, int T, int d, const float *E,
                      const int64_t *off, int64_t N, int K,
                      double *S, int64_t *out_ids, double *out_scores)
{
    if (!Q || !E || !off || nq < 1 || T < 1 || d < 1 || N < 1 || K < 0 || K > N)
        return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < N; ++i)
        if (off[i + 1] <= off[i])
            return ORACLE_ERR_EMPTY_DOC;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        const float *Qq = Q + (size_t)q * T * d;
        double *Sq = S ? S + (size_t)q * N : (double *)malloc(sizeof(double) * (size_t)N);
        if (!Sq) { err = ORACLE_ERR_NOMEM; continue; }
        for (int64_t i = 0; i < N; ++i) {
            double s = 0.0;
            for (int t = 0; t < T; ++t)
                s += oracle_cell(Qq, t, d, E, off, i);
            Sq[i] = s;
        }
        if (K > 0 && out_ids)
            oracle_topk(Sq, NULL, N, K, out_ids + (size_t)q * K,
                        out_scores ? out_scores + (size_t)q * K : NULL);
        if (!S) free(Sq);
    }
    return err;
}

/* Col-Bandit (lazy reveals) for nq queries; pi is [nq x T].  cells [nq x 3],
 * rounds [nq] may be NULL. */
int oracle_colbandit_batch(const float *Q, int nq, int T, int d, const float *E,
                           const int64_t *off, int64_t N, int K, int M, int B,
                           double alpha, double delta, double a, double b,
                           const int32_t *pi, int64_t *out_ids, double *out_scores,
                           int64_t *cells, int32_t *rounds)
{
    if (!Q || !E || !off || !pi || !out_ids || nq < 1)
        return ORACLE_ERR_ARG;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < nq; ++q) {
        int rc = oracle_colbandit_lazy(Q + (size_t)q * T * d, T, d, E, off, N, K, M, B,
                                       alpha, delta, a, b, pi + (size_t)q * T,
                                       out_ids + (size_t)q * K,
                                       out_scores ? out_scores + (size_t)q * K : NULL,
                                       NULL, NULL, NULL, NULL,
                                       cells ? cells + (size_t)q * 3 : NULL);
        if (rc < 0) err = rc;
        else if (rounds) rounds[q] = rc;
    }
    return err;
}
