/*
 * colbandit.h - C-ABI of the MI355X-native Col-Bandit scoring library.
 *
 * Two scoring paths over one packed, ragged corpus of token embeddings:
 *
 *   colbandit_full_maxsim  exhaustive late-interaction scoring.  Cell (i,t) of the
 *                          MaxSim matrix is max_j <q_t, e_{i,j}> (paper Eq. (1)/(4)),
 *                          a document's score is the row sum (Eq. (2)/(5)), and the
 *                          result is the top-K of the scores (Eq. (3)).
 *   colbandit_topk         the Col-Bandit estimator of that top-K (Sec. 4, Algorithm 1
 *                          and its detailed listing in the implementation appendix):
 *                          batched cell reveals in a seeded order shared by all
 *                          documents of a query, per-document Bernstein-Serfling
 *                          intervals (Eq. (7)-(8), Appendix A), elimination of every
 *                          document whose UCB is below the K-th largest LCB, exact
 *                          rescoring of the survivors and a final top-K.
 *
 * Conventions common to all entry points
 *   - Pointers documented as DEVICE point to memory of the current HIP device, owned
 *     by the caller; the library never frees or keeps them.  HOST pointers are plain
 *     process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     kernels are enqueued on it.  Unless stated otherwise a call returns after
 *     enqueueing; outputs are valid once the caller has synchronised the stream.
 *   - Return value: COLBANDIT_OK (0) or a negative COLBANDIT_ERR_* code.  On an
 *     argument error nothing is enqueued and no output is written.
 *   - Layout: Q is [n_queries][T][d] row-major; doc_tokens is [total_tokens][d]
 *     row-major with document i owning rows doc_offsets[i] .. doc_offsets[i+1]-1;
 *     both in the storage type `dt`.  Q and doc_tokens must be 16-byte aligned.
 *   - Preconditions the host cannot check without a copy: doc_offsets is
 *     non-decreasing, doc_offsets[0] >= 0, doc_offsets[N] <= total_tokens and every
 *     document has at least one token.  Kernels clamp row indices into
 *     [0,total_tokens), so a violation gives meaningless scores, never an
 *     out-of-bounds access; colbandit_validate_offsets checks them on the device.
 */
#ifndef COLBANDIT_H
#define COLBANDIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { COLBANDIT_F32 = 0, COLBANDIT_BF16 = 1 } colbandit_dtype;

enum {
    COLBANDIT_OK = 0,
    COLBANDIT_ERR_NULL = -1,         /* a required pointer is NULL                    */
    COLBANDIT_ERR_SHAPE = -2,        /* n_queries, T, d, N, total_tokens or K invalid */
    COLBANDIT_ERR_KNOB = -3,         /* alpha_ef, delta, M, B or [a,b] out of range   */
    COLBANDIT_ERR_UNSUPPORTED = -4,  /* valid request outside what the kernels cover  */
    COLBANDIT_ERR_WORKSPACE = -5,    /* workspace or trace buffer too small           */
    COLBANDIT_ERR_ALIGNMENT = -6,    /* Q / doc_tokens / workspace misaligned         */
    COLBANDIT_ERR_HIP = -7,          /* a HIP runtime call failed                     */
    COLBANDIT_ERR_BAD_OFFSETS = -8,  /* colbandit_validate_offsets found a violation  */
    COLBANDIT_ERR_TOO_LARGE = -9     /* colbandit_topk_static: the sizes need more scratch
                                        than the library's built-in buffer holds       */
};

/* Limits of this build (requests beyond them return COLBANDIT_ERR_UNSUPPORTED).
 * Embedding width d: 32, 64, 96 or 128.  The corpus-streaming kernels and the int8 codes
 * cover 64 and 128; at 32 and 96 every pass runs on the per-pair gather kernels (same
 * results, lower throughput) and opts.docs_i8 / colbandit_coarse_maxsim are refused.
 * Query tokens T: up to COLBANDIT_MAX_T for bf16, up to 64 for fp32. */
#define COLBANDIT_MAX_T 128          /* query tokens                                  */
#define COLBANDIT_MAX_K 1024         /* size of the returned top-K                    */
#define COLBANDIT_MAX_B 16           /* cells revealed per document per round         */
#define COLBANDIT_MAX_ROUNDS 64      /* ceil(T/B)                                     */

/*
 * Optional knobs of colbandit_topk.  A zero-initialised struct selects the paper's
 * deployed defaults (implementation appendix, "Default parameter setting").
 */
typedef struct {
    int B;              /* round size; 0 -> 4 (Sec. 4.2)                               */
    float a, b;         /* support [a,b] of a cell; a == b == 0 -> [-1,1] (Sec. 4.1)   */
    const int32_t *pi;  /* DEVICE [n_queries][T] reveal orders, each a permutation of
                           0..T-1; NULL -> drawn on the device from `seed`, see
                           colbandit_permutation                                        */
    void *trace;        /* DEVICE buffer of colbandit_trace_bytes() bytes or NULL;
                           test aid, layout below                                       */
    size_t trace_bytes;
    int force_gather;   /* nonzero: reveal round 1 with the gather kernel as well
                           (test aid; the default picks the dense kernel for bf16)      */
    int no_cell_cache;  /* nonzero: re-gather the documents in every round instead of
                           caching a small active set's cells at its first gather
                           (test aid; the decisions are the same either way)            */
    const int8_t *docs_i8;    /* DEVICE [total_tokens][d] int8 codes of doc_tokens, or NULL.
                                 When given, the elimination rounds run on int8 codes
                                 (implementation appendix, "Cache-separated quantized
                                 layout"): every revealed cell is the exact integer
                                 maximum of <code(q_t), code(e_j)> times the two decode
                                 scales; the queries are coded by the call itself (per
                                 query, same scheme).  The survivors are still rescored
                                 from doc_tokens, so topk_scores keep the exact bits.
                                 Make the codes with colbandit_quantize_i8.            */
    const float *docs_scale;  /* DEVICE [1]: decode scale of docs_i8 (required with it)  */
    int coarse_permille;      /* percentile, in 1/1000, of |Q| at which a query is clipped
                                 before coding; 0 -> 999 (the paper's 99.9th)            */
    int later_rounds;   /* reveal path of rounds >= 2 for bf16 inputs.  0: chosen on the
                           device each round - one corpus-streaming pass shared by all
                           queries when the active sets are so large that gathering
                           every (query, document) pair would move more bytes, else the
                           per-pair gather; 1: the streaming pass in every such round;
                           2: always the gather.  The decisions are the same either way */
} colbandit_opts;

/*
 * Per-query statistics, HOST memory (Sec. 3.1 coverage; implementation appendix,
 * "Complexity": cells touched = sum_r |B_r||A_r| + T|A_final|).
 */
typedef struct {
    int32_t rounds;                                   /* elimination rounds executed   */
    int32_t survivors[COLBANDIT_MAX_ROUNDS + 2];      /* |A_1| = N, then |A_{r+1}|
                                                         after each executed round     */
    int64_t cells_elim;                               /* sum_r |B_r| |A_r|             */
    int64_t cells_rescore;                            /* T |A_final|                   */
    int64_t cells_unique;                             /* |Omega| with set semantics    */
    float ms_total;                                   /* device time of the whole call
                                                         (all queries of the batch)    */
    float ms_first_reveal;                            /* of which: reveal of round 1   */
    float ms_later_reveals;                           /* reveals of rounds >= 2        */
    float ms_select_prune;                            /* thresholds and pruning        */
    float ms_rescore_topk;                            /* rescore and final top-K
                                                         (cf. the paper's stage split in
                                                         its overhead-breakdown table)  */
    float ms_reveal_round2;                           /* of ms_later_reveals: the reveal
                                                         launches of round 2 alone          */
    uint64_t corpus_pass_rounds;                      /* bit r-1 set: the batch revealed
                                                         round r (r >= 2) by one pass over
                                                         the corpus instead of per-pair
                                                         gathers (same for all queries)  */
    int64_t cells_computed;                           /* cells the kernels COMPUTED for this
                                                         query, which can exceed the cells
                                                         revealed to the bounds: a corpus
                                                         pass computes a round's batch for
                                                         all N documents, the first gathered
                                                         round of a list that fits the cell
                                                         cache computes all T cells of its
                                                         documents once (later rounds and
                                                         the rescore then compute none)   */
    uint64_t pairs_round2;                            /* (query, document) pairs of the whole
                                                         batch that entered round 2 still
                                                         held as document ids, and           */
    uint64_t tokens_round2;                           /* the document tokens of those pairs:
                                                         what a gathered round 2 has to
                                                         read (same for all queries)       */
} colbandit_stats;

/* sizeof(colbandit_opts) / sizeof(colbandit_stats) as this library was compiled: lets a
 * binding written in another language check its own struct definitions. */
size_t colbandit_sizeof_opts(void);
size_t colbandit_sizeof_stats(void);

/*
 * Trace buffer layout (R = ceil(T/B) rounds, nq = n_queries), in this order:
 *   int32   count[(R+1)][nq]     |A| entering round r+1 (count[0] = N)
 *   float   tau[R][nq]           threshold of each executed round (NaN if not run)
 *   float   lcb[R][nq][N]        interval of every document active in the round,
 *   float   ucb[R][nq][N]        NaN elsewhere
 *   uint8   alive[R][nq][N]      1 iff the document is in the next active set
 */
size_t colbandit_trace_bytes(int n_queries, int T, int B, int64_t N);

/* Scratch the two scoring calls need for these sizes (bytes; 0 on invalid sizes). */
size_t colbandit_workspace_bytes(int n_queries, int T, int d, int64_t N,
                                 int64_t total_tokens, int K, int M);

/*
 * int8 codes for the coarse elimination pass (implementation appendix, paragraph on the
 * quantized layout: magnitudes are clipped at a high percentile, 999 per mille, and the
 * clipped range is coded linearly in 8 bits).  The input is n_segments consecutive matrices of
 * rows_per_segment x d values; each segment gets its own clip value: the nearest-rank
 * percentile of |x|, i.e. the element of rank ceil(n * permille / 1000) of the ascending
 * order of the segment's n = rows_per_segment * d absolute values (exact, no
 * interpolation).  code = round-half-even(x * (127 / clip)) saturated to [-127, 127],
 * evaluated in single precision; scales[s] = clip / 127 decodes segment s.  An all-zero
 * segment gives zero codes and scale 0.
 *   x          DEVICE, dtype dt, 16-byte aligned
 *   permille   1..1000 (999 = the paper's 99.9th percentile)
 *   codes      DEVICE int8, same shape as x
 *   scales     DEVICE float [n_segments]
 *   workspace  DEVICE, 256-byte aligned, >= colbandit_quantize_workspace_bytes(n_segments)
 * A corpus is one segment (n_segments = 1, rows_per_segment = total_tokens): an
 * index-time step.  Fully asynchronous.
 */
size_t colbandit_quantize_workspace_bytes(int64_t n_segments);
int colbandit_quantize_i8(const void *x, colbandit_dtype dt, int64_t n_segments,
                          int64_t rows_per_segment, int d, int permille, int8_t *codes,
                          float *scales, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * Exhaustive MaxSim on the int8 codes: the coarse cell matrix the elimination rounds of
 * colbandit_topk see when opts->docs_i8 is given (and a fast approximate scorer).  The
 * queries are coded by the call (per query, clip at `permille`).
 *   scores     DEVICE float [n_queries][N]: row sums of the coarse cells
 *   cells      DEVICE float [n_queries][N][T] or NULL
 *   q_codes    DEVICE int8 [n_queries][T][d] or NULL: receives the query codes
 *   q_scales   DEVICE float [n_queries] or NULL: receives their decode scales
 * Other arguments as for colbandit_full_maxsim (Q and dt are the uncoded queries).
 */
int colbandit_coarse_maxsim(const void *Q, int n_queries, int T, int d, colbandit_dtype dt,
                            const int8_t *docs_i8, const float *docs_scale,
                            const int64_t *doc_offsets, int64_t N, int64_t total_tokens,
                            int permille, float *scores, float *cells, int8_t *q_codes,
                            float *q_scales, void *workspace, size_t workspace_bytes,
                            void *stream);

/*
 * Exhaustive Full-MaxSim (Eq. (1)-(3)).
 *   Q, doc_tokens, doc_offsets   DEVICE, see layout above; doc_offsets is int64 [N+1]
 *   K                            0 -> scores only; else 1 <= K <= min(N, MAX_K)
 *   scores                       DEVICE float [n_queries][N], fp32 row sums; may be
 *                                NULL when K > 0 (then they live in the workspace)
 *   topk_ids, topk_scores        DEVICE int64 / float [n_queries][K], ordered by
 *                                (score descending, document index ascending);
 *                                required when K > 0
 *   cells                        DEVICE float [n_queries][N][T] or NULL: the MaxSim
 *                                matrix itself (test aid)
 *   phase_ms                     HOST float [2] or NULL.  When non-NULL the call
 *                                synchronises the stream before returning and writes
 *                                the device time of the scoring kernel alone
 *                                (phase_ms[0]) and of the top-K selection
 *                                (phase_ms[1]), in milliseconds, taken with events
 *                                on `stream`
 *   workspace                    DEVICE, 256-byte aligned, >= colbandit_workspace_bytes
 * bf16 inputs are multiplied on the matrix cores with fp32 accumulation; fp32 inputs
 * use fp32 matrix instructions.  Fully asynchronous unless phase_ms is given.
 */
int colbandit_full_maxsim(const void *Q, int n_queries, int T, int d, colbandit_dtype dt,
                          const void *doc_tokens, const int64_t *doc_offsets, int64_t N,
                          int64_t total_tokens, int K, float *scores, int64_t *topk_ids,
                          float *topk_scores, float *cells, float *phase_ms,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Col-Bandit top-K (Algorithm 1).
 *   K              1 <= K <= min(N, MAX_K)
 *   alpha_ef       relaxation of the radius, 0 < alpha_ef <= 1 (Eq. (7))
 *   delta          0 < delta < 1
 *   M              rescore margin, >= 0: the loop stops once |A| <= K + M
 *   seed           seed of the per-query reveal permutations (ignored if opts->pi)
 *   opts           HOST, may be NULL
 *   topk_ids       DEVICE int64 [n_queries][K]; entries beyond the number of
 *                  survivors (possible only if cells leave [a,b]) are -1
 *   topk_scores    DEVICE float [n_queries][K]: exact scores of the survivors,
 *                  computed by the same kernel arithmetic as colbandit_full_maxsim
 *                  (same bits); -inf where the id is -1
 *   stats          HOST [n_queries] or NULL.  When non-NULL the call synchronises
 *                  the stream before returning; otherwise it is fully asynchronous
 *                  (all round control stays on the device).
 * Queries are independent: each has its own permutation, active set and stopping
 * round; the batch only shares kernel launches.
 */
int colbandit_topk(const void *Q, int n_queries, int T, int d, colbandit_dtype dt,
                   const void *doc_tokens, const int64_t *doc_offsets, int64_t N,
                   int64_t total_tokens, int K, float alpha_ef, float delta, int M,
                   uint64_t seed, const colbandit_opts *opts, int64_t *topk_ids,
                   float *topk_scores, colbandit_stats *stats, void *workspace,
                   size_t workspace_bytes, void *stream);

/*
 * colbandit_topk for callers that cannot allocate device memory or hand over a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same computation, same kernels and same results (bit for bit) as
 * colbandit_topk with stats == NULL, but the scratch memory is a buffer of
 * COLBANDIT_STATIC_SCRATCH_BYTES that is part of the library's device image: every GPU the
 * library runs on holds one copy from the first use of the library on it until the process
 * ends.  The call allocates nothing (no hipMalloc / hipFree, no events, no host heap) and is
 * fully asynchronous; statistics are not available here.
 *   - Sizes whose colbandit_workspace_bytes() exceeds COLBANDIT_STATIC_SCRATCH_BYTES are
 *     rejected with COLBANDIT_ERR_TOO_LARGE before anything is enqueued.
 *   - The device that is current at the call is the one whose buffer is used (its address is
 *     looked up once per device, at the first call on it; make that first call outside a
 *     graph capture).  A failed lookup returns COLBANDIT_ERR_HIP.
 *   - All calls on one GPU share that GPU's buffer.  A call does not rely on what an earlier
 *     call left there (every field it reads is written by its own kernels first), but two
 *     calls that overlap in time on one GPU - different streams, or replays of two captured
 *     graphs at once - race on it.  Calls on one stream are ordered and safe.
 *   - opts->trace, if given, is still the caller's own buffer.
 * Other arguments as for colbandit_topk.
 */
#define COLBANDIT_STATIC_SCRATCH_BYTES (64u << 20)
int colbandit_topk_static(const void *Q, int n_queries, int T, int d, colbandit_dtype dt,
                          const void *doc_tokens, const int64_t *doc_offsets, int64_t N,
                          int64_t total_tokens, int K, float alpha_ef, float delta, int M,
                          uint64_t seed, const colbandit_opts *opts, int64_t *topk_ids,
                          float *topk_scores, void *stream);

/*
 * Doc-Uniform, the paper's static random-reveal baseline (appendix "Compared Methods",
 * Doc-Uniform paragraph and its algorithm box): every (query, document) pair reveals its own
 * uniformly drawn subset of `cells_per_doc` = ceil(gamma * T) query tokens, without
 * replacement, and documents are ranked by the sum of the revealed cells.
 *   cells_per_doc   1 .. T (colbandit_cells_per_doc turns a coverage gamma into it; T <= 64)
 *   seed            the subset of (query q, document i) is Floyd's subset sampling -- for
 *                   j = T-m .. T-1: t = floor(next() * (j+1) / 2^64); insert t, or j if t is
 *                   in already -- on a SplitMix64 stream of its own: one SplitMix64 step from state
 *                   seed + (q+1) * 0x9E3779B97F4A7C15 gives the query's key, the stream of
 *                   document i starts at state key + (i+1) * 0xD1B54A32D192ED03
 *   scores          DEVICE float [n_queries][N]: partial row sums, cells added in ascending
 *                   token order in fp32; may be NULL when K > 0
 *   masks           DEVICE uint64 [n_queries][N] or NULL: bit t set = token t revealed
 *   K, topk_ids, topk_scores   as for colbandit_full_maxsim, ranking by the partial sums
 * Subsets that differ per document leave no query column for a matrix tile to share, so the
 * call computes the whole MaxSim matrix with the exhaustive kernel into the workspace
 * (4 * n_queries * N * T bytes on top of colbandit_workspace_bytes) and then sums each row
 * over its subset: on this machine the baseline costs a little more than Full-MaxSim whatever
 * gamma is.  Fully asynchronous.  Other arguments as for colbandit_full_maxsim.
 */
size_t colbandit_doc_uniform_workspace_bytes(int n_queries, int T, int d, int64_t N,
                                             int64_t total_tokens);
/*
 * Cells per document of Doc-Uniform at coverage gamma (first line of its algorithm box in the
 * appendix "Compared Methods": ceil(gamma * T) cells per row).  gamma is a decimal knob (the
 * paper sweeps 0.05, 0.10, ..., 1.00) whose nearest double can lie a hair above the decimal,
 * so a product within 1e-9 of an integer counts as that integer: 0.1 * 30 gives 3, not 4.
 * Returns ceil(gamma * T - 1e-9) clamped to [1, T], or COLBANDIT_ERR_KNOB unless
 * 0 < gamma <= 1, COLBANDIT_ERR_SHAPE unless T >= 1.  Pure host code.
 */
int colbandit_cells_per_doc(double gamma, int T);
int colbandit_doc_uniform(const void *Q, int n_queries, int T, int d, colbandit_dtype dt,
                          const void *doc_tokens, const int64_t *doc_offsets, int64_t N,
                          int64_t total_tokens, int K, int cells_per_doc, uint64_t seed,
                          float *scores, uint64_t *masks, int64_t *topk_ids,
                          float *topk_scores, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * Ball-carving, the paper's query-compression baseline (appendix "Compared Methods",
 * Ball-carving paragraph and its algorithm box).  Step 1, per query: the smallest remaining
 * token index is the pivot; its cluster takes every remaining token whose cosine with the
 * pivot is >= tau; the cluster is replaced by the sum of its (unnormalised) members; repeat
 * until no token remains (k clusters).  Step 2: Score(doc) = sum over the k centroids of
 * max_j <c, e_j>; documents are ranked by it.  Coverage in the paper's sense is k / T.
 *   tau          0 < tau <= 1; T <= 64
 *   membership   token i joins pivot p iff dot > 0 and dot*dot >= ((tau*tau)*|p|^2)*|i|^2,
 *                evaluated in double precision with sums over the components in ascending
 *                order (cos >= tau without a square root or a division, so that the outcome
 *                is reproducible bit for bit); the pivot always belongs to its own cluster
 *   centroid     single-precision sum of the members in ascending index, then stored in
 *                `dt` (bf16: round to nearest even) because the scoring kernels take query
 *                rows in the storage type
 *   n_clusters   DEVICE int32 [n_queries] or NULL: k of each query
 *   labels       DEVICE int32 [n_queries][T] or NULL: cluster of each token (pivot order)
 *   centroids    DEVICE `dt` [n_queries][T][d] or NULL: centroid c in row c, zero rows after
 *   scores       DEVICE float [n_queries][N]; may be NULL when K > 0
 *   K, topk_ids, topk_scores   as for colbandit_full_maxsim, ranking by Score
 * bf16: the centroids of the whole batch are packed four to a group and scored by the
 * corpus-streaming kernel, whose work follows the number of query columns, so the time
 * follows sum_q 4*ceil(k_q/4); the call synchronises the stream once (it reads the number
 * of groups back).  fp32: the zero-padded centroid matrix goes through the exhaustive
 * gather kernel (a zero row's cell is 0).  Workspace: colbandit_ball_carving_workspace_bytes
 * (for bf16 it holds 8 * n_queries * ceil(T/4) * N bytes of group sums).
 */
size_t colbandit_ball_carving_workspace_bytes(int n_queries, int T, int d, colbandit_dtype dt,
                                              int64_t N, int64_t total_tokens);
int colbandit_ball_carving(const void *Q, int n_queries, int T, int d, colbandit_dtype dt,
                           const void *doc_tokens, const int64_t *doc_offsets, int64_t N,
                           int64_t total_tokens, int K, float tau, int32_t *n_clusters,
                           int32_t *labels, void *centroids, float *scores,
                           int64_t *topk_ids, float *topk_scores, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * The reveal order used for query `query_index` under `seed` (Sec. 4.2: one uniform
 * permutation of [T] per query, fixed seed; the generator itself is this library's
 * choice): SplitMix64 started at seed + (query_index+1)*0x9E3779B97F4A7C15, then a
 * Fisher-Yates shuffle for i = T-1..1 with j = next() mod (i+1).  pi is HOST [T].
 * Pure host code.
 */
int colbandit_permutation(uint64_t seed, int64_t query_index, int T, int32_t *pi);

/*
 * Radius pre-factor per unit sigma_hat after n revealed cells (Eq. (7), c = 1,
 * natural log, rho_n of Appendix A): alpha_ef*T*sqrt(2 ln(N T/delta)/n)*sqrt(rho_n),
 * +inf for n <= 1.  Pure host code, double precision; the kernels receive its value
 * rounded to float.
 */
double colbandit_radius_prefactor(float alpha_ef, float delta, int T, int64_t N, int n);

/*
 * Checks the doc_offsets preconditions on the device, synchronises the stream and
 * returns COLBANDIT_OK or COLBANDIT_ERR_BAD_OFFSETS.  `workspace` needs 256 bytes.
 */
int colbandit_validate_offsets(const int64_t *doc_offsets, int64_t N, int64_t total_tokens,
                               void *workspace, size_t workspace_bytes, void *stream);

/* Static description of an error code. */
const char *colbandit_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* COLBANDIT_H */
