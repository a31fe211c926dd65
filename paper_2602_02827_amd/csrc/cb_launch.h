// Host-side launch interface between the C-ABI layer and the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cb_device.h"

namespace cb {

enum { DT_F32 = 0, DT_BF16 = 1 };

struct Problem {
    const void* Q;
    int nq, T, d, dt;
    const void* docs;
    const int64_t* off;
    int64_t N, total;
};

// Views into the caller's workspace (all device pointers).
struct Work {
    QueryCtl* ctl;        // [nq]
    int32_t* list[2];     // [nq][N] each: ids of the active set, ascending
    float2* stat;         // [nq][N] per (query, doc): revealed sum, centred sum of squares
    float2* stat2;        // [nq][N] batch (sum, centred squares) of a later round's dense pass
    unsigned long long* pairs;   // [R+2] pairs[r]: (query, doc) pairs round r would have to gather;
                                 // then [R+2]: the document tokens of those pairs
    int32_t* seg_cnt;     // [nq][64] candidates per segment of a segmented pre-filter
    float* rescored;      // [nq][N] exact score of the k-th survivor
    float* scores;        // [nq][N] Full-MaxSim scores when the caller keeps none
    int32_t* cnt_hist;    // [(R+1)][nq]
    float* tau_hist;      // [R][nq]
    int32_t* pi;          // [nq][T]
    int32_t* chunk_doc;   // [nchunks+1] first document of each token chunk (dense kernel)
    int* flag;            // [64] error / scratch flags
    // cell cache of queries whose active set has shrunk to <= cache_cap documents
    int cache_cap;        // slots per query (0: caching off)
    int TP;               // floats per slot: T rounded up to whole 16-column tiles
    int32_t* cid;         // [nq][cache_cap] document id of a slot
    float2* cstat;        // [nq][cache_cap] revealed sum / centred squares of a slot
    float* ccell;         // [nq][cache_cap][TP] the slot's MaxSim cells
    // coarse pass: int8 codes of the queries, written per call
    int8_t* q8;           // [nq][T][d]
    float* qscale;        // [nq]
    void* qscratch;       // quantize_scratch_bytes(nq)
};

// int8 codes for the coarse elimination pass (implementation appendix, quantized layout):
// a code c decodes to c * scale.  All device pointers.
struct Coarse {
    const int8_t* docs8;  // [total][d] codes of the document tokens
    const float* dscale;  // [1] their decode scale
    int8_t* Q8;           // [nq][T][d] codes of the queries (written by the call)
    float* qscale;        // [nq] decode scale of each query
};

struct Trace {            // all null when tracing is off
    int32_t* count;
    float* tau;
    float* lcb;
    float* ucb;
    uint8_t* alive;
};

struct RevealRound {
    int r;                // 1-based round
    int lo, nb;           // batch = pi[lo .. lo+nb)
    int n_prev, n;        // cells revealed before / after the round
    float kappa;          // radius per unit sigma_hat at n
    // Rounds >= 2 pick their reveal path on the device: the corpus-streaming pass if
    // pairs[r] > dense_thr, else the per-pair gather.  Every kernel of the round evaluates the
    // same test.  ~0: always gather (also round 1, whose path the host fixes).
    unsigned long long dense_thr;
};

struct Knobs {
    int K, M, B;
    float a, b;
};

hipError_t launch_init(const Problem& P, const Work& W, const Knobs& kn, int R, uint64_t seed,
                       const int32_t* user_pi, const Trace& tr, hipStream_t st);

// Reveal one batch for every active (query, doc) pair by gathering the documents.
hipError_t launch_gather_reveal(const Problem& P, const Work& W, const RevealRound& rr,
                                const Coarse* co, hipStream_t st);

// The reveal of round rr for queries that fit the cell cache: all T cells of every active
// document are computed once and cached; later rounds and the rescore read them back.
hipError_t launch_gather_cells(const Problem& P, const Work& W, const RevealRound& rr,
                               const Coarse* co, hipStream_t st);
hipError_t launch_cached_score(const Problem& P, const Work& W, float* out, hipStream_t st);

// Exact scores from the stored embeddings.  ctl == nullptr: all documents of every query,
// written by doc id into `out` ([nq][N]); otherwise the current active set, written by list
// position (score_slots: including the queries whose list holds cache slots, whose cached
// cells are coarse and cannot give the exact score).
hipError_t launch_gather_score(const Problem& P, const Work& W, bool use_ctl, float* out,
                               float* cells, bool score_slots, hipStream_t st);

// Dense (corpus-streaming) kernel for bf16: Full-MaxSim scores or the first reveal batch.
hipError_t launch_dense_prepare(const Problem& P, const Work& W, int chunk_tokens, int* n_chunks,
                                hipStream_t st);
// co != nullptr: the pass runs on the int8 codes (integer matrix instructions, exact int32
// maxima decoded by the two scales) instead of the stored embeddings.
hipError_t launch_dense_score(const Problem& P, const Work& W, int chunk_tokens, int n_chunks,
                              float* out, float* cells, const Coarse* co, hipStream_t st);
hipError_t launch_dense_reveal(const Problem& P, const Work& W, int chunk_tokens, int n_chunks,
                               const RevealRound& rr, int G, const Coarse* co, hipStream_t st);
// The same pass for a round >= 2: runs only if the round's device-side test picks it, writes the
// batch statistics of every (active ids-mode query, document) to stat2; k_select_prune merges
// them into the running statistics of the documents still active.
hipError_t launch_dense_reveal_later(const Problem& P, const Work& W, int chunk_tokens,
                                     int n_chunks, const RevealRound& rr, int G, const Coarse* co,
                                     hipStream_t st);
bool dense_supported(const Problem& P, const Coarse* co);

// R: number of rounds of the call (layout of W.pairs).
hipError_t launch_select_prune(const Problem& P, const Work& W, const Knobs& kn,
                               const RevealRound& rr, int R, const Trace& tr, hipStream_t st);

// Top-K of `vals` per query.  use_ctl: candidates are the active set (vals indexed by
// list position); else all N documents (vals indexed by id).
hipError_t launch_topk(const Problem& P, const Work& W, bool use_ctl, const float* vals, int K,
                       int64_t* out_ids, float* out_scores, hipStream_t st);

// int8 codes of x ([n_segments][seg_elems] values of dtype dt): per segment, clip = the
// nearest-rank permille/1000 percentile of |x|, code = rint(x * 127 / clip) saturated to
// +-127, scales[seg] = clip / 127.  scratch: quantize_scratch_bytes(n_segments).
size_t quantize_scratch_bytes(int64_t n_segments);
hipError_t launch_quantize_i8(const void* x, int dt, int64_t n_segments, int64_t seg_elems,
                              int permille, int8_t* codes, float* scales, void* scratch,
                              hipStream_t st);

// Doc-Uniform (appendix "Compared Methods"): scores[q][i] = sum of cells[q][i][t] over the
// seeded random subset of m tokens of (q, i); masks (nullable) receives the subsets.
hipError_t launch_uniform_score(const float* cells, int nq, int64_t N, int T, int m, uint64_t seed,
                                float* scores, uint64_t* masks, hipStream_t st);
// Ball-carving (same appendix): greedy clustering of each query's tokens at cosine threshold
// tau.  Cz [nq][T][d] (storage type): centroid c of query q in row c, zero rows past the last;
// labels [nq][T] (nullable): cluster of each token; kq [nq]: clusters per query.
hipError_t launch_ball_carve(const Problem& P, float tau, void* Cz, int32_t* labels, int32_t* kq,
                             hipStream_t st);
// bf16: packs the centroids four to a group.  goff [nq+1]: first group of each query and the
// total; Qg [total groups][4][d]; ident [total groups][4] = 0,1,2,3.
hipError_t launch_ball_groups(const Problem& P, const void* Cz, const int32_t* kq, int32_t* goff,
                              void* Qg, int32_t* ident, hipStream_t st);
// scores[q][i] = sum over the groups of q, ascending, of part[(g * N + i) * stride].
hipError_t launch_ball_reduce(const float* part, int stride, const int32_t* goff, int nq, int64_t N,
                              float* scores, hipStream_t st);

hipError_t launch_validate_offsets(const int64_t* off, int64_t N, int64_t total, int* flag,
                                   hipStream_t st);

}  // namespace cb
