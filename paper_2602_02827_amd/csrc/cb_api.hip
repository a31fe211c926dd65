// C-ABI of the library: argument validation, workspace carving and the host-side
// sequencing of the kernels.  No device arithmetic lives here.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/colbandit.h"
#include "cb_launch.h"

using namespace cb;

namespace {

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Token chunk owned by one workgroup of the dense kernel.
constexpr int kChunkTokens = 4096;

struct Layout {
    size_t ctl, list0, list1, stat, stat2, pairs, seg_cnt, rescored, scores, cnt_hist, tau_hist, pi,
        chunk_doc, flag, cid, cstat, ccell, q8, qscale, qscratch, total;
    int cache_cap, TP;
};

// Slots per query in the cell cache.
constexpr int64_t kCacheCapMax = 16384;

Layout make_layout(int nq, int T, int d, int64_t N, int64_t total_tokens) {
    Layout L{};
    size_t o = 0;
    const size_t qn = (size_t)nq * (size_t)N;
    auto take = [&](size_t bytes) {
        const size_t at = o;
        o = align_up(o + bytes);
        return at;
    };
    L.ctl = take(sizeof(QueryCtl) * (size_t)nq);
    L.list0 = take(4 * qn);
    L.list1 = take(4 * qn);
    L.stat = take(8 * qn);
    L.stat2 = take(8 * qn);
    L.pairs = take(8 * 2 * (size_t)(COLBANDIT_MAX_ROUNDS + 4));
    L.seg_cnt = take(4 * (size_t)nq * 64);
    // Two arrays share storage with arrays that are dead while they live: the exhaustive
    // path's score rows (no call uses them together with the running statistics) lie over
    // `stat`, and the rescored survivors (written after the last round) over `stat2`, which
    // only a round's corpus pass and the prune right after it use.
    L.scores = L.stat;
    L.rescored = L.stat2;
    L.cnt_hist = take(4 * (size_t)(COLBANDIT_MAX_ROUNDS + 2) * nq);
    L.tau_hist = take(4 * (size_t)(COLBANDIT_MAX_ROUNDS + 2) * nq);
    L.pi = take(4 * (size_t)nq * T);
    L.chunk_doc = take(4 * (size_t)(total_tokens / kChunkTokens + 16));
    L.flag = take(256);
    L.cache_cap = (int)(N < kCacheCapMax ? N : kCacheCapMax);
    {   // floats per cached document: whole 16-column tiles, in the kernels' 1/2/4/8 tile shapes
        const int tq = (T + 15) / 16;
        L.TP = 16 * (tq <= 1 ? 1 : tq <= 2 ? 2 : tq <= 4 ? 4 : 8);
    }
    L.cid = take(4 * (size_t)nq * L.cache_cap);
    L.cstat = take(8 * (size_t)nq * L.cache_cap);
    L.ccell = take(4 * (size_t)nq * L.cache_cap * L.TP);
    L.q8 = take((size_t)nq * T * d);                 // int8 codes of the queries
    L.qscale = take(4 * (size_t)nq);
    L.qscratch = take(quantize_scratch_bytes(nq));
    L.total = o;
    return L;
}

Work carve(void* ws, const Layout& L) {
    char* b = (char*)ws;
    Work W{};
    W.ctl = (QueryCtl*)(b + L.ctl);
    W.list[0] = (int32_t*)(b + L.list0);
    W.list[1] = (int32_t*)(b + L.list1);
    W.stat = (float2*)(b + L.stat);
    W.stat2 = (float2*)(b + L.stat2);
    W.pairs = (unsigned long long*)(b + L.pairs);
    W.seg_cnt = (int32_t*)(b + L.seg_cnt);
    W.rescored = (float*)(b + L.rescored);
    W.scores = (float*)(b + L.scores);
    W.cnt_hist = (int32_t*)(b + L.cnt_hist);
    W.tau_hist = (float*)(b + L.tau_hist);
    W.pi = (int32_t*)(b + L.pi);
    W.chunk_doc = (int32_t*)(b + L.chunk_doc);
    W.flag = (int*)(b + L.flag);
    W.cache_cap = L.cache_cap;
    W.TP = L.TP;
    W.cid = (int32_t*)(b + L.cid);
    W.cstat = (float2*)(b + L.cstat);
    W.ccell = (float*)(b + L.ccell);
    W.q8 = (int8_t*)(b + L.q8);
    W.qscale = (float*)(b + L.qscale);
    W.qscratch = (void*)(b + L.qscratch);
    return W;
}

int check_shapes(const void* Q, int nq, int T, int d, int dt, const void* docs,
                 const int64_t* off, int64_t N, int64_t total) {
    if (!Q || !docs || !off) return COLBANDIT_ERR_NULL;
    if (nq < 1 || T < 1 || d < 1 || N < 1 || total < N) return COLBANDIT_ERR_SHAPE;
    if (dt != COLBANDIT_F32 && dt != COLBANDIT_BF16) return COLBANDIT_ERR_SHAPE;
    // the selection kernels index a list a few chunks (of up to 16,384 entries) past its end
    if (N > 0x7fffffff - (1 << 17) || nq > 65535) return COLBANDIT_ERR_UNSUPPORTED;
    if (d != 32 && d != 64 && d != 96 && d != 128) return COLBANDIT_ERR_UNSUPPORTED;
    if (T > (dt == COLBANDIT_BF16 ? COLBANDIT_MAX_T : 64)) return COLBANDIT_ERR_UNSUPPORTED;
    if (((uintptr_t)Q & 15) || ((uintptr_t)docs & 15) || ((uintptr_t)off & 7))
        return COLBANDIT_ERR_ALIGNMENT;
    return COLBANDIT_OK;
}

int check_workspace(const void* ws, size_t bytes, size_t need) {
    if (!ws) return COLBANDIT_ERR_NULL;
    if ((uintptr_t)ws & 255) return COLBANDIT_ERR_ALIGNMENT;
    if (bytes < need) return COLBANDIT_ERR_WORKSPACE;
    return COLBANDIT_OK;
}

// Phase timing for colbandit_stats: one HIP event per phase boundary on the call's stream.
enum { PH_FIRST_REVEAL = 0, PH_LATER_REVEAL = 1, PH_SELECT = 2, PH_RESCORE = 3, PH_ROUND2_REVEAL = 4,
       PH_COUNT = 5 };
struct PhaseTimer {
    static constexpr int kMax = 4 * (COLBANDIT_MAX_ROUNDS + 4);
    hipEvent_t ev[kMax];
    int phase[kMax];       // phase that ENDS at event i (event 0 is the start)
    int n = 0;
    bool on = false;
    hipStream_t st = nullptr;
    bool start(hipStream_t s) {
        on = true;
        st = s;
        return mark(-1);
    }
    bool mark(int ph) {
        if (!on) return true;
        if (n >= kMax) return true;
        if (hipEventCreate(&ev[n]) != hipSuccess) return false;
        phase[n] = ph;
        (void)hipEventRecord(ev[n], st);
        ++n;
        return true;
    }
    void collect(float (&ms)[PH_COUNT], float& total) {      // after the stream was synchronised
        for (int i = 0; i < PH_COUNT; ++i) ms[i] = 0.f;
        total = 0.f;
        for (int i = 1; i < n; ++i) {
            float t = 0.f;
            (void)hipEventElapsedTime(&t, ev[i - 1], ev[i]);
            if (phase[i] >= 0) ms[phase[i]] += t;
            total += t;
        }
    }
    void destroy() {
        for (int i = 0; i < n; ++i) (void)hipEventDestroy(ev[i]);
        n = 0;
    }
};

// Number of (query, document) pairs above which a later round is cheaper as one corpus pass
// shared by all queries than as per-pair gathers.  Time model (seconds), with the rates these
// kernels reach on an MI355X: a corpus pass costs the larger of streaming the tokens once
// (~3.5 TB/s) and the matrix work of all query rows against them (~1.15 PFLOP/s); a gathered
// pair streams its document once (~4.5 TB/s) and nothing is shared between queries.  A
// gathered visit also caches the document's cells for the remaining rounds when the query fits
// the cache, so the gather is preferred up to twice the cost of the pass.
unsigned long long dense_pairs_threshold(const Problem& P, int G, bool codes) {
    const double row_bytes = (codes ? 1.0 : 2.0) * P.d;   // int8 codes: half the bytes, twice the rate
    const double rows = (double)(((int64_t)P.nq * G + 15) / 16 * 16);
    const double per_token = fmax(row_bytes / 3.5e12, 2.0 * rows * P.d / (codes ? 2.3e15 : 1.15e15));
    const double t_pass = (double)P.total * per_token;
    const double t_pair = ((double)P.total / (double)P.N) * row_bytes / 4.5e12;
    const double thr = 2.0 * t_pass / t_pair;
    return thr >= 1.8e19 ? ~0ull - 1 : (unsigned long long)thr;
}

// Scratch of colbandit_topk_static: part of the device image, one copy per GPU.  Host code
// never uses this name as an address; it asks the runtime for the copy of the current device.
__device__ __align__(256) unsigned char scratch[COLBANDIT_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, once known
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up once per device).
hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

double rho_n(int n, int T) {
    // finite-population correction, Appendix A
    if (2 * n <= T) return 1.0 - (double)(n - 1) / (double)T;
    return (1.0 - (double)n / (double)T) * (1.0 + 1.0 / (double)n);
}

}  // namespace

extern "C" {

const char* colbandit_strerror(int code) {
    switch (code) {
        case COLBANDIT_OK: return "ok";
        case COLBANDIT_ERR_NULL: return "a required pointer is NULL";
        case COLBANDIT_ERR_SHAPE: return "invalid size (n_queries, T, d, N, total_tokens, K or dtype)";
        case COLBANDIT_ERR_KNOB: return "knob out of range (alpha_ef, delta, M, B or support [a,b])";
        case COLBANDIT_ERR_UNSUPPORTED: return "request outside what this build's kernels cover";
        case COLBANDIT_ERR_WORKSPACE: return "workspace or trace buffer too small";
        case COLBANDIT_ERR_ALIGNMENT: return "pointer not aligned as required";
        case COLBANDIT_ERR_HIP: return "HIP runtime error";
        case COLBANDIT_ERR_BAD_OFFSETS: return "doc_offsets violates its preconditions";
        case COLBANDIT_ERR_TOO_LARGE:
            return "sizes need more scratch than the library's built-in buffer "
                   "(COLBANDIT_STATIC_SCRATCH_BYTES): use colbandit_topk with a workspace";
        default: return "unknown error code";
    }
}

int colbandit_permutation(uint64_t seed, int64_t query_index, int T, int32_t* pi) {
    if (!pi) return COLBANDIT_ERR_NULL;
    if (T < 1 || query_index < 0) return COLBANDIT_ERR_SHAPE;
    uint64_t s = seed + ((uint64_t)query_index + 1ull) * 0x9E3779B97F4A7C15ull;
    for (int t = 0; t < T; ++t) pi[t] = t;
    for (int i = T - 1; i >= 1; --i) {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        z ^= z >> 31;
        const int j = (int)(z % (uint64_t)(i + 1));
        const int32_t tmp = pi[i];
        pi[i] = pi[j];
        pi[j] = tmp;
    }
    return COLBANDIT_OK;
}

double colbandit_radius_prefactor(float alpha_ef, float delta, int T, int64_t N, int n) {
    if (n <= 1) return INFINITY;
    const double lg = log((double)N * (double)T / (double)delta);
    return (double)alpha_ef * (double)T * sqrt(2.0 * lg / (double)n) * sqrt(rho_n(n, T));
}

size_t colbandit_trace_bytes(int n_queries, int T, int B, int64_t N) {
    if (n_queries < 1 || T < 1 || B < 1 || N < 1) return 0;
    const size_t R = (size_t)((T + B - 1) / B), nq = (size_t)n_queries;
    return align_up(4 * (R + 1) * nq) + align_up(4 * R * nq) + 2 * align_up(4 * R * nq * (size_t)N) +
           align_up(R * nq * (size_t)N);
}

size_t colbandit_workspace_bytes(int n_queries, int T, int d, int64_t N, int64_t total_tokens,
                                 int K, int M) {
    (void)K; (void)M;
    if (n_queries < 1 || T < 1 || N < 1 || total_tokens < N) return 0;
    return make_layout(n_queries, T, d, N, total_tokens).total;
}

int colbandit_validate_offsets(const int64_t* doc_offsets, int64_t N, int64_t total_tokens,
                               void* workspace, size_t workspace_bytes, void* stream) {
    if (!doc_offsets) return COLBANDIT_ERR_NULL;
    if (N < 1 || total_tokens < N) return COLBANDIT_ERR_SHAPE;
    int rc = check_workspace(workspace, workspace_bytes, 256);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    int* flag = (int*)workspace;
    if (launch_validate_offsets(doc_offsets, N, total_tokens, flag, st) != hipSuccess)
        return COLBANDIT_ERR_HIP;
    int h = 0;
    if (hipMemcpyAsync(&h, flag, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess)
        return COLBANDIT_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return COLBANDIT_ERR_HIP;
    return h ? COLBANDIT_ERR_BAD_OFFSETS : COLBANDIT_OK;
}

size_t colbandit_quantize_workspace_bytes(int64_t n_segments) {
    if (n_segments < 1) return 0;
    return align_up(quantize_scratch_bytes(n_segments));
}

int colbandit_quantize_i8(const void* x, colbandit_dtype dt, int64_t n_segments,
                          int64_t rows_per_segment, int d, int permille, int8_t* codes,
                          float* scales, void* workspace, size_t workspace_bytes, void* stream) {
    if (!x || !codes || !scales) return COLBANDIT_ERR_NULL;
    if (n_segments < 1 || n_segments > 65535 || rows_per_segment < 1 || d < 1)
        return COLBANDIT_ERR_SHAPE;
    if (dt != COLBANDIT_F32 && dt != COLBANDIT_BF16) return COLBANDIT_ERR_SHAPE;
    if (permille < 1 || permille > 1000) return COLBANDIT_ERR_KNOB;
    if (rows_per_segment > (int64_t)0x7fffffffffffLL / d) return COLBANDIT_ERR_UNSUPPORTED;
    if (((uintptr_t)x & 15) || ((uintptr_t)scales & 3)) return COLBANDIT_ERR_ALIGNMENT;
    int rc = check_workspace(workspace, workspace_bytes, colbandit_quantize_workspace_bytes(n_segments));
    if (rc) return rc;
    const hipError_t e = launch_quantize_i8(x, (int)dt, n_segments, rows_per_segment * d, permille,
                                            codes, scales, workspace, (hipStream_t)stream);
    return e == hipSuccess ? COLBANDIT_OK : COLBANDIT_ERR_HIP;
}

int colbandit_coarse_maxsim(const void* Q, int n_queries, int T, int d, colbandit_dtype dt,
                            const int8_t* docs_i8, const float* docs_scale,
                            const int64_t* doc_offsets, int64_t N, int64_t total_tokens,
                            int permille, float* scores, float* cells, int8_t* q_codes,
                            float* q_scales, void* workspace, size_t workspace_bytes,
                            void* stream) {
    int rc = check_shapes(Q, n_queries, T, d, (int)dt, docs_i8, doc_offsets, N, total_tokens);
    if (rc) return rc;
    if (!docs_scale || !scores) return COLBANDIT_ERR_NULL;
    if (permille < 1 || permille > 1000) return COLBANDIT_ERR_KNOB;
    const Layout L = make_layout(n_queries, T, d, N, total_tokens);
    rc = check_workspace(workspace, workspace_bytes, L.total);
    if (rc) return rc;
    const Work W = carve(workspace, L);
    const Problem P{Q, n_queries, T, d, (int)dt, docs_i8, doc_offsets, N, total_tokens};
    hipStream_t st = (hipStream_t)stream;
    Coarse co{docs_i8, docs_scale, W.q8, W.qscale};
    if (!dense_supported(P, &co)) return COLBANDIT_ERR_UNSUPPORTED;
    hipError_t e = launch_quantize_i8(Q, (int)dt, n_queries, (int64_t)T * d, permille, W.q8,
                                      W.qscale, W.qscratch, st);
    int n_chunks = 0;
    if (e == hipSuccess) e = launch_dense_prepare(P, W, kChunkTokens, &n_chunks, st);
    if (e == hipSuccess) e = launch_dense_score(P, W, kChunkTokens, n_chunks, scores, cells, &co, st);
    if (e == hipSuccess && q_codes)
        e = hipMemcpyAsync(q_codes, W.q8, (size_t)n_queries * T * d, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && q_scales)
        e = hipMemcpyAsync(q_scales, W.qscale, sizeof(float) * n_queries, hipMemcpyDeviceToDevice, st);
    return e == hipSuccess ? COLBANDIT_OK : COLBANDIT_ERR_HIP;
}

// ---- the two non-adaptive baselines (appendix "Compared Methods")

namespace {
struct UniformLayout { size_t base, cells, total; };
UniformLayout uniform_layout(int nq, int T, int d, int64_t N, int64_t total_tokens) {
    UniformLayout U{};
    U.base = make_layout(nq, T, d, N, total_tokens).total;
    U.cells = U.base;
    U.total = U.cells + align_up(4 * (size_t)nq * (size_t)N * (size_t)T);
    return U;
}
struct BallLayout { size_t base, Cz, kq, labels, goff, Qg, ident, part, total; int TG; };
BallLayout ball_layout(int nq, int T, int d, int dt, int64_t N, int64_t total_tokens) {
    BallLayout B{};
    size_t o = make_layout(nq, T, d, N, total_tokens).total;
    B.base = o;
    auto take = [&](size_t bytes) {
        const size_t at = o;
        o = align_up(o + bytes);
        return at;
    };
    const size_t elem = dt == COLBANDIT_BF16 ? 2 : 4;
    B.TG = (T + 3) / 4;
    B.Cz = take(elem * (size_t)nq * T * d);
    B.kq = take(4 * (size_t)nq);
    B.labels = take(4 * (size_t)nq * T);
    B.goff = take(4 * ((size_t)nq + 1));
    if (dt == COLBANDIT_BF16) {
        B.Qg = take(2 * (size_t)nq * B.TG * 4 * d);
        B.ident = take(4 * (size_t)nq * B.TG * 4);
        B.part = take(8 * (size_t)nq * B.TG * (size_t)N);
    }
    B.total = o;
    return B;
}
}  // namespace

size_t colbandit_doc_uniform_workspace_bytes(int n_queries, int T, int d, int64_t N,
                                             int64_t total_tokens) {
    if (n_queries < 1 || T < 1 || N < 1 || total_tokens < N) return 0;
    return uniform_layout(n_queries, T, d, N, total_tokens).total;
}

int colbandit_cells_per_doc(double gamma, int T) {
    if (T < 1) return COLBANDIT_ERR_SHAPE;
    if (!(gamma > 0.0) || !(gamma <= 1.0)) return COLBANDIT_ERR_KNOB;
    const double m = ceil(gamma * (double)T - 1e-9);
    return m < 1.0 ? 1 : (m > (double)T ? T : (int)m);
}

int colbandit_doc_uniform(const void* Q, int n_queries, int T, int d, colbandit_dtype dt,
                          const void* doc_tokens, const int64_t* doc_offsets, int64_t N,
                          int64_t total_tokens, int K, int cells_per_doc, uint64_t seed,
                          float* scores, uint64_t* masks, int64_t* topk_ids, float* topk_scores,
                          void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_shapes(Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens);
    if (rc) return rc;
    if (K < 0 || K > N) return COLBANDIT_ERR_SHAPE;
    if (K > COLBANDIT_MAX_K || T > 64) return COLBANDIT_ERR_UNSUPPORTED;
    if (cells_per_doc < 1 || cells_per_doc > T) return COLBANDIT_ERR_KNOB;
    if (K == 0 && !scores) return COLBANDIT_ERR_NULL;
    if (K > 0 && (!topk_ids || !topk_scores)) return COLBANDIT_ERR_NULL;
    if ((uintptr_t)masks & 7) return COLBANDIT_ERR_ALIGNMENT;
    const UniformLayout U = uniform_layout(n_queries, T, d, N, total_tokens);
    rc = check_workspace(workspace, workspace_bytes, U.total);
    if (rc) return rc;
    const Work W = carve(workspace, make_layout(n_queries, T, d, N, total_tokens));
    const Problem P{Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens};
    hipStream_t st = (hipStream_t)stream;
    float* cells = (float*)((char*)workspace + U.cells);
    float* out = scores ? scores : W.scores;
    // the whole MaxSim matrix (exhaustive row sums go to a scratch array), then the subset sums
    hipError_t e = hipSuccess;
    if (dense_supported(P, nullptr)) {
        int n_chunks = 0;
        e = launch_dense_prepare(P, W, kChunkTokens, &n_chunks, st);
        if (e == hipSuccess)
            e = launch_dense_score(P, W, kChunkTokens, n_chunks, W.rescored, cells, nullptr, st);
    } else {
        e = launch_gather_score(P, W, false, W.rescored, cells, false, st);
    }
    if (e == hipSuccess)
        e = launch_uniform_score(cells, n_queries, N, T, cells_per_doc, seed, out, masks, st);
    if (e == hipSuccess && K > 0) e = launch_topk(P, W, false, out, K, topk_ids, topk_scores, st);
    return e == hipSuccess ? COLBANDIT_OK : COLBANDIT_ERR_HIP;
}

size_t colbandit_ball_carving_workspace_bytes(int n_queries, int T, int d, colbandit_dtype dt,
                                              int64_t N, int64_t total_tokens) {
    if (n_queries < 1 || T < 1 || N < 1 || total_tokens < N) return 0;
    if (dt != COLBANDIT_F32 && dt != COLBANDIT_BF16) return 0;
    return ball_layout(n_queries, T, d, (int)dt, N, total_tokens).total;
}

int colbandit_ball_carving(const void* Q, int n_queries, int T, int d, colbandit_dtype dt,
                           const void* doc_tokens, const int64_t* doc_offsets, int64_t N,
                           int64_t total_tokens, int K, float tau, int32_t* n_clusters,
                           int32_t* labels, void* centroids, float* scores, int64_t* topk_ids,
                           float* topk_scores, void* workspace, size_t workspace_bytes,
                           void* stream) {
    int rc = check_shapes(Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens);
    if (rc) return rc;
    if (K < 0 || K > N) return COLBANDIT_ERR_SHAPE;
    if (K > COLBANDIT_MAX_K || T > 64) return COLBANDIT_ERR_UNSUPPORTED;
    if (!(tau > 0.f) || !(tau <= 1.f)) return COLBANDIT_ERR_KNOB;
    if (K == 0 && !scores) return COLBANDIT_ERR_NULL;
    if (K > 0 && (!topk_ids || !topk_scores)) return COLBANDIT_ERR_NULL;
    if (((uintptr_t)n_clusters & 3) || ((uintptr_t)labels & 3) || ((uintptr_t)centroids & 15))
        return COLBANDIT_ERR_ALIGNMENT;
    const BallLayout B = ball_layout(n_queries, T, d, (int)dt, N, total_tokens);
    rc = check_workspace(workspace, workspace_bytes, B.total);
    if (rc) return rc;
    const Work W = carve(workspace, make_layout(n_queries, T, d, N, total_tokens));
    const Problem P{Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens};
    hipStream_t st = (hipStream_t)stream;
    char* b = (char*)workspace;
    void* Cz = b + B.Cz;
    int32_t* kq = (int32_t*)(b + B.kq);
    int32_t* lab = (int32_t*)(b + B.labels);
    int32_t* goff = (int32_t*)(b + B.goff);
    float* out = scores ? scores : W.scores;
    const size_t elem = dt == COLBANDIT_BF16 ? 2 : 4;

    hipError_t e = launch_ball_carve(P, tau, Cz, lab, kq, st);
    if (e == hipSuccess && dt == COLBANDIT_BF16 && dense_supported(P, nullptr)) {
        // centroids of the batch, four to a group, through the corpus-streaming reveal kernel:
        // its work follows the number of query columns, i.e. the number of centroids
        void* Qg = b + B.Qg;
        int32_t* ident = (int32_t*)(b + B.ident);
        float2* part = (float2*)(b + B.part);
        e = launch_ball_groups(P, Cz, kq, goff, Qg, ident, st);
        int32_t ng = 0;
        if (e == hipSuccess)
            e = hipMemcpyAsync(&ng, goff + n_queries, sizeof(int32_t), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess && (ng < n_queries || (int64_t)ng > (int64_t)n_queries * B.TG))
            e = hipErrorUnknown;
        int n_chunks = 0;
        if (e == hipSuccess) e = launch_dense_prepare(P, W, kChunkTokens, &n_chunks, st);
        if (e == hipSuccess) {
            const Problem P2{Qg, ng, 4, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens};
            Work W2 = W;
            W2.pi = ident;
            W2.stat = part;
            RevealRound rr{};
            rr.r = 1;
            rr.lo = 0;
            rr.nb = 4;
            rr.n = 4;
            rr.dense_thr = ~0ull;
            e = launch_dense_reveal(P2, W2, kChunkTokens, n_chunks, rr, 4, nullptr, st);
        }
        if (e == hipSuccess) e = launch_ball_reduce((const float*)part, 2, goff, n_queries, N, out, st);
    } else if (e == hipSuccess) {
        // fp32: exhaustive scoring of the zero-padded centroid matrix (a zero row's cell is 0)
        const Problem P3{Cz, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens};
        e = launch_gather_score(P3, W, false, out, nullptr, false, st);
    }
    if (e == hipSuccess && n_clusters)
        e = hipMemcpyAsync(n_clusters, kq, 4 * (size_t)n_queries, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && labels)
        e = hipMemcpyAsync(labels, lab, 4 * (size_t)n_queries * T, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && centroids)
        e = hipMemcpyAsync(centroids, Cz, elem * (size_t)n_queries * T * d, hipMemcpyDeviceToDevice, st);
    if (e == hipSuccess && K > 0) e = launch_topk(P, W, false, out, K, topk_ids, topk_scores, st);
    return e == hipSuccess ? COLBANDIT_OK : COLBANDIT_ERR_HIP;
}

size_t colbandit_sizeof_opts(void) { return sizeof(colbandit_opts); }
size_t colbandit_sizeof_stats(void) { return sizeof(colbandit_stats); }

int colbandit_full_maxsim(const void* Q, int n_queries, int T, int d, colbandit_dtype dt,
                          const void* doc_tokens, const int64_t* doc_offsets, int64_t N,
                          int64_t total_tokens, int K, float* scores, int64_t* topk_ids,
                          float* topk_scores, float* cells, float* phase_ms, void* workspace,
                          size_t workspace_bytes, void* stream) {
    int rc = check_shapes(Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens);
    if (rc) return rc;
    if (K < 0 || K > N) return COLBANDIT_ERR_SHAPE;
    if (K > COLBANDIT_MAX_K) return COLBANDIT_ERR_UNSUPPORTED;
    if (K == 0 && !scores) return COLBANDIT_ERR_NULL;
    if (K > 0 && (!topk_ids || !topk_scores)) return COLBANDIT_ERR_NULL;
    const Layout L = make_layout(n_queries, T, d, N, total_tokens);
    rc = check_workspace(workspace, workspace_bytes, L.total);
    if (rc) return rc;

    const Work W = carve(workspace, L);
    const Problem P{Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens};
    hipStream_t st = (hipStream_t)stream;
    float* out = scores ? scores : W.scores;

    // phase_ms: event 0 | chunk table | event 1 | scoring kernel | event 2 | top-K | event 3
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    int n_ev = 0;
    auto mark = [&]() {
        if (phase_ms && n_ev < 4 && hipEventCreate(&ev[n_ev]) == hipSuccess) (void)hipEventRecord(ev[n_ev++], st);
    };
    hipError_t e = hipSuccess;
    mark();
    if (dense_supported(P, nullptr)) {
        int n_chunks = 0;
        e = launch_dense_prepare(P, W, kChunkTokens, &n_chunks, st);
        mark();
        if (e == hipSuccess)
            e = launch_dense_score(P, W, kChunkTokens, n_chunks, out, cells, nullptr, st);
    } else {
        mark();
        e = launch_gather_score(P, W, false, out, cells, false, st);
    }
    mark();
    if (e == hipSuccess && K > 0) e = launch_topk(P, W, false, out, K, topk_ids, topk_scores, st);
    mark();
    if (phase_ms) {
        phase_ms[0] = phase_ms[1] = 0.f;
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess && n_ev == 4) {
            (void)hipEventElapsedTime(&phase_ms[0], ev[1], ev[2]);
            (void)hipEventElapsedTime(&phase_ms[1], ev[2], ev[3]);
        } else if (e == hipSuccess) {
            e = hipErrorUnknown;
        }
        for (int i = 0; i < n_ev; ++i) (void)hipEventDestroy(ev[i]);
    }
    return e == hipSuccess ? COLBANDIT_OK : COLBANDIT_ERR_HIP;
}

// Body of colbandit_topk and colbandit_topk_static.  builtin_scratch: the workspace is the
// current device's copy of `scratch` (looked up only after every argument has passed).
static int topk_impl(const void* Q, int n_queries, int T, int d, colbandit_dtype dt,
                     const void* doc_tokens, const int64_t* doc_offsets, int64_t N,
                     int64_t total_tokens, int K, float alpha_ef, float delta, int M, uint64_t seed,
                     const colbandit_opts* opts, int64_t* topk_ids, float* topk_scores,
                     colbandit_stats* stats, void* workspace, size_t workspace_bytes,
                     bool builtin_scratch, void* stream) {
    int rc = check_shapes(Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens);
    if (rc) return rc;
    if (!topk_ids || !topk_scores) return COLBANDIT_ERR_NULL;
    if (K < 1 || K > N) return COLBANDIT_ERR_SHAPE;
    if (K > COLBANDIT_MAX_K) return COLBANDIT_ERR_UNSUPPORTED;
    if (!(alpha_ef > 0.f) || !(alpha_ef <= 1.f) || !(delta > 0.f) || !(delta < 1.f) || M < 0)
        return COLBANDIT_ERR_KNOB;
    Knobs kn{K, M, 4, -1.f, 1.f};
    const int32_t* user_pi = nullptr;
    void* trace = nullptr;
    size_t trace_bytes = 0;
    bool force_gather = false, no_cache = false;
    int later_rounds = 0;
    Coarse coarse{};
    int q_permille = 999;
    if (opts) {
        if (opts->B < 0) return COLBANDIT_ERR_KNOB;
        if (opts->B > 0) kn.B = opts->B;
        if (!(opts->a == 0.f && opts->b == 0.f)) {
            if (!(opts->a < opts->b)) return COLBANDIT_ERR_KNOB;
            kn.a = opts->a;
            kn.b = opts->b;
        }
        user_pi = opts->pi;
        trace = opts->trace;
        trace_bytes = opts->trace_bytes;
        force_gather = opts->force_gather != 0;
        no_cache = opts->no_cell_cache != 0;
        if (opts->later_rounds < 0 || opts->later_rounds > 2) return COLBANDIT_ERR_KNOB;
        later_rounds = opts->later_rounds;
        if (opts->docs_i8) {
            if (!opts->docs_scale) return COLBANDIT_ERR_NULL;
            if (d % 64 != 0) return COLBANDIT_ERR_UNSUPPORTED;   // int8 MFMA contracts 64 at a time
            if (((uintptr_t)opts->docs_i8 & 15) || ((uintptr_t)opts->docs_scale & 3))
                return COLBANDIT_ERR_ALIGNMENT;
            if (opts->coarse_permille < 0 || opts->coarse_permille > 1000) return COLBANDIT_ERR_KNOB;
            if (opts->coarse_permille > 0) q_permille = opts->coarse_permille;
            coarse.docs8 = opts->docs_i8;
            coarse.dscale = opts->docs_scale;
        }
    }
    if (kn.B > COLBANDIT_MAX_B) return COLBANDIT_ERR_UNSUPPORTED;
    const int R = (T + kn.B - 1) / kn.B;
    if (R > COLBANDIT_MAX_ROUNDS) return COLBANDIT_ERR_UNSUPPORTED;
    const Layout L = make_layout(n_queries, T, d, N, total_tokens);
    if (builtin_scratch) {
        if (L.total > (size_t)COLBANDIT_STATIC_SCRATCH_BYTES) return COLBANDIT_ERR_TOO_LARGE;
        workspace_bytes = (size_t)COLBANDIT_STATIC_SCRATCH_BYTES;
    } else {
        rc = check_workspace(workspace, workspace_bytes, L.total);
        if (rc) return rc;
    }

    Trace tr{};
    if (trace) {
        if ((uintptr_t)trace & 255) return COLBANDIT_ERR_ALIGNMENT;
        if (trace_bytes < colbandit_trace_bytes(n_queries, T, kn.B, N)) return COLBANDIT_ERR_WORKSPACE;
        char* b = (char*)trace;
        const size_t nq = (size_t)n_queries, Rn = (size_t)R;
        tr.count = (int32_t*)b;
        b += align_up(4 * (Rn + 1) * nq);
        tr.tau = (float*)b;
        b += align_up(4 * Rn * nq);
        tr.lcb = (float*)b;
        b += align_up(4 * Rn * nq * (size_t)N);
        tr.ucb = (float*)b;
        b += align_up(4 * Rn * nq * (size_t)N);
        tr.alive = (uint8_t*)b;
    }

    if (builtin_scratch && static_scratch(&workspace) != hipSuccess) return COLBANDIT_ERR_HIP;
    Work W = carve(workspace, L);
    if (no_cache) W.cache_cap = 0;
    const Problem P{Q, n_queries, T, d, (int)dt, doc_tokens, doc_offsets, N, total_tokens};
    hipStream_t st = (hipStream_t)stream;

    PhaseTimer pt;
    if (stats && !pt.start(st)) return COLBANDIT_ERR_HIP;

    hipError_t e = launch_init(P, W, kn, R, seed, user_pi, tr, st);
    const bool loop = N > (int64_t)K + M;    // |A_1| > K + M, else the loop body never runs
    // coarse pass: code the queries (per query) and reveal from the int8 codes
    const Coarse* co = nullptr;
    if (coarse.docs8) {
        coarse.Q8 = W.q8;
        coarse.qscale = W.qscale;
        co = &coarse;
        if (e == hipSuccess && loop)
            e = launch_quantize_i8(Q, (int)dt, n_queries, (int64_t)T * d, q_permille, W.q8,
                                   W.qscale, W.qscratch, st);
    }
    const bool dense = dense_supported(P, co) && !force_gather;
    int n_chunks = 0;
    if (e == hipSuccess && loop && dense) e = launch_dense_prepare(P, W, kChunkTokens, &n_chunks, st);
    unsigned long long round_thr[COLBANDIT_MAX_ROUNDS + 2];
    for (int r = 0; r <= R + 1; ++r) round_thr[r] = ~0ull;
    for (int r = 1; e == hipSuccess && loop && r <= R; ++r) {
        RevealRound rr{};
        rr.r = r;
        rr.lo = (r - 1) * kn.B;
        rr.nb = (r * kn.B < T ? r * kn.B : T) - rr.lo;
        rr.n_prev = rr.lo;
        rr.n = rr.lo + rr.nb;
        const double kap = colbandit_radius_prefactor(alpha_ef, delta, T, N, rr.n);
        rr.kappa = isinf(kap) ? 0.f : (float)kap;   // unused by the kernels when n <= 1
        int G = 1;
        while (G < rr.nb) G <<= 1;
        rr.dense_thr = ~0ull;
        if (r == 1 && dense) {
            e = launch_dense_reveal(P, W, kChunkTokens, n_chunks, rr, G, co, st);
        } else {
            if (r >= 2 && dense && later_rounds != 2)
                rr.dense_thr = later_rounds == 1 ? 0ull : dense_pairs_threshold(P, G, co != nullptr);
            round_thr[r] = rr.dense_thr;
            e = launch_dense_reveal_later(P, W, kChunkTokens, n_chunks, rr, G, co, st);
            if (e == hipSuccess) e = launch_gather_reveal(P, W, rr, co, st);
            if (e == hipSuccess && r >= 2) e = launch_gather_cells(P, W, rr, co, st);
        }
        pt.mark(r == 1 ? PH_FIRST_REVEAL : (r == 2 ? PH_ROUND2_REVEAL : PH_LATER_REVEAL));
        if (e == hipSuccess) e = launch_select_prune(P, W, kn, rr, R, tr, st);
        pt.mark(PH_SELECT);
    }
    // exact rescore from the stored embeddings; cached cells give it only when they are exact
    if (e == hipSuccess) e = launch_gather_score(P, W, true, W.rescored, nullptr, co != nullptr, st);
    if (e == hipSuccess && !co) e = launch_cached_score(P, W, W.rescored, st);
    if (e == hipSuccess) e = launch_topk(P, W, true, W.rescored, K, topk_ids, topk_scores, st);
    pt.mark(PH_RESCORE);
    if (e != hipSuccess) {
        pt.destroy();
        return COLBANDIT_ERR_HIP;
    }
    if (!stats) return COLBANDIT_OK;

    // statistics: the per-round survivor counts come back in one copy after the last kernel
    const size_t nh = (size_t)(R + 1) * n_queries;
    int32_t* hist = (int32_t*)malloc(sizeof(int32_t) * nh);
    if (!hist) { pt.destroy(); return COLBANDIT_ERR_HIP; }
    hipError_t ce = hipMemcpyAsync(hist, W.cnt_hist, sizeof(int32_t) * nh, hipMemcpyDeviceToHost, st);
    unsigned long long pairs_h[2 * (COLBANDIT_MAX_ROUNDS + 2)];
    if (ce == hipSuccess)
        ce = hipMemcpyAsync(pairs_h, W.pairs, sizeof(unsigned long long) * 2 * (size_t)(R + 2),
                            hipMemcpyDeviceToHost, st);
    if (ce == hipSuccess) ce = hipStreamSynchronize(st);
    // the rounds whose device-side test took the corpus pass (the same test as the kernels')
    uint64_t corpus_rounds = 0;
    for (int r = 2; ce == hipSuccess && loop && r <= R; ++r)
        if (round_thr[r] != ~0ull && pairs_h[r] > round_thr[r]) corpus_rounds |= 1ull << (r - 1);
    float ms = 0.f, phase_ms[PH_COUNT] = {0.f, 0.f, 0.f, 0.f, 0.f};
    if (ce == hipSuccess) pt.collect(phase_ms, ms);
    pt.destroy();
    if (ce != hipSuccess) { free(hist); return COLBANDIT_ERR_HIP; }
    for (int q = 0; q < n_queries; ++q) {
        colbandit_stats& s = stats[q];
        memset(&s, 0, sizeof(s));
        s.survivors[0] = (int32_t)N;
        int64_t count = N;
        int n = 0, r = 0;
        bool cached = false;        // the query's list holds cache slots (its cells are cached)
        while (loop && count > (int64_t)K + M && r * kn.B < T) {   // the loop condition of Algorithm 1
            const int lo = r * kn.B, hi = (r + 1) * kn.B < T ? (r + 1) * kn.B : T;
            s.cells_elim += (int64_t)(hi - lo) * count;
            // cells COMPUTED for this round: a corpus pass (round 1 always covers all N documents)
            // computes the batch for every document; the first gathered round of a list that fits
            // the cache computes all T cells of its documents once, later rounds read them back
            const bool pass = r == 0 || ((corpus_rounds >> r) & 1ull);
            if (!cached) {
                if (pass) s.cells_computed += (int64_t)(hi - lo) * N;
                else if (W.cache_cap > 0 && count <= W.cache_cap) {
                    s.cells_computed += (int64_t)T * count;
                    cached = true;
                } else s.cells_computed += (int64_t)(hi - lo) * count;
            }
            n = hi;
            ++r;
            count = hist[(size_t)r * n_queries + q];
            s.survivors[r] = (int32_t)count;
        }
        s.rounds = r;
        s.cells_rescore = (int64_t)T * count;
        s.cells_unique = s.cells_elim + (int64_t)(T - n) * count;
        if (!cached || co) s.cells_computed += (int64_t)T * count;   // the rescore gathers the survivors
        s.ms_total = ms;
        s.ms_first_reveal = phase_ms[PH_FIRST_REVEAL];
        s.ms_later_reveals = phase_ms[PH_LATER_REVEAL] + phase_ms[PH_ROUND2_REVEAL];
        s.ms_reveal_round2 = phase_ms[PH_ROUND2_REVEAL];
        s.ms_select_prune = phase_ms[PH_SELECT];
        s.ms_rescore_topk = phase_ms[PH_RESCORE];
        s.corpus_pass_rounds = corpus_rounds;
        s.pairs_round2 = R >= 2 ? pairs_h[2] : 0ull;
        s.tokens_round2 = R >= 2 ? pairs_h[(R + 2) + 2] : 0ull;
    }
    free(hist);
    return COLBANDIT_OK;
}

int colbandit_topk(const void* Q, int n_queries, int T, int d, colbandit_dtype dt,
                   const void* doc_tokens, const int64_t* doc_offsets, int64_t N,
                   int64_t total_tokens, int K, float alpha_ef, float delta, int M, uint64_t seed,
                   const colbandit_opts* opts, int64_t* topk_ids, float* topk_scores,
                   colbandit_stats* stats, void* workspace, size_t workspace_bytes,
                   void* stream) {
    return topk_impl(Q, n_queries, T, d, dt, doc_tokens, doc_offsets, N, total_tokens, K, alpha_ef,
                     delta, M, seed, opts, topk_ids, topk_scores, stats, workspace, workspace_bytes,
                     false, stream);
}

int colbandit_topk_static(const void* Q, int n_queries, int T, int d, colbandit_dtype dt,
                          const void* doc_tokens, const int64_t* doc_offsets, int64_t N,
                          int64_t total_tokens, int K, float alpha_ef, float delta, int M,
                          uint64_t seed, const colbandit_opts* opts, int64_t* topk_ids,
                          float* topk_scores, void* stream) {
    // stats == NULL: kernel launches only (no events, no host allocation, no read-back)
    return topk_impl(Q, n_queries, T, d, dt, doc_tokens, doc_offsets, N, total_tokens, K, alpha_ef,
                     delta, M, seed, opts, topk_ids, topk_scores, nullptr, nullptr, 0, true, stream);
}

}  // extern "C"
