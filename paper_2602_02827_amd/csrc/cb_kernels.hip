// Gather-reveal / rescore kernel, bound-driven selection and pruning, top-K, and the
// small control kernels.  gfx950 only.
#include <type_traits>

#include "cb_launch.h"

namespace cb {

// =====================================================================================
// init: per-query control, reveal permutations, history and trace fill
// =====================================================================================
__device__ __forceinline__ uint64_t splitmix64_next(uint64_t& s) {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ void k_init(QueryCtl* ctl, int32_t* pi, const int32_t* user_pi, int32_t* cnt_hist,
                       float* tau_hist, int nq, int T, int R, int64_t N, int KM, uint64_t seed,
                       int32_t* tr_count, float* tr_tau, unsigned long long* pairs) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q == 0)
        for (int r = 0; r < 2 * (R + 2); ++r) pairs[r] = 0ull;   // pair counts, then their token counts
    if (q >= nq) return;
    QueryCtl c;
    c.count = (int)N;
    c.cur = 0;
    c.implicit = 1;
    c.active = N > (int64_t)KM;
    c.mode = 0;
    c.pad0 = c.pad1 = c.pad2 = 0;
    ctl[q] = c;
    for (int r = 0; r <= R; ++r) {
        cnt_hist[r * nq + q] = (int)N;
        if (tr_count) tr_count[r * nq + q] = (int)N;
    }
    for (int r = 0; r < R; ++r) {
        tau_hist[r * nq + q] = __uint_as_float(0x7fc00000u);   // quiet NaN: "round not run"
        if (tr_tau) tr_tau[r * nq + q] = __uint_as_float(0x7fc00000u);
    }
    int32_t* p = pi + (size_t)q * T;
    if (user_pi) {
        for (int t = 0; t < T; ++t) {   // clamped: a bad table must not steer a read out of Q
            const int32_t v = user_pi[(size_t)q * T + t];
            p[t] = v < 0 ? 0 : (v >= T ? T - 1 : v);
        }
    } else {
        // Fisher-Yates driven by SplitMix64 (Sec. 4.2: one seeded uniform permutation per query)
        uint64_t s = seed + ((uint64_t)q + 1ull) * 0x9E3779B97F4A7C15ull;
        for (int t = 0; t < T; ++t) p[t] = t;
        for (int i = T - 1; i >= 1; --i) {
            const int j = (int)(splitmix64_next(s) % (uint64_t)(i + 1));
            const int32_t tmp = p[i];
            p[i] = p[j];
            p[j] = tmp;
        }
    }
}

__global__ void k_fill_f32(float* p, size_t n, float v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}
__global__ void k_fill_u8(uint8_t* p, size_t n, uint8_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

hipError_t launch_init(const Problem& P, const Work& W, const Knobs& kn, int R, uint64_t seed,
                       const int32_t* user_pi, const Trace& tr, hipStream_t st) {
    k_init<<<(P.nq + 63) / 64, 64, 0, st>>>(W.ctl, W.pi, user_pi, W.cnt_hist, W.tau_hist, P.nq,
                                            P.T, R, P.N, kn.K + kn.M, seed, tr.count, tr.tau,
                                            W.pairs);
    if (tr.lcb) {
        const size_t n = (size_t)R * P.nq * P.N;
        const int g = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
        k_fill_f32<<<g, 256, 0, st>>>(tr.lcb, n, __builtin_nanf(""));
        k_fill_f32<<<g, 256, 0, st>>>(tr.ucb, n, __builtin_nanf(""));
        k_fill_u8<<<g, 256, 0, st>>>(tr.alive, n, 0);
    }
    return hipGetLastError();
}

// =====================================================================================
// gather kernel: one wavefront per (query, document) pair.
//
// The wavefront keeps the query rows it needs as B operands in registers, streams the
// document's tokens from global memory in blocks of 16 rows (A operand, rows past the
// end of the document repeat its last token, which cannot change a max), runs the MFMA
// chain over d and folds the 16x16 result into a running per-column maximum.
//   GM_REVEAL: one 16-column tile, column c < nb is query token pi[lo+c]; the epilogue
//              merges the batch into the pair's (sum, M2).     [Algorithm 1, reveal step]
//   GM_SCORE : TQ tiles = all T tokens; the epilogue is the row sum. [Eq. (2); rescore]
//   GM_CELLS : TQ tiles = all T tokens; the epilogue stores the pair's T cells in the
//              query's cell cache, merges this round's batch from them and turns the
//              list entry into a cache slot.  A gathered reveal is bound by the bytes of
//              the document, not by the cells computed from them, so a document is
//              visited once and the later rounds (and the rescore) read its cells back;
//              the order in which cells are REVEALED to the bounds is unchanged.
// Which queries a launch serves (uniform per query, from QueryCtl):
//   GM_REVEAL: active, ids mode, and (implicit or count > cache_cap)
//   GM_CELLS : active, ids mode, not implicit, count <= cache_cap
//   GM_SCORE : ctl == nullptr (all documents) or ids mode
// =====================================================================================
enum { GM_REVEAL = 0, GM_SCORE = 1, GM_CELLS = 2 };

struct GatherArgs {
    const void* Q;
    const void* docs;
    const int64_t* off;
    int64_t N, total;
    int T;
    const QueryCtl* ctl;      // nullptr: every query scores all N documents
    int32_t* list0;
    int32_t* list1;
    // reveal
    const int32_t* pi;
    int lo, nb, n_prev, G;
    float2* stat;
    const unsigned long long* pairs_r;   // see dense_round(); nullptr: always gather
    unsigned long long dense_thr;
    // cell cache
    int cache_cap, TP;
    int32_t* cid;
    float2* cstat;
    float* ccell;
    // score
    float* out;
    float* cells;
    int score_slots;          // GM_SCORE: also serve queries whose list holds cache slots
    // int8 codes: a cell is the integer maximum times qscale[q] * dscale[0]
    const float* qscale;
    const float* dscale;
};

template <typename Tag, int D, int TQ, int MODE>
__global__ __launch_bounds__(256) void k_gather(GatherArgs A) {
    using F = Frag<Tag, D>;
    using V = typename F::val_t;
    constexpr bool CODES = !__is_same(V, float);
    const int q = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 15;
    const int kg = lane >> 4;
    const size_t row_bytes = (size_t)D * F::ELEM_BYTES;

    int count = (int)A.N;
    int32_t* list = nullptr;
    const int32_t* slot_ids = nullptr;      // list entries are cache slots: slot -> document id
    if (MODE != GM_SCORE && dense_round(A.pairs_r, A.dense_thr)) return;   // the dense pass serves it
    if (A.ctl) {
        const QueryCtl c = A.ctl[q];
        if (c.mode != 0 && !(MODE == GM_SCORE && A.score_slots)) return;
        if (c.mode != 0) slot_ids = A.cid + (size_t)q * A.cache_cap;
        if (MODE != GM_SCORE && !c.active) return;
        const bool cacheable = !c.implicit && c.count <= A.cache_cap;
        if (MODE == GM_REVEAL && cacheable) return;
        if (MODE == GM_CELLS && !cacheable) return;
        count = c.count;
        if (!c.implicit) list = (c.cur ? A.list1 : A.list0) + (size_t)q * A.N;
    }
    const int first = blockIdx.x * 4 + wave;
    if (first >= count) return;

    // query rows -> B fragments
    F bq[TQ];
    const char* Qq = (const char*)A.Q + (size_t)q * A.T * row_bytes;
#pragma unroll
    for (int tt = 0; tt < TQ; ++tt) {
        int trow;
        if (MODE == GM_REVEAL) {
            trow = A.pi[(size_t)q * A.T + A.lo + (col < A.nb ? col : 0)];
        } else {
            const int t = tt * 16 + col;
            trow = t < A.T ? t : 0;
        }
        bq[tt].load(Qq + (size_t)trow * row_bytes, kg);
    }

    const int stride = gridDim.x * 4;
    for (int k = first; k < count; k += stride) {
        int id = list ? list[k] : k;
        if (slot_ids) id = slot_ids[id];
        int64_t o0 = A.off[id], o1 = A.off[id + 1];
        o0 = o0 < 0 ? 0 : (o0 > A.total ? A.total : o0);
        o1 = o1 < o0 ? o0 : (o1 > A.total ? A.total : o1);

        V h[TQ];
#pragma unroll
        for (int tt = 0; tt < TQ; ++tt) h[tt] = lowest_val<V>();

        // One block of 16 rows in flight per wavefront: the many wavefronts a CU holds already
        // fill the memory system (a deeper per-wavefront pipeline - two blocks and the next
        // pair's offsets in flight - was measured and changed neither the time nor the traffic).
        for (int64_t r0 = o0; r0 < o1; r0 += 16) {
            int64_t row = r0 + col;
            row = row < o1 ? row : o1 - 1;
            F a;
            a.load((const char*)A.docs + (size_t)row * row_bytes, kg);
#pragma unroll
            for (int tt = 0; tt < TQ; ++tt) {
                typename F::acc_t acc = {0, 0, 0, 0};
                F::mma(acc, a, bq[tt]);
                h[tt] = fold_max(h[tt], acc);
            }
        }

        // cross-lane column maxima, decoded to float cells
        constexpr int NWQ = Pack<MODE == GM_REVEAL ? 1 : TQ>::NW;
        float w[NWQ];
        if constexpr (CODES) {
            V wi[NWQ];
            Pack<MODE == GM_REVEAL ? 1 : TQ>::colmax(h, wi);
            const float scale = A.qscale[q] * A.dscale[0];
#pragma unroll
            for (int j = 0; j < NWQ; ++j) w[j] = (float)wi[j] * scale;
        } else {
            Pack<MODE == GM_REVEAL ? 1 : TQ>::colmax(h, w);
        }

        if constexpr (MODE == GM_REVEAL) {
            float sb, m2b;
            batch_stats(w[0], col % A.G, A.nb, A.G, sb, m2b);
            if (lane == 0) {
                const size_t x = (size_t)q * A.N + id;
                float2 st = make_float2(0.f, 0.f);
                if (A.n_prev > 0) st = A.stat[x];
                merge_stats(st.x, st.y, A.n_prev, sb, m2b, A.nb);
                A.stat[x] = st;
            }
        } else if constexpr (MODE == GM_CELLS) {
            using P = Pack<TQ>;
            const int row = lane >> 4;
            const size_t slot = (size_t)q * A.cache_cap + k;
            float* crow = A.ccell + slot * A.TP;
#pragma unroll
            for (int j = 0; j < P::NW; ++j)
                if (P::row_is_primary(row)) crow[P::tile_of_row(j, row) * 16 + col] = w[j];
            // this round's batch: slot s (lane s of row 0) fetches cell pi[lo+s] from its owner
            const int sl = lane < A.nb ? lane : 0;
            const int t = A.pi[(size_t)q * A.T + A.lo + sl];
            const int tile = t >> 4;
            const int src = P::row_of_tile(tile) * 16 + (t & 15);
            float v = __shfl(w[0], src);
            if constexpr (P::NW > 1) {
                const float v1 = __shfl(w[1], src);
                v = tile >= 4 ? v1 : v;
            }
            float sb, m2b;
            batch_stats(v, col % A.G, A.nb, A.G, sb, m2b);
            if (lane == 0) {
                float2 st = A.stat[(size_t)q * A.N + id];
                merge_stats(st.x, st.y, A.n_prev, sb, m2b, A.nb);
                A.cstat[slot] = st;
                A.cid[slot] = id;
                list[k] = k;          // the entry now names its cache slot
            }
        } else {
            using SC = Score<TQ, TQ>;
            float sc[SC::NS];
            SC::finish(w, A.T, col, sc);
            if (lane == 0) A.out[(size_t)q * A.N + (A.ctl ? k : id)] = sc[0];
            if (A.cells) {
                const int row = lane >> 4;
#pragma unroll
                for (int j = 0; j < SC::NW; ++j) {
                    const int t = Pack<TQ>::tile_of_row(j, row) * 16 + col;
                    if (Pack<TQ>::row_is_primary(row) && t < A.T)
                        A.cells[((size_t)q * A.N + id) * A.T + t] = w[j];
                }
            }
        }
    }
}

template <typename Tag, int D, int MODE>
static hipError_t gather_tq(const GatherArgs& A, dim3 grid, hipStream_t st) {
    const dim3 block(256);
    const int tq = (A.T + 15) / 16;
    if (tq <= 1) k_gather<Tag, D, 1, MODE><<<grid, block, 0, st>>>(A);
    else if (tq <= 2) k_gather<Tag, D, 2, MODE><<<grid, block, 0, st>>>(A);
    else if (tq <= 4) k_gather<Tag, D, 4, MODE><<<grid, block, 0, st>>>(A);
    else if constexpr (Tag::wide) k_gather<Tag, D, 8, MODE><<<grid, block, 0, st>>>(A);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

template <typename Tag, int D>
static hipError_t gather_dispatch(const GatherArgs& A, int mode, int nq, int64_t max_count,
                                  hipStream_t st) {
    // Workgroups per query: enough for every pair of a short list to have its own wavefront, at
    // most 256.  (Capping the total over all queries makes the many launches that find nothing
    // to do end sooner, but starves the few queries with long lists when the list lengths are
    // uneven: 256 queries at alpha_ef = 0.5, K = 1 went from 5.5 to 7.6 ms.)
    int gx = (int)((max_count + 3) / 4);
    if (gx > 256) gx = 256;
    if (gx < 1) gx = 1;
    const dim3 grid(gx, nq);
    if (mode == GM_REVEAL) {
        k_gather<Tag, D, 1, GM_REVEAL><<<grid, dim3(256), 0, st>>>(A);
        return hipGetLastError();
    }
    if (mode == GM_CELLS) return gather_tq<Tag, D, GM_CELLS>(A, grid, st);
    return gather_tq<Tag, D, GM_SCORE>(A, grid, st);
}

static void fill_gather_common(GatherArgs& A, const Problem& P, const Work& W) {
    A.Q = P.Q;
    A.docs = P.docs;
    A.off = P.off;
    A.N = P.N;
    A.total = P.total;
    A.T = P.T;
    A.list0 = W.list[0];
    A.list1 = W.list[1];
    A.pi = W.pi;
    A.stat = W.stat;
    A.cache_cap = W.cache_cap;
    A.TP = W.TP;
    A.cid = W.cid;
    A.cstat = W.cstat;
    A.ccell = W.ccell;
}

template <typename Tag>
static hipError_t gather_by_d(const GatherArgs& A, int mode, const Problem& P, int64_t max_count,
                              hipStream_t st) {
    if (P.d == 128) return gather_dispatch<Tag, 128>(A, mode, P.nq, max_count, st);
    if (P.d == 64) return gather_dispatch<Tag, 64>(A, mode, P.nq, max_count, st);
    // widths that only the gather kernels cover (the int8 MFMA contracts 64 elements at a time)
    if constexpr (!__is_same(Tag, i8_tag)) {
        if (P.d == 96) return gather_dispatch<Tag, 96>(A, mode, P.nq, max_count, st);
        if (P.d == 32) return gather_dispatch<Tag, 32>(A, mode, P.nq, max_count, st);
    }
    return hipErrorInvalidValue;
}

static void fill_round(GatherArgs& A, const Work& W, const RevealRound& rr) {
    A.pairs_r = rr.dense_thr == ~0ull ? nullptr : W.pairs + rr.r;
    A.dense_thr = rr.dense_thr;
    A.lo = rr.lo;
    A.nb = rr.nb;
    A.n_prev = rr.n_prev;
    A.G = 1;
    while (A.G < rr.nb) A.G <<= 1;
}

// co != nullptr: the reveal reads the int8 codes instead of the stored embeddings
static hipError_t gather_any(GatherArgs& A, int mode, const Problem& P, int64_t max_count,
                             const Coarse* co, hipStream_t st) {
    if (co) {
        A.Q = co->Q8;
        A.docs = co->docs8;
        A.qscale = co->qscale;
        A.dscale = co->dscale;
        return gather_by_d<i8_tag>(A, mode, P, max_count, st);
    }
    return P.dt == DT_BF16 ? gather_by_d<bf16_tag>(A, mode, P, max_count, st)
                           : gather_by_d<f32_tag>(A, mode, P, max_count, st);
}

hipError_t launch_gather_reveal(const Problem& P, const Work& W, const RevealRound& rr,
                                const Coarse* co, hipStream_t st) {
    GatherArgs A{};
    fill_gather_common(A, P, W);
    A.ctl = W.ctl;
    fill_round(A, W, rr);
    return gather_any(A, GM_REVEAL, P, P.N, co, st);
}

hipError_t launch_gather_cells(const Problem& P, const Work& W, const RevealRound& rr,
                               const Coarse* co, hipStream_t st) {
    if (W.cache_cap <= 0) return hipSuccess;
    GatherArgs A{};
    fill_gather_common(A, P, W);
    A.ctl = W.ctl;
    fill_round(A, W, rr);
    return gather_any(A, GM_CELLS, P, W.cache_cap, co, st);
}

hipError_t launch_gather_score(const Problem& P, const Work& W, bool use_ctl, float* out,
                               float* cells, bool score_slots, hipStream_t st) {
    GatherArgs A{};
    fill_gather_common(A, P, W);
    A.ctl = use_ctl ? W.ctl : nullptr;
    A.out = out;
    A.cells = cells;
    A.score_slots = score_slots ? 1 : 0;
    return gather_any(A, GM_SCORE, P, P.N, nullptr, st);
}

// Exact scores of cached survivors: the T cells of a slot are laid out as the column
// maxima of TQ tiles and summed by the same routine as everywhere else (same bits).
struct CachedScoreArgs {
    const QueryCtl* ctl;
    const int32_t* list0;
    const int32_t* list1;
    const float* ccell;
    int64_t N;
    int T, TP, cache_cap;
    float* out;
};

template <int TQ>
__global__ __launch_bounds__(256) void k_cached_score(CachedScoreArgs A) {
    const int q = blockIdx.y;
    const QueryCtl c = A.ctl[q];
    if (c.mode != 1) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 15;
    const int32_t* list = (c.cur ? A.list1 : A.list0) + (size_t)q * A.N;
    using SC = Score<TQ, TQ>;
    for (int k = blockIdx.x * 4 + wave; k < c.count; k += gridDim.x * 4) {
        const float* crow = A.ccell + ((size_t)q * A.cache_cap + list[k]) * A.TP;
        float h[TQ], w[SC::NW], sc[SC::NS];
#pragma unroll
        for (int tt = 0; tt < TQ; ++tt) h[tt] = crow[tt * 16 + col];
        SC::run(h, A.T, col, w, sc);
        if (lane == 0) A.out[(size_t)q * A.N + k] = sc[0];
    }
}

hipError_t launch_cached_score(const Problem& P, const Work& W, float* out, hipStream_t st) {
    if (W.cache_cap <= 0) return hipSuccess;
    CachedScoreArgs A{W.ctl, W.list[0], W.list[1], W.ccell, P.N, P.T, W.TP, W.cache_cap, out};
    const dim3 grid(16, P.nq), block(256);
    const int tq = (P.T + 15) / 16;
    if (tq <= 1) k_cached_score<1><<<grid, block, 0, st>>>(A);
    else if (tq <= 2) k_cached_score<2><<<grid, block, 0, st>>>(A);
    else if (tq <= 4) k_cached_score<4><<<grid, block, 0, st>>>(A);
    else k_cached_score<8><<<grid, block, 0, st>>>(A);
    return hipGetLastError();
}

// =====================================================================================
// block-wide helpers for the one-workgroup-per-query kernels (1024 threads)
// =====================================================================================
constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_ITEMS = 4;                       // consecutive entries per thread per chunk
constexpr int SEL_CHUNK = SEL_THREADS * SEL_ITEMS;
constexpr int SEL_ITEMS_WIDE = 8;                  // the same for the one streaming pass over a long list
constexpr int SEL_SAMPLE = 16384;                 // sample behind the pre-filter
constexpr int SEL_PREFILTER_MIN = 8 * SEL_SAMPLE;  // lists longer than this are pre-filtered
constexpr int SEL_RUN = 16;                        // the sample is taken in runs of adjacent entries

// Position of sample j in a list of `count` > SEL_PREFILTER_MIN entries: SEL_SAMPLE / SEL_RUN
// evenly spaced runs of SEL_RUN adjacent entries (whole cache lines instead of one entry per
// line; any subset gives a valid lower threshold).
__device__ __forceinline__ int sample_pos(int j, int count) {
    const int run_stride = count / (SEL_SAMPLE / SEL_RUN);
    return (j / SEL_RUN) * run_stride + (j % SEL_RUN);
}

// Exclusive scan of v over the block in thread order; returns the thread's offset and the
// block total.  wtot: LDS int[SEL_WAVES].  Two barriers.
__device__ __forceinline__ int block_excl_scan(int v, int* wtot, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wtot[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) {
        const int x = wtot[w];
        if (w < wave) base += x;
        tot += x;
    }
    __syncthreads();
    total = tot;
    return base + incl - v;
}

// hist[bin] += 1 for every lane with `on`.  Keys of similar magnitude share their leading
// digit, so plain LDS atomics of a wavefront would pile onto one address: up to four rounds of
// "first pending lane's bin, one add for all lanes that share it" come first, the rest (spread
// digits) go as ordinary atomics.
__device__ __forceinline__ void hist_add(uint32_t* hist, int bin, bool on) {
    unsigned long long pending = __ballot(on);
#pragma unroll 1
    for (int it = 0; it < 4 && pending != 0ull; ++it) {
        const int leader = __ffsll((long long)pending) - 1;
        const int lbin = __shfl(bin, leader);
        const unsigned long long same = __ballot(on && bin == lbin) & pending;
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[lbin], (uint32_t)__popcll(same));
        pending &= ~same;
    }
    if ((pending >> (threadIdx.x & 63)) & 1ull) atomicAdd(&hist[bin], 1u);
}

// Key of the K-th largest element (1 <= K <= count) of key_of(0..count-1): three radix
// passes (11+11+10 bits) over the candidates with an LDS histogram each.  Each thread
// takes SEL_ITEMS strided entries per trip so that several loads are in flight.
// hist: LDS uint32[2048]; pick: LDS int[2].
template <class KeyFn>
__device__ uint32_t block_kth_largest(int count, int K, KeyFn key_of, uint32_t* hist, int* pick) {
    uint32_t prefix = 0, pmask = 0;
    int kk = K;
#pragma unroll 1
    for (int p = 0; p < 3; ++p) {
        const int shift = p == 0 ? 21 : (p == 1 ? 10 : 0);
        const int nbins = p == 2 ? 1024 : 2048;
        for (int i = threadIdx.x; i < 2048; i += SEL_THREADS) hist[i] = 0;
        if (threadIdx.x == 0) {
            pick[0] = 0;
            pick[1] = 1;
        }
        __syncthreads();
        for (int base = 0; base < count; base += SEL_CHUNK) {
            uint32_t key[SEL_ITEMS];
#pragma unroll
            for (int u = 0; u < SEL_ITEMS; ++u) {
                const int idx = base + u * SEL_THREADS + threadIdx.x;
                key[u] = idx < count ? key_of(idx) : 0u;
            }
#pragma unroll
            for (int u = 0; u < SEL_ITEMS; ++u) {
                const int idx = base + u * SEL_THREADS + threadIdx.x;
                hist_add(hist, (int)((key[u] >> shift) & (nbins - 1)),
                         idx < count && (key[u] & pmask) == prefix);
            }
        }
        __syncthreads();
        if (threadIdx.x < 64) {
            const int lane = threadIdx.x;
            const int per = nbins / 64;
            const int hi = nbins - 1 - lane * per;       // this lane's bins, descending
            int local = 0;
            for (int j = 0; j < per; ++j) local += (int)hist[hi - j];
            int incl = local;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            const int excl = incl - local;
            if (excl < kk && kk <= incl) {
                int run = excl;
                for (int j = 0; j < per; ++j) {
                    const int c = (int)hist[hi - j];
                    if (run + c >= kk) {
                        pick[0] = hi - j;
                        pick[1] = kk - run;
                        break;
                    }
                    run += c;
                }
            }
        }
        __syncthreads();
        prefix |= (uint32_t)pick[0] << shift;
        pmask |= (uint32_t)(nbins - 1) << shift;
        kk = pick[1];
        __syncthreads();
    }
    return prefix;
}

// The same selection over SEL_SAMPLE keys that each thread computes once and keeps in
// registers for all three passes (thread t holds keys t, t + SEL_THREADS, ...).
constexpr int SEL_SAMPLE_PER_THREAD = SEL_SAMPLE / SEL_THREADS;
template <class KeyFn>
__device__ uint32_t block_kth_largest_sample(int K, KeyFn key_of, uint32_t* hist, int* pick) {
    uint32_t key[SEL_SAMPLE_PER_THREAD];
#pragma unroll
    for (int u = 0; u < SEL_SAMPLE_PER_THREAD; ++u) key[u] = key_of(u * SEL_THREADS + (int)threadIdx.x);
    uint32_t prefix = 0, pmask = 0;
    int kk = K;
#pragma unroll 1
    for (int p = 0; p < 3; ++p) {
        const int shift = p == 0 ? 21 : (p == 1 ? 10 : 0);
        const int nbins = p == 2 ? 1024 : 2048;
        for (int i = threadIdx.x; i < 2048; i += SEL_THREADS) hist[i] = 0;
        if (threadIdx.x == 0) {
            pick[0] = 0;
            pick[1] = 1;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < SEL_SAMPLE_PER_THREAD; ++u)
            hist_add(hist, (int)((key[u] >> shift) & (nbins - 1)), (key[u] & pmask) == prefix);
        __syncthreads();
        if (threadIdx.x < 64) {
            const int lane = threadIdx.x;
            const int per = nbins / 64;
            const int hi = nbins - 1 - lane * per;       // this lane's bins, descending
            int local = 0;
            for (int j = 0; j < per; ++j) local += (int)hist[hi - j];
            int incl = local;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            const int excl = incl - local;
            if (excl < kk && kk <= incl) {
                int run = excl;
                for (int j = 0; j < per; ++j) {
                    const int c = (int)hist[hi - j];
                    if (run + c >= kk) {
                        pick[0] = hi - j;
                        pick[1] = kk - run;
                        break;
                    }
                    run += c;
                }
            }
        }
        __syncthreads();
        prefix |= (uint32_t)pick[0] << shift;
        pmask |= (uint32_t)(nbins - 1) << shift;
        kk = pick[1];
        __syncthreads();
    }
    return prefix;
}

// The batch statistics of batch_stats_g<G> evaluated by ONE thread on the G slot values
// (same pairing of additions, lane by lane, so the bits are those of the cross-lane form).
__device__ __forceinline__ void lanes_sum(float (&v)[16], int G) {
    float t[16];
    if (G >= 16) {
        for (int i = 0; i < 16; ++i) t[i] = v[i] + v[15 - i];
        for (int i = 0; i < 16; ++i) v[i] = t[i];
    }
    if (G >= 8) {
        for (int i = 0; i < 16; ++i) t[i] = v[i] + v[(i & 8) | (7 - (i & 7))];
        for (int i = 0; i < 16; ++i) v[i] = t[i];
    }
    if (G >= 4) {
        for (int i = 0; i < 16; ++i) t[i] = v[i] + v[i ^ 2];
        for (int i = 0; i < 16; ++i) v[i] = t[i];
    }
    if (G >= 2) {
        for (int i = 0; i < 16; ++i) t[i] = v[i] + v[i ^ 1];
        for (int i = 0; i < 16; ++i) v[i] = t[i];
    }
}
__device__ __forceinline__ void batch_stats_thread(const float (&c)[16], int nb, int G, float& s,
                                                   float& m2) {
    float v[16];
    for (int i = 0; i < 16; ++i) v[i] = (i < nb) ? c[i] : 0.f;
    lanes_sum(v, G);
    s = v[0];
    float dv[16];
    for (int i = 0; i < 16; ++i) {
        const float d = (i < nb) ? (c[i] - div_count(v[i], nb)) : 0.f;
        dv[i] = d * d;
    }
    lanes_sum(dv, G);
    m2 = dv[0];
}

// =====================================================================================
// threshold + prune: tau_r = K-th largest LCB over the active set, A_{r+1} = {UCB >= tau_r}
// (Algorithm 1, threshold and elimination steps), one workgroup per query, stable.
// For a query whose cells are cached the round's reveal is folded in first: each entry's
// (sum, M2) takes the batch pi[lo..lo+nb) from its cached cells.
// =====================================================================================
struct SelArgs {
    QueryCtl* ctl;
    int32_t* list0;
    int32_t* list1;
    float2* stat;
    const float2* stat2;
    unsigned long long* pairs;           // [R+2] pairs, then [R+2] document tokens of those pairs
    const int64_t* off;                  // document offsets (token counts of the kept pairs)
    int R;
    unsigned long long dense_thr;        // ~0: this round cannot be a dense one
    int64_t N;
    int nq, T, K, KM;
    int r, n, n_prev, lo, nb, G;
    float kappa, a, b;
    const int32_t* pi;
    int cache_cap, TP;
    const int32_t* cid;
    float2* cstat;
    const float* ccell;
    int32_t* cnt_hist;
    float* tau_hist;
    int32_t* tr_count;
    float* tr_tau;
    float* tr_lcb;
    float* tr_ucb;
    uint8_t* tr_alive;
    // segmented pre-filter of long lists (k_select_segments): candidates of segment s sit at
    // out[s * seg_len(count, n_seg) ...], seg_cnt[q][s] of them
    int n_seg;                // 0: no segmented pre-filter ran
    int32_t* seg_cnt;         // [nq][SEG_MAX]
};

constexpr int SEG_MAX = 64;
// entries per segment: a multiple of the widest per-thread run
__device__ __host__ __forceinline__ int seg_len(int count, int n_seg) {
    return ((count + n_seg - 1) / n_seg + 15) & ~15;
}

// Candidates that the segment workgroups left at the segment starts of `buf` -> one contiguous
// run at the front, order kept.  A destination never lies beyond its source, and a chunk is read
// completely before it is written.
__device__ int merge_segments(int32_t* buf, const int32_t* cnt, int count, int n_seg) {
    const int len = seg_len(count, n_seg);
    int base = 0;
    for (int sg = 0; sg < n_seg; ++sg) {
        const int c = cnt[sg];
        const int src = sg * len;
        if (src != base) {
            for (int k0 = 0; k0 < c; k0 += SEL_THREADS) {
                const int k = k0 + (int)threadIdx.x;
                const int v = k < c ? buf[src + k] : 0;
                __syncthreads();
                if (k < c) buf[base + k] = v;
                __syncthreads();
            }
        }
        base += c;
    }
    __syncthreads();
    return base;
}

__global__ __launch_bounds__(SEL_THREADS) void k_select_prune(SelArgs A) {
    __shared__ uint32_t hist[2048];
    __shared__ int pick[2];
    __shared__ int wtot[SEL_WAVES];
    __shared__ unsigned long long kept_tokens;
    const int q = blockIdx.x;
    const QueryCtl c = A.ctl[q];
    if (!c.active) {
        if (threadIdx.x == 0) {
            A.cnt_hist[A.r * A.nq + q] = c.count;
            if (A.tr_count) A.tr_count[A.r * A.nq + q] = c.count;
        }
        return;
    }
    const int count = c.count;
    const int32_t* in = c.implicit ? nullptr : (c.cur ? A.list1 : A.list0) + (size_t)q * A.N;
    const int out_sel = c.implicit ? 0 : (c.cur ^ 1);
    int32_t* out = (out_sel ? A.list1 : A.list0) + (size_t)q * A.N;
    // entries are cache slots if the query was switched earlier (mode 1) or by this
    // round's cell-caching gather (same rule as in k_gather)
    const bool dense = A.dense_thr != ~0ull && dense_round(A.pairs + A.r, A.dense_thr);
    const bool slots = c.mode == 1 || (c.mode == 0 && !c.implicit && count <= A.cache_cap && !dense);
    const float2* stat = slots ? A.cstat + (size_t)q * A.cache_cap : A.stat + (size_t)q * A.N;
    const int32_t* cid = A.cid + (size_t)q * A.cache_cap;
    const int n = A.n, T = A.T;
    const float kappa = A.kappa, a = A.a, b = A.b;
    if (threadIdx.x == 0) kept_tokens = 0ull;       // published by the barriers of the passes below
    long long my_tokens = 0;                        // tokens of the documents this thread keeps

    if (c.mode == 1) {          // fold this round's batch in from the cached cells
        float2* cst = A.cstat + (size_t)q * A.cache_cap;
        const int32_t* pq = A.pi + (size_t)q * T + A.lo;
        for (int idx = threadIdx.x; idx < count; idx += SEL_THREADS) {
            const int e = in[idx];
            const float* crow = A.ccell + ((size_t)q * A.cache_cap + e) * A.TP;
            float cv[16];
            for (int i = 0; i < 16; ++i) cv[i] = i < A.nb ? crow[pq[i]] : 0.f;
            float sb, m2b;
            batch_stats_thread(cv, A.nb, A.G, sb, m2b);
            float2 st = cst[e];
            merge_stats(st.x, st.y, A.n_prev, sb, m2b, A.nb);
            cst[e] = st;
        }
        __syncthreads();
    }

    const bool segmented = A.n_seg > 0 && count > SEL_PREFILTER_MIN && !slots;
    if (dense && c.mode == 0 && in && !segmented) {   // fold in the batch a dense pass left in stat2
        float2* dst = A.stat + (size_t)q * A.N;
        const float2* bat = A.stat2 + (size_t)q * A.N;
        for (int idx = threadIdx.x; idx < count; idx += SEL_THREADS) {
            const int e = in[idx];
            float2 st = dst[e];
            const float2 bb = bat[e];
            merge_stats(st.x, st.y, A.n_prev, bb.x, bb.y, A.nb);
            dst[e] = st;
        }
        __syncthreads();
    }

    auto key_of = [&](const int32_t* l, int idx) -> uint32_t {
        const int e = l ? l[idx] : idx;
        float lcb, ucb;
        const float2 st = stat[e];
        interval(st.x, st.y, n, T, kappa, a, b, lcb, ucb);
        return float_key(lcb);
    };
    const size_t tro = ((size_t)(A.r - 1) * A.nq + q) * A.N;
    // Stable compaction of {entry of l[0..cnt) : UCB >= thr} into outl (outl may be l itself:
    // a chunk is read completely before anything is written, and writes stay below the
    // next chunk).  The trace takes every dropped entry, and the kept ones if trace_kept.
    auto filter = [&](auto items_c, const int32_t* l, int cnt, int32_t* outl, float thr,
                      bool trace_kept) -> int {
        constexpr int ITEMS = decltype(items_c)::value;      // entries per thread per chunk
        constexpr int CHUNK = SEL_THREADS * ITEMS;
        int base = 0;
        // software pipeline over chunks: the entries are fetched two chunks ahead and their
        // statistics one chunk ahead, so the loads of the next chunk are in flight across
        // this chunk's scan and its barriers
        const int t0 = threadIdx.x * ITEMS;                 // ITEMS consecutive entries
        auto load_e = [&](int start, int (&e)[ITEMS]) {
#pragma unroll
            for (int u = 0; u < ITEMS; ++u) {
                const int idx = start + t0 + u;
                e[u] = idx < cnt ? (l ? l[idx] : idx) : 0;
            }
        };
        auto load_s = [&](int start, const int (&e)[ITEMS], float2 (&st)[ITEMS]) {
#pragma unroll
            for (int u = 0; u < ITEMS; ++u)
                st[u] = (start + t0 + u < cnt) ? stat[e[u]] : make_float2(0.f, 0.f);
        };
        int e[ITEMS], e_next[ITEMS];
        float2 st[ITEMS];
        load_e(0, e);
        load_s(0, e, st);
        load_e(CHUNK, e_next);
        for (int start = 0; start < cnt; start += CHUNK) {
            const int i0 = start + t0;
            int e_next2[ITEMS];
            float2 st_next[ITEMS];
            load_s(start + CHUNK, e_next, st_next);
            load_e(start + 2 * CHUNK, e_next2);
            unsigned keep = 0;
#pragma unroll
            for (int u = 0; u < ITEMS; ++u) {
                if (i0 + u < cnt) {
                    float lcb, ucb;
                    interval(st[u].x, st[u].y, n, T, kappa, a, b, lcb, ucb);
                    const bool kp = ucb >= thr;
                    keep |= (kp ? 1u : 0u) << u;
                    if (A.tr_lcb && (trace_kept || !kp)) {
                        const int id = slots ? cid[e[u]] : e[u];
                        A.tr_lcb[tro + id] = lcb;
                        A.tr_ucb[tro + id] = ucb;
                        A.tr_alive[tro + id] = kp ? 1 : 0;
                    }
                }
            }
            if (__syncthreads_or(keep != 0)) {          // a pre-filter keeps nothing of most chunks
                int total;
                int pos = base + block_excl_scan(__popc(keep), wtot, total);
#pragma unroll
                for (int u = 0; u < ITEMS; ++u)
                    if (keep & (1u << u)) {
                        outl[pos++] = e[u];
                        // the final pass over document ids also adds up what a gather of the
                        // survivors would have to read
                        if (trace_kept && !slots) my_tokens += A.off[e[u] + 1] - A.off[e[u]];
                    }
                base += total;
            }
#pragma unroll
            for (int u = 0; u < ITEMS; ++u) {
                e[u] = e_next[u];
                st[u] = st_next[u];
                e_next[u] = e_next2[u];
            }
        }
        return base;
    };

    // Large active sets (the first round): a strided sample gives a threshold tau_lo that
    // cannot exceed tau (the K-th largest of a subset is at most that of the whole set), so
    // one streaming pass keeps the candidates {UCB >= tau_lo}, a superset of both the
    // survivors and the K largest LCBs; the exact threshold and the prune then run on
    // those few.
    const int32_t* sel_in = in;
    int sel_count = count;
    if (segmented) {
        // the segment workgroups have folded, sampled and pre-filtered; gather their candidates
        sel_count = merge_segments(out, A.seg_cnt + (size_t)q * SEG_MAX, count, A.n_seg);
        sel_in = out;
        if (dense && c.mode == 0 && in) {       // the candidates' statistics take the round's batch
            float2* dst = A.stat + (size_t)q * A.N;
            const float2* bat = A.stat2 + (size_t)q * A.N;
            for (int idx = threadIdx.x; idx < sel_count; idx += SEL_THREADS) {
                const int e = out[idx];
                float2 st = dst[e];
                const float2 bb = bat[e];
                merge_stats(st.x, st.y, A.n_prev, bb.x, bb.y, A.nb);
                dst[e] = st;
            }
            __syncthreads();
        }
    } else if (count > SEL_PREFILTER_MIN) {
        auto key_s = [&](int j) -> uint32_t { return key_of(in, sample_pos(j, count)); };
        const float tau_lo = key_float(block_kth_largest_sample(A.K, key_s, hist, pick));
        // the streaming pass: wide chunks keep enough loads in flight for one workgroup
        sel_count = filter(std::integral_constant<int, SEL_ITEMS_WIDE>{}, in, count, out, tau_lo, false);
        sel_in = out;
    }
    uint32_t tkey;
    if (sel_count > SEL_PREFILTER_MIN) {
        // Still a long list (a conservative radius prunes little): the exact threshold depends
        // only on the entries whose LCB reaches a sampled lower threshold (the K-th largest of
        // a subset cannot exceed that of the whole list, so these include the K largest).  One
        // pass collects them, in any order, into the list buffer that this round no longer
        // reads; the three radix passes then run over those few instead of the whole list.
        auto key_s = [&](int j) -> uint32_t { return key_of(sel_in, sample_pos(j, sel_count)); };
        const uint32_t lo_key = block_kth_largest_sample(A.K, key_s, hist, pick);
        int32_t* few = (out_sel ? A.list0 : A.list1) + (size_t)q * A.N;   // sel_in == out here
        if (threadIdx.x == 0) pick[0] = 0;
        __syncthreads();
        const int lane = threadIdx.x & 63;
        for (int base0 = 0; base0 < sel_count; base0 += SEL_CHUNK) {
            int e[SEL_ITEMS];
            bool on[SEL_ITEMS];
#pragma unroll
            for (int u = 0; u < SEL_ITEMS; ++u) {
                const int idx = base0 + u * SEL_THREADS + (int)threadIdx.x;
                e[u] = idx < sel_count ? sel_in[idx] : 0;
            }
#pragma unroll
            for (int u = 0; u < SEL_ITEMS; ++u) {
                const int idx = base0 + u * SEL_THREADS + (int)threadIdx.x;
                float lcb, ucb;
                const float2 st = stat[e[u]];
                interval(st.x, st.y, n, T, kappa, a, b, lcb, ucb);
                on[u] = idx < sel_count && float_key(lcb) >= lo_key;
            }
#pragma unroll
            for (int u = 0; u < SEL_ITEMS; ++u) {
                const unsigned long long m = __ballot(on[u]);
                if (m != 0ull) {                            // uniform over the wavefront
                    int at = 0;
                    if (lane == 0) at = atomicAdd(&pick[0], __popcll(m));
                    at = __shfl(at, 0);
                    if (on[u]) few[at + __popcll(m & ((1ull << lane) - 1ull))] = e[u];
                }
            }
        }
        __syncthreads();
        const int n_few = pick[0];
        __syncthreads();
        auto key_few = [&](int idx) -> uint32_t { return key_of(few, idx); };
        tkey = block_kth_largest(n_few, A.K, key_few, hist, pick);
    } else {
        auto key_sel = [&](int idx) -> uint32_t { return key_of(sel_in, idx); };
        tkey = block_kth_largest(sel_count, A.K, key_sel, hist, pick);
    }
    const float tau = key_float(tkey);
    const int base = filter(std::integral_constant<int, SEL_ITEMS>{}, sel_in, sel_count, out, tau, true);
    if (!slots) {                       // uniform over the workgroup
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) my_tokens += __shfl_down(my_tokens, o);
        if ((threadIdx.x & 63) == 0 && my_tokens != 0)
            atomicAdd(&kept_tokens, (unsigned long long)my_tokens);
        __syncthreads();
    }

    if (threadIdx.x == 0) {
        QueryCtl nc;
        nc.count = base;
        nc.cur = out_sel;
        nc.implicit = 0;
        nc.active = base > A.KM;
        nc.mode = slots ? 1 : 0;
        nc.pad0 = nc.pad1 = nc.pad2 = 0;
        A.ctl[q] = nc;
        // what the next round would have to gather: the active sets still held as ids
        if (nc.active && nc.mode == 0) {
            atomicAdd(A.pairs + A.r + 1, (unsigned long long)base);
            atomicAdd(A.pairs + (A.R + 2) + A.r + 1, kept_tokens);
        }
        A.cnt_hist[A.r * A.nq + q] = base;
        A.tau_hist[(A.r - 1) * A.nq + q] = tau;
        if (A.tr_count) {
            A.tr_count[A.r * A.nq + q] = base;
            A.tr_tau[(A.r - 1) * A.nq + q] = tau;
        }
    }
}

// A cheap upper estimate of interval()'s UCB for the pre-filter (n, T, kappa, b uniform).
struct FastUcb {
    float c_hat, c_sig, rest_b;
    int mode;           // 0: hard bound only (n <= 1), 1: hybrid, 2: exact sum (n >= T)
};
__device__ __forceinline__ FastUcb fast_ucb_consts(int n, int T, float kappa, float b) {
    FastUcb f;
    f.mode = n <= 1 ? 0 : (n >= T ? 2 : 1);
    f.c_hat = n > 0 ? (float)T / (float)n : 0.f;
    f.c_sig = n > 1 ? kappa * kappa / (float)(n - 1) : 0.f;
    f.rest_b = (float)(T - n) * b;
    return f;
}
__device__ __forceinline__ float fast_ucb(float S, float M2, int n, int T, const FastUcb& f) {
    (void)n; (void)T;
    const float ub = S + f.rest_b;
    if (f.mode == 0) return ub;
    if (f.mode == 2) return S;
    const float r = __builtin_amdgcn_sqrtf(fmaxf(M2, 0.f) * f.c_sig);
    return fminf(ub, S * f.c_hat + r);
}

// Pre-filter of a long active list, spread over n_seg workgroups per query (one workgroup cannot
// pull a multi-megabyte list from memory fast enough).  Every workgroup of a query derives the
// same lower threshold tau_lo from the same sample, then streams its own segment once and keeps
// {UCB >= tau_lo} in order at the start of its segment of the output list, recording how many.
// In a corpus-pass round the round's batch (stat2) is merged in registers only: nothing is
// written back here, because other workgroups of the query are still sampling; k_select_prune
// gathers the segments and stores the merged statistics of the candidates, the only entries
// that are ever read again.
__global__ __launch_bounds__(SEL_THREADS) void k_select_segments(SelArgs A) {
    __shared__ uint32_t hist[2048];
    __shared__ int pick[2];
    __shared__ int wtot[SEL_WAVES];
    const int q = blockIdx.y, sg = blockIdx.x;
    const QueryCtl c = A.ctl[q];
    if (!c.active) return;
    const int count = c.count;
    if (count <= SEL_PREFILTER_MIN) return;
    const bool dense = A.dense_thr != ~0ull && dense_round(A.pairs + A.r, A.dense_thr);
    const bool slots = c.mode == 1 || (c.mode == 0 && !c.implicit && count <= A.cache_cap && !dense);
    if (slots) return;                      // cache-sized lists are never this long
    const int32_t* in = c.implicit ? nullptr : (c.cur ? A.list1 : A.list0) + (size_t)q * A.N;
    const int out_sel = c.implicit ? 0 : (c.cur ^ 1);
    int32_t* out = (out_sel ? A.list1 : A.list0) + (size_t)q * A.N;
    const float2* stat = A.stat + (size_t)q * A.N;
    const float2* bat = A.stat2 + (size_t)q * A.N;
    const bool fold = dense && in != nullptr;
    const int n = A.n, T = A.T;
    const float kappa = A.kappa, a = A.a, b = A.b;

    auto stat_of = [&](int e) -> float2 {
        float2 st = stat[e];
        if (fold) {
            const float2 bb = bat[e];
            merge_stats(st.x, st.y, A.n_prev, bb.x, bb.y, A.nb);
        }
        return st;
    };
    auto key_s = [&](int j) -> uint32_t {
        const int pos = sample_pos(j, count);
        const float2 st = stat_of(in ? in[pos] : pos);
        float lcb, ucb;
        interval(st.x, st.y, n, T, kappa, a, b, lcb, ucb);
        return float_key(lcb);
    };
    const float tau_lo = key_float(block_kth_largest_sample(A.K, key_s, hist, pick));
    const FastUcb fk = fast_ucb_consts(n, T, kappa, b);
    const float tau_fast = tau_lo - (1e-3f + 1e-5f * fabsf(tau_lo));

    const int len = seg_len(count, A.n_seg);
    const int lo = sg * len;
    const int hi = lo + len < count ? lo + len : count;
    const size_t tro = ((size_t)(A.r - 1) * A.nq + q) * A.N;
    constexpr int ITEMS = SEL_ITEMS_WIDE;
    constexpr int CHUNK = SEL_THREADS * ITEMS;
    const int t0 = threadIdx.x * ITEMS;
    auto load_e = [&](int start, int (&e)[ITEMS]) {
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const int idx = start + t0 + u;
            e[u] = idx < hi ? (in ? in[idx] : idx) : 0;
        }
    };
    auto load_s = [&](int start, const int (&e)[ITEMS], float2 (&st)[ITEMS], float2 (&bb)[ITEMS]) {
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            const bool ok = start + t0 + u < hi;
            st[u] = ok ? stat[e[u]] : make_float2(0.f, 0.f);
            bb[u] = (ok && fold) ? bat[e[u]] : make_float2(0.f, 0.f);
        }
    };
    int base = 0;
    int e[ITEMS], e_next[ITEMS];
    float2 st[ITEMS], bb[ITEMS];
    load_e(lo, e);
    load_s(lo, e, st, bb);
    load_e(lo + CHUNK, e_next);
    for (int start = lo; start < hi; start += CHUNK) {
        const int i0 = start + t0;
        int e_next2[ITEMS];
        float2 st_next[ITEMS], bb_next[ITEMS];
        load_s(start + CHUNK, e_next, st_next, bb_next);
        load_e(start + 2 * CHUNK, e_next2);
        unsigned keep = 0;
        if (A.tr_lcb || fold) {
            // exact intervals: the trace records every dropped entry's interval
#pragma unroll
            for (int u = 0; u < ITEMS; ++u) {
                if (i0 + u < hi) {
                    if (fold) merge_stats(st[u].x, st[u].y, A.n_prev, bb[u].x, bb[u].y, A.nb);
                    float lcb, ucb;
                    interval(st[u].x, st[u].y, n, T, kappa, a, b, lcb, ucb);
                    const bool kp = ucb >= tau_lo;
                    keep |= (kp ? 1u : 0u) << u;
                    if (A.tr_lcb && !kp) {
                        A.tr_lcb[tro + e[u]] = lcb;
                        A.tr_ucb[tro + e[u]] = ucb;
                        A.tr_alive[tro + e[u]] = 0;
                    }
                }
            }
        } else {
            // A pre-filter may keep too much but never too little: the UCB is evaluated with
            // reciprocal multiplications and the hardware square root, and compared with the
            // threshold lowered by far more than the error of that shortcut (values are of
            // size <= T; the shortcut is good to a few ulps).
#pragma unroll
            for (int u = 0; u < ITEMS; ++u) {
                if (i0 + u < hi) {
                    const float ucb = fast_ucb(st[u].x, st[u].y, n, T, fk);
                    keep |= (ucb >= tau_fast ? 1u : 0u) << u;
                }
            }
        }
        if (__syncthreads_or(keep != 0)) {
            int total;
            int pos = lo + base + block_excl_scan(__popc(keep), wtot, total);
#pragma unroll
            for (int u = 0; u < ITEMS; ++u)
                if (keep & (1u << u)) out[pos++] = e[u];
            base += total;
        }
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) {
            e[u] = e_next[u];
            st[u] = st_next[u];
            bb[u] = bb_next[u];
            e_next[u] = e_next2[u];
        }
    }
    if (threadIdx.x == 0) A.seg_cnt[(size_t)q * SEG_MAX + sg] = base;
}

hipError_t launch_select_prune(const Problem& P, const Work& W, const Knobs& kn,
                               const RevealRound& rr, int R, const Trace& tr, hipStream_t st) {
    SelArgs A{};
    A.ctl = W.ctl;
    A.list0 = W.list[0];
    A.list1 = W.list[1];
    A.stat = W.stat;
    A.stat2 = W.stat2;
    A.pairs = W.pairs;
    A.off = P.off;
    A.R = R;
    A.dense_thr = rr.dense_thr;
    A.N = P.N;
    A.nq = P.nq;
    A.T = P.T;
    A.K = kn.K;
    A.KM = kn.K + kn.M;
    A.r = rr.r;
    A.n = rr.n;
    A.n_prev = rr.n_prev;
    A.lo = rr.lo;
    A.nb = rr.nb;
    A.G = 1;
    while (A.G < rr.nb) A.G <<= 1;
    A.kappa = rr.kappa;
    A.a = kn.a;
    A.b = kn.b;
    A.pi = W.pi;
    A.cache_cap = W.cache_cap;
    A.TP = W.TP;
    A.cid = W.cid;
    A.cstat = W.cstat;
    A.ccell = W.ccell;
    A.cnt_hist = W.cnt_hist;
    A.tau_hist = W.tau_hist;
    A.tr_count = tr.count;
    A.tr_tau = tr.tau;
    A.tr_lcb = tr.lcb;
    A.tr_ucb = tr.ucb;
    A.tr_alive = tr.alive;
    // lists longer than the pre-filter limit are first cut down by several workgroups per query
    A.n_seg = 0;
    A.seg_cnt = W.seg_cnt;
    if (P.N > SEL_PREFILTER_MIN) {
        int n_seg = 512 / P.nq;      // about two workgroups per CU in total
        n_seg = n_seg < 2 ? 2 : (n_seg > SEG_MAX ? SEG_MAX : n_seg);
        A.n_seg = n_seg;
        k_select_segments<<<dim3(n_seg, P.nq), SEL_THREADS, 0, st>>>(A);
    }
    k_select_prune<<<P.nq, SEL_THREADS, 0, st>>>(A);
    return hipGetLastError();
}

// =====================================================================================
// top-K by (value descending, document index ascending), one workgroup per query
// (Eq. (3); final step of Algorithm 1).  Candidates arrive in ascending id order, so
// ties at the K-th value are resolved towards the lower index by taking them in order.
// =====================================================================================
struct TopkArgs {
    const QueryCtl* ctl;   // nullptr: all N documents, vals indexed by id
    int32_t* list0;        // the list that is not the query's current one doubles as scratch
    int32_t* list1;        // for candidate positions of long inputs
    const int32_t* cid;
    int cache_cap;
    const float* vals;     // [nq][N]
    int64_t N;
    int K;
    int64_t* out_ids;
    float* out_scores;
    int n_seg;             // > 0: k_topk_segments has pre-filtered the positions (ctl == nullptr)
    int32_t* seg_cnt;      // [nq][SEG_MAX]
};

// The pre-filter of k_topk for all-documents inputs, spread over n_seg workgroups per query:
// same sample threshold in every workgroup, one streaming pass over the workgroup's segment,
// candidate positions in order at the segment's start of the scratch list.
__global__ __launch_bounds__(SEL_THREADS) void k_topk_segments(TopkArgs A) {
    __shared__ uint32_t hist[2048];
    __shared__ int pick[2];
    __shared__ int wtot[SEL_WAVES];
    const int q = blockIdx.y, sg = blockIdx.x;
    const int count = (int)A.N;
    if (count <= SEL_PREFILTER_MIN) return;
    const float* vals = A.vals + (size_t)q * A.N;
    int32_t* tmp = A.list0 + (size_t)q * A.N;
    const int Kq = A.K < count ? A.K : count;
    auto key_s = [&](int j) -> uint32_t { return float_key(vals[sample_pos(j, count)]); };
    const uint32_t lo_key = block_kth_largest_sample(Kq, key_s, hist, pick);
    const int len = seg_len(count, A.n_seg);
    const int lo = sg * len;
    const int hi = lo + len < count ? lo + len : count;
    constexpr int ITEMS = SEL_ITEMS_WIDE;
    constexpr int CHUNK = SEL_THREADS * ITEMS;
    const int t0 = threadIdx.x * ITEMS;
    int base = 0;
    float v[ITEMS];
#pragma unroll
    for (int u = 0; u < ITEMS; ++u) v[u] = lo + t0 + u < hi ? vals[lo + t0 + u] : 0.f;
    for (int start = lo; start < hi; start += CHUNK) {
        const int i0 = start + t0;
        float v_next[ITEMS];
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) v_next[u] = i0 + CHUNK + u < hi ? vals[i0 + CHUNK + u] : 0.f;
        unsigned keep = 0;
#pragma unroll
        for (int u = 0; u < ITEMS; ++u)
            if (i0 + u < hi && float_key(v[u]) >= lo_key) keep |= 1u << u;
#pragma unroll
        for (int u = 0; u < ITEMS; ++u) v[u] = v_next[u];
        if (__syncthreads_or(keep != 0)) {
            int total;
            int pos = lo + base + block_excl_scan(__popc(keep), wtot, total);
#pragma unroll
            for (int u = 0; u < ITEMS; ++u)
                if (keep & (1u << u)) tmp[pos++] = i0 + u;
            base += total;
        }
    }
    if (threadIdx.x == 0) A.seg_cnt[(size_t)q * SEG_MAX + sg] = base;
}

__global__ __launch_bounds__(SEL_THREADS) void k_topk(TopkArgs A) {
    __shared__ uint32_t hist[2048];
    __shared__ int pick[2];
    __shared__ int wtot[SEL_WAVES];
    __shared__ float cs[1024];
    __shared__ int ci[1024];
    const int q = blockIdx.x;
    int count = (int)A.N;
    const int32_t* list = nullptr;
    const int32_t* cid = nullptr;
    int32_t* scratch = A.list0 + (size_t)q * A.N;
    if (A.ctl) {
        const QueryCtl c = A.ctl[q];
        count = c.count;
        if (!c.implicit) {
            list = (c.cur ? A.list1 : A.list0) + (size_t)q * A.N;
            scratch = (c.cur ? A.list0 : A.list1) + (size_t)q * A.N;
        }
        if (c.mode == 1) cid = A.cid + (size_t)q * A.cache_cap;
    }
    const float* vals = A.vals + (size_t)q * A.N;
    const int Kq = A.K < count ? A.K : count;
    if (Kq > 0) {
        // candidate positions: all of 0..count-1, or (long inputs) those whose value reaches
        // the K-th largest value of a strided sample, which cannot exceed the true K-th
        const int32_t* cand = nullptr;
        int ncand = count;
        if (A.n_seg > 0 && !A.ctl && count > SEL_PREFILTER_MIN) {
            ncand = merge_segments(scratch, A.seg_cnt + (size_t)q * SEG_MAX, count, A.n_seg);
            cand = scratch;
        } else if (count > SEL_PREFILTER_MIN) {
            int32_t* tmp = scratch;
            auto key_s = [&](int j) -> uint32_t { return float_key(vals[sample_pos(j, count)]); };
            const uint32_t lo = block_kth_largest_sample(Kq, key_s, hist, pick);
            int base = 0;
            const int t0 = threadIdx.x * SEL_ITEMS_WIDE;
            float v[SEL_ITEMS_WIDE];                       // the next chunk's values are fetched
#pragma unroll                                        // before this chunk's barriers
            for (int u = 0; u < SEL_ITEMS_WIDE; ++u) v[u] = t0 + u < count ? vals[t0 + u] : 0.f;
            for (int start = 0; start < count; start += (SEL_THREADS * SEL_ITEMS_WIDE)) {
                const int i0 = start + t0;
                float v_next[SEL_ITEMS_WIDE];
#pragma unroll
                for (int u = 0; u < SEL_ITEMS_WIDE; ++u)
                    v_next[u] = i0 + (SEL_THREADS * SEL_ITEMS_WIDE) + u < count ? vals[i0 + (SEL_THREADS * SEL_ITEMS_WIDE) + u] : 0.f;
                unsigned keep = 0;
#pragma unroll
                for (int u = 0; u < SEL_ITEMS_WIDE; ++u)
                    if (i0 + u < count && float_key(v[u]) >= lo) keep |= 1u << u;
#pragma unroll
                for (int u = 0; u < SEL_ITEMS_WIDE; ++u) v[u] = v_next[u];
                if (__syncthreads_or(keep != 0)) {
                    int total;
                    int pos = base + block_excl_scan(__popc(keep), wtot, total);
#pragma unroll
                    for (int u = 0; u < SEL_ITEMS_WIDE; ++u)
                        if (keep & (1u << u)) tmp[pos++] = i0 + u;
                    base += total;
                }
            }
            __syncthreads();
            cand = tmp;
            ncand = base;
        }
        auto key_of = [&](int j) -> uint32_t { return float_key(vals[cand ? cand[j] : j]); };
        const uint32_t tkey = block_kth_largest(ncand, Kq, key_of, hist, pick);
        // how many are strictly above the K-th value
        int gt_local = 0;
        for (int j = threadIdx.x; j < ncand; j += SEL_THREADS) gt_local += key_of(j) > tkey;
        int n_gt;
        block_excl_scan(gt_local, wtot, n_gt);
        const int need_eq = Kq - n_gt;
        int base_gt = 0, base_eq = 0;
        for (int start = 0; start < ncand; start += SEL_CHUNK) {
            const int i0 = start + threadIdx.x * SEL_ITEMS;
            float v[SEL_ITEMS];
            int p[SEL_ITEMS];
            unsigned gt = 0, eq = 0;
#pragma unroll
            for (int u = 0; u < SEL_ITEMS; ++u) {
                p[u] = (i0 + u < ncand) ? (cand ? cand[i0 + u] : i0 + u) : 0;
                v[u] = (i0 + u < ncand) ? vals[p[u]] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < SEL_ITEMS; ++u) {
                if (i0 + u < ncand) {
                    const uint32_t key = float_key(v[u]);
                    gt |= (key > tkey ? 1u : 0u) << u;
                    eq |= (key == tkey ? 1u : 0u) << u;
                }
            }
            if (__syncthreads_or((gt | eq) != 0)) {      // most chunks hold no winner
                int tot;
                const int pos = block_excl_scan(__popc(gt) | (__popc(eq) << 16), wtot, tot);
                int pg = base_gt + (pos & 0xffff), pe = base_eq + (pos >> 16);
#pragma unroll
                for (int u = 0; u < SEL_ITEMS; ++u) {
                    int slot = -1;
                    if (gt & (1u << u)) slot = pg++;
                    else if (eq & (1u << u)) {
                        if (pe < need_eq) slot = n_gt + pe;
                        ++pe;
                    }
                    if (slot >= 0) {
                        const int e = list ? list[p[u]] : p[u];
                        cs[slot] = v[u];
                        ci[slot] = cid ? cid[e] : e;
                    }
                }
                base_gt += tot & 0xffff;
                base_eq += tot >> 16;
            }
        }
        __syncthreads();
        if (threadIdx.x < Kq) {
            const float v = cs[threadIdx.x];
            const int id = ci[threadIdx.x];
            int rank = 0;
            for (int j = 0; j < Kq; ++j) {
                const float u = cs[j];
                rank += (u > v) || (u == v && ci[j] < id);
            }
            A.out_ids[(size_t)q * A.K + rank] = id;
            A.out_scores[(size_t)q * A.K + rank] = v;
        }
    }
    for (int k = Kq + threadIdx.x; k < A.K; k += SEL_THREADS) {
        A.out_ids[(size_t)q * A.K + k] = -1;
        A.out_scores[(size_t)q * A.K + k] = -__builtin_inff();
    }
}

hipError_t launch_topk(const Problem& P, const Work& W, bool use_ctl, const float* vals, int K,
                       int64_t* out_ids, float* out_scores, hipStream_t st) {
    TopkArgs A{};
    A.ctl = use_ctl ? W.ctl : nullptr;
    A.list0 = W.list[0];
    A.list1 = W.list[1];
    A.cid = W.cid;
    A.cache_cap = W.cache_cap;
    A.vals = vals;
    A.N = P.N;
    A.K = K;
    A.out_ids = out_ids;
    A.out_scores = out_scores;
    A.n_seg = 0;
    A.seg_cnt = W.seg_cnt;
    if (!use_ctl && P.N > SEL_PREFILTER_MIN) {
        int n_seg = 512 / P.nq;
        n_seg = n_seg < 2 ? 2 : (n_seg > SEG_MAX ? SEG_MAX : n_seg);
        A.n_seg = n_seg;
        k_topk_segments<<<dim3(n_seg, P.nq), SEL_THREADS, 0, st>>>(A);
    }
    k_topk<<<P.nq, SEL_THREADS, 0, st>>>(A);
    return hipGetLastError();
}

// =====================================================================================
// offsets validation
// =====================================================================================
__global__ void k_validate_offsets(const int64_t* off, int64_t N, int64_t total, int* flag) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (int64_t)gridDim.x * blockDim.x) {
        bool bad = off[i + 1] <= off[i];
        if (i == 0) bad = bad || off[0] < 0 || off[N] > total;
        if (bad) atomicOr(flag, 1);
    }
}
__global__ void k_zero_flag(int* flag) { flag[0] = 0; }

hipError_t launch_validate_offsets(const int64_t* off, int64_t N, int64_t total, int* flag,
                                   hipStream_t st) {
    k_zero_flag<<<1, 1, 0, st>>>(flag);
    int g = (int)((N + 255) / 256);
    if (g > 2048) g = 2048;
    k_validate_offsets<<<g, 256, 0, st>>>(off, N, total, flag);
    return hipGetLastError();
}

}  // namespace cb
