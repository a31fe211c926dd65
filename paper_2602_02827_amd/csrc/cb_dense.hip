// Dense corpus-streaming MaxSim kernel for bf16 (gfx950).
//
// Shape of the work: a [tokens x d] corpus against a few thousand query rows, d = 64/128.
// The result matrix is never written; each 16x16 MFMA tile is folded at once into a
// running per-(document, query row) maximum, and a document's maxima are summed when
// its last token has passed (paper Eq. (1)-(2), (4)-(5)).
//
// Mapping onto the machine
//   * A workgroup (4 wavefronts) owns one token chunk (whole documents whose first token
//     falls into a fixed-size token range) and one group of 64*NT query columns.
//   * Query rows are the B operand and stay in registers for the whole kernel: each
//     wavefront holds NT column tiles of 16 rows, full depth (NT*d/8 VGPRs).
//   * Document tokens are the A operand.  They stream through a four-slot LDS ring of
//     64-token stages (global -> registers -> LDS, two stages ahead of the reader), so a
//     token is read from memory once per workgroup and from LDS once per wavefront.
//     Rows are stored with their 16-byte pieces XOR-swizzled by the row index, which
//     spreads the 16 rows of an operand block over all banks.
//   * Blocks of 16 tokens are aligned to the start of each document; a short last block
//     re-reads the document's last token (duplicates do not change a max), so the
//     epilogue needs no masking and documents of any length >= 1 are handled.
//   * Workgroup ids are laid out so that the column groups of one token chunk run on the
//     same XCD and share its L2.
#include "cb_launch.h"

namespace cb {

constexpr int DENSE_THREADS = 256;
constexpr int STAGE_ROWS = 64;
constexpr int RING_ROWS = 256;   // 4 stages

struct DenseArgs {
    const void* Q;
    const void* docs;
    const int64_t* off;
    const int32_t* chunk_doc;
    int64_t N, total;
    int nq, T;
    int n_chunks, n_groups;
    // score
    float* out;
    float* cells;
    // reveal
    const int32_t* pi;
    int lo, nb, G;
    float2* stat;
};

template <int D, int NT, int TQ, bool REVEAL>
__global__ __launch_bounds__(DENSE_THREADS, 2) void k_dense(DenseArgs A) {
    using F = Frag<bf16_tag, D>;
    constexpr int ROWB = D * 2;            // bytes per token row
    constexpr int NCH = ROWB / 16;         // 16-byte pieces per row
    constexpr int LD_PER_THREAD = STAGE_ROWS * NCH / DENSE_THREADS;
    __shared__ __attribute__((aligned(16))) char ring[RING_ROWS * ROWB];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 15;
    const int kg = lane >> 4;

    // workgroup -> (token chunk, column group); chunks of one XCD are contiguous in `slot`
    const int b = blockIdx.x;
    const int xcd = b & 7, slot = b >> 3;
    const int group = slot % A.n_groups;
    const int chunk = (slot / A.n_groups) * 8 + xcd;
    if (chunk >= A.n_chunks) return;
    int i0 = A.chunk_doc[chunk], i1 = A.chunk_doc[chunk + 1];
    i0 = i0 < 0 ? 0 : (i0 > (int)A.N ? (int)A.N : i0);
    i1 = i1 < i0 ? i0 : (i1 > (int)A.N ? (int)A.N : i1);
    if (i0 >= i1) return;
    int64_t tok_begin = A.off[i0], tok_end = A.off[i1];
    tok_begin = tok_begin < 0 ? 0 : (tok_begin > A.total ? A.total : tok_begin);
    tok_end = tok_end < tok_begin ? tok_begin : (tok_end > A.total ? A.total : tok_end);
    const int ntok = (int)(tok_end - tok_begin);
    if (ntok <= 0) return;

    // ---- query rows of this wavefront's column tiles -> B fragments (registers)
    const int tile0 = (group * 4 + wave) * NT;
    F bq[NT];
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
        const int g = tile0 + tt;
        int q, trow;
        if (REVEAL) {
            const int x = g * 16 + col;
            q = x / A.G;
            const int sl = x % A.G;
            q = q < A.nq ? q : 0;
            trow = A.pi[(size_t)q * A.T + A.lo + (sl < A.nb ? sl : 0)];
        } else {
            q = g / TQ;
            const int t = (g % TQ) * 16 + col;
            q = q < A.nq ? q : 0;
            trow = t < A.T ? t : 0;
        }
        bq[tt].load((const char*)A.Q + ((size_t)q * A.T + trow) * ROWB, kg);
    }

    // ---- stage loader: 64 rows x ROWB bytes, 16 bytes per thread per step
    const char* src = (const char*)A.docs + (size_t)tok_begin * ROWB;
    u32x4_t stage_regs[LD_PER_THREAD];
    auto stage_fetch = [&](int s) {
#pragma unroll
        for (int i = 0; i < LD_PER_THREAD; ++i) {
            const int x = i * DENSE_THREADS + threadIdx.x;
            int row = s * STAGE_ROWS + x / NCH;
            row = row < ntok ? row : ntok - 1;      // past the end: re-read the last row (never used)
            stage_regs[i] = *(const u32x4_t*)(src + (size_t)row * ROWB + (x % NCH) * 16);
        }
    };
    auto stage_commit = [&](int s) {
#pragma unroll
        for (int i = 0; i < LD_PER_THREAD; ++i) {
            const int x = i * DENSE_THREADS + threadIdx.x;
            const int row = s * STAGE_ROWS + x / NCH;
            const int ch = x % NCH;
            if (row < ntok)
                *(u32x4_t*)(ring + (row & (RING_ROWS - 1)) * ROWB + ((ch ^ (row & (NCH - 1))) * 16)) =
                    stage_regs[i];
        }
    };

    // ---- document walk state (identical in all four wavefronts)
    int ibase = i0;
    auto fetch_offs = [&](int base) -> int {
        int j = base + lane;
        j = j > i1 ? i1 : j;
        int64_t o = A.off[j] - tok_begin;
        o = o < 0 ? 0 : (o > ntok ? ntok : o);
        return (int)o;
    };
    int offv = fetch_offs(ibase);
    auto rel_off = [&](int i) -> int {
        if (i - ibase >= 64) {
            ibase = i;
            offv = fetch_offs(ibase);
        }
        return __builtin_amdgcn_readlane(offv, i - ibase);
    };

    float h[NT];
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) h[tt] = -__builtin_inff();

    // per-document epilogue: cross-lane maxima, then the row sum (score) or the batch
    // statistics (reveal), written by the lanes that own a query
    auto finalize = [&](int doc) {
        if constexpr (REVEAL) {
            using P = Pack<NT>;
            float w[P::NW];
            P::colmax(h, w);
            const int row = lane >> 4;
#pragma unroll
            for (int j = 0; j < P::NW; ++j) {
                const int x = (tile0 + P::tile_of_row(j, row)) * 16 + col;
                const int q = x / A.G, sl = x % A.G;
                float sb, m2b;
                batch_stats(w[j], sl, A.nb, A.G, sb, m2b);
                if (sl == 0 && q < A.nq && P::row_is_primary(row))
                    A.stat[(size_t)q * A.N + doc] = make_float2(sb, m2b);
            }
        } else {
            using SC = Score<NT, TQ>;
            float w[SC::NW], sc[SC::NS];
            SC::run(h, A.T, col, w, sc);
#pragma unroll
            for (int j = 0; j < SC::NS; ++j) {
                const int lq = SC::writer(j, lane);
                const int q = tile0 / TQ + lq;
                if (lq >= 0 && q < A.nq) A.out[(size_t)q * A.N + doc] = sc[j];
            }
            if (A.cells) {
                const int row = lane >> 4;
#pragma unroll
                for (int j = 0; j < SC::NW; ++j) {
                    const int g = tile0 + Pack<NT>::tile_of_row(j, row);
                    const int q = g / TQ, t = (g % TQ) * 16 + col;
                    if (Pack<NT>::row_is_primary(row) && q < A.nq && t < A.T)
                        A.cells[((size_t)q * A.N + doc) * A.T + t] = w[j];
                }
            }
        }
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) h[tt] = -__builtin_inff();
    };

    // one block of 16 tokens against all NT column tiles
    auto compute = [&](const F& a) {
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
            F::mma(acc, a, bq[tt]);
            h[tt] = fold_max(h[tt], acc);
        }
    };
    // A fragment of the block whose lane row sits at ring byte offset `ro`; `co` are the
    // lane's swizzled piece offsets
    auto load_a = [&](F& a, int ro, const int (&co)[F::KS]) {
#pragma unroll
        for (int ks = 0; ks < F::KS; ++ks) a.v[ks] = *(const bf16x8_t*)(ring + ro + co[ks]);
    };
    constexpr int RING_BYTES = RING_ROWS * ROWB;
    constexpr int BLOCK_BYTES = 16 * ROWB;

    const int nst = (ntok + STAGE_ROWS - 1) / STAGE_ROWS;
    stage_fetch(0);
    stage_commit(0);
    if (nst > 1) {
        stage_fetch(1);
        stage_commit(1);
    }
    __syncthreads();

    int doc = i0 - 1;      // current document; its tokens are [.., dend) relative to tok_begin
    int dend = 0, cur = 0;
    bool started = false, finished = false;

#pragma unroll 1
    for (int s = 0; s < nst; ++s) {
        const bool more = s + 2 < nst;
        if (more) stage_fetch(s + 2);
        const int avail = (s == nst - 1) ? ntok : (s + 1) * STAGE_ROWS;
        while (!finished) {
            if (cur >= dend) {
                if (started) finalize(doc);
                ++doc;
                if (doc >= i1) {
                    finished = true;
                    break;
                }
                started = true;
                cur = dend;
                dend = rel_off(doc + 1);
                continue;
            }
            // blocks of this document that are complete in the ring: n full ones, and the
            // short last one if the document ends inside what has arrived
            const int lim = dend < avail ? dend : avail;
            int n = (lim - cur) >> 4;
            const bool tail = dend <= avail && ((dend - cur) & 15) != 0;
            if (n == 0 && !tail) break;
            const int row0 = cur + col;
            const int sw = row0 & (NCH - 1);          // blocks step by 16 rows: sw is invariant
            int co[F::KS];
#pragma unroll
            for (int ks = 0; ks < F::KS; ++ks) co[ks] = ((ks * 4 + kg) ^ sw) * 16;
            int ro = (row0 & (RING_ROWS - 1)) * ROWB;
            cur += n * 16;
            if (n > 0) {
                F a0, a1;
                load_a(a0, ro, co);
                while (n >= 2) {                       // two blocks per trip, loads one ahead
                    load_a(a1, (ro + BLOCK_BYTES) & (RING_BYTES - 1), co);
                    compute(a0);
                    ro = (ro + 2 * BLOCK_BYTES) & (RING_BYTES - 1);
                    if (n > 2) load_a(a0, ro, co);
                    compute(a1);
                    n -= 2;
                }
                if (n == 1) compute(a0);
            }
            if (tail) {                                // rows past the end repeat the last token
                int row = cur + col;
                row = row < dend ? row : dend - 1;
                const int swt = row & (NCH - 1);
                const int rot = (row & (RING_ROWS - 1)) * ROWB;
                F a;
#pragma unroll
                for (int ks = 0; ks < F::KS; ++ks)
                    a.v[ks] = *(const bf16x8_t*)(ring + rot + (((ks * 4 + kg) ^ swt) * 16));
                compute(a);
                cur = dend;
            }
        }
        if (more) stage_commit(s + 2);
        __syncthreads();
    }
}

// ---- first document of every token chunk: chunk_doc[c] = min{ i : off[i] >= c*C }
__global__ void k_chunk_docs(const int64_t* off, int64_t N, int C, int n_chunks, int32_t* chunk_doc) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i > N) return;
    int64_t lo = (i == 0) ? 0 : off[i - 1] / C + 1;
    int64_t hi = off[i] / C;
    if (off[i] < 0) hi = -1;
    if (i > 0 && off[i - 1] < 0) lo = 0;
    if (i == N) hi = n_chunks;       // everything past the last offset is empty
    lo = lo < 0 ? 0 : lo;
    hi = hi > n_chunks ? n_chunks : hi;
    for (int64_t c = lo; c <= hi; ++c) chunk_doc[c] = (int32_t)i;
}

bool dense_supported(const Problem& P) {
    return P.dt == DT_BF16 && (P.d == 64 || P.d == 128) && P.total / 4096 < 0x7fffff00;
}

hipError_t launch_dense_prepare(const Problem& P, const Work& W, int C, int* n_chunks,
                                hipStream_t st) {
    const int nc = (int)((P.total + C - 1) / C);
    *n_chunks = nc;
    const int64_t n = P.N + 1;
    k_chunk_docs<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(P.off, P.N, C, nc, W.chunk_doc);
    return hipGetLastError();
}

static void fill_dense(DenseArgs& A, const Problem& P, const Work& W, int n_chunks) {
    A.Q = P.Q;
    A.docs = P.docs;
    A.off = P.off;
    A.chunk_doc = W.chunk_doc;
    A.N = P.N;
    A.total = P.total;
    A.nq = P.nq;
    A.T = P.T;
    A.n_chunks = n_chunks;
    A.pi = W.pi;
    A.stat = W.stat;
}

template <int D, int NT, int TQ, bool REVEAL>
static hipError_t dense_go(DenseArgs& A, int tiles, hipStream_t st) {
    A.n_groups = (tiles + 4 * NT - 1) / (4 * NT);
    const int chunks8 = (A.n_chunks + 7) / 8 * 8;
    const long long blocks = (long long)chunks8 * A.n_groups;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    k_dense<D, NT, TQ, REVEAL><<<(unsigned)blocks, DENSE_THREADS, 0, st>>>(A);
    return hipGetLastError();
}

template <int D, int TQ>
static hipError_t dense_score_nt(DenseArgs& A, int tiles, hipStream_t st) {
    if constexpr (TQ <= 2) {
        if (tiles <= 8) return dense_go<D, 2, TQ, false>(A, tiles, st);
    }
    if constexpr (TQ <= 4) {
        if (tiles <= 16) return dense_go<D, 4, TQ, false>(A, tiles, st);
    }
    return dense_go<D, 8, TQ, false>(A, tiles, st);
}

template <int D>
static hipError_t dense_score_d(DenseArgs& A, hipStream_t st) {
    const int tq = (A.T + 15) / 16;
    if (tq <= 1) return dense_score_nt<D, 1>(A, A.nq * 1, st);
    if (tq <= 2) return dense_score_nt<D, 2>(A, A.nq * 2, st);
    if (tq <= 4) return dense_score_nt<D, 4>(A, A.nq * 4, st);
    return dense_score_nt<D, 8>(A, A.nq * 8, st);
}

hipError_t launch_dense_score(const Problem& P, const Work& W, int C, int n_chunks, float* out,
                              float* cells, hipStream_t st) {
    (void)C;
    DenseArgs A{};
    fill_dense(A, P, W, n_chunks);
    A.out = out;
    A.cells = cells;
    return P.d == 128 ? dense_score_d<128>(A, st) : dense_score_d<64>(A, st);
}

template <int D>
static hipError_t dense_reveal_d(DenseArgs& A, hipStream_t st) {
    const int tiles = (A.nq * A.G + 15) / 16;
    if (tiles <= 4) return dense_go<D, 1, 1, true>(A, tiles, st);
    if (tiles <= 8) return dense_go<D, 2, 1, true>(A, tiles, st);
    if (tiles <= 16) return dense_go<D, 4, 1, true>(A, tiles, st);
    return dense_go<D, 8, 1, true>(A, tiles, st);
}

hipError_t launch_dense_reveal(const Problem& P, const Work& W, int C, int n_chunks,
                               const RevealRound& rr, int G, hipStream_t st) {
    (void)C;
    DenseArgs A{};
    fill_dense(A, P, W, n_chunks);
    A.lo = rr.lo;
    A.nb = rr.nb;
    A.G = G;
    return P.d == 128 ? dense_reveal_d<128>(A, st) : dense_reveal_d<64>(A, st);
}

}  // namespace cb
