// Dense corpus-streaming MaxSim kernel for bf16 embeddings and int8 codes (gfx950).
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
//     64-token stages (direct global -> LDS copies issued two stages ahead of the reader), so
//     a token is read from memory once per workgroup and from LDS once per wavefront.
//     Rows are stored with their 16-byte pieces XOR-swizzled by the row index, which
//     spreads the 16 rows of an operand block over all banks.
//   * The chunk's tokens form one stream of aligned 16-token blocks, whatever the document
//     boundaries, so no token is multiplied twice.  A block inside one document folds into
//     the running maxima directly; where a document ends inside a block the fold is split
//     by accumulator row (block_mma_split_rows / block_mma_split).  Documents of any length
//     >= 1 are handled.  Runs of whole blocks inside one document go through a loop that holds
//     only operand reads and MFMAs.
//   * Workgroup ids are laid out so that the column groups of one token chunk run on the
//     same XCD and share its L2; eight consecutive chunks go to the eight XCDs in a rotating
//     order.
#include "cb_launch.h"

namespace cb {

constexpr int DENSE_THREADS = 256;
// Ring geometry: four stages.  Kernels with few column tiles per wavefront (small query
// batches: bound by memory, little register use) take 32-row stages, so that four workgroups fit
// a CU instead of two and more wavefronts hide the latencies; the others take 64-row stages.
template <int NT, int ROWB> struct RingShape {
    static constexpr int ROWS_PER_LOAD = 64 / (ROWB / 16);
    static constexpr bool SMALL = NT <= 4 && 32 / ROWS_PER_LOAD / 4 >= 1;
    static constexpr int STAGE_ROWS = SMALL ? 32 : 64;
    static constexpr int RING_ROWS = 4 * STAGE_ROWS;
    static constexpr int MIN_BLOCKS = SMALL ? (NT <= 2 ? 4 : 3) : 2;
};

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
    // a round >= 2: run only if dense_round(pairs_r, dense_thr); skip queries that are
    // finished or read their cells from the cache
    const unsigned long long* pairs_r;
    unsigned long long dense_thr;
    const QueryCtl* ctl;
    // int8 codes: a cell is the integer maximum times qscale[q] * dscale[0]
    const float* qscale;
    const float* dscale;
};

template <typename Tag, int D, int NT, int TQ, bool REVEAL, int SPLIT_DOCS = 0>
__global__ __launch_bounds__(DENSE_THREADS, (RingShape<NT, D * Frag<Tag, D>::ELEM_BYTES>::MIN_BLOCKS))
void k_dense(DenseArgs A) {
    using F = Frag<Tag, D>;
    using RS = RingShape<NT, D * F::ELEM_BYTES>;
    constexpr int STAGE_ROWS = RS::STAGE_ROWS;
    constexpr int RING_ROWS = RS::RING_ROWS;
    using V = typename F::val_t;           // float, or int for int8 codes
    constexpr bool CODES = !__is_same(V, float);
    constexpr int ROWB = D * F::ELEM_BYTES;   // bytes per token row
    constexpr int NCH = ROWB / 16;         // 16-byte pieces per row
    // Cache policy of the token copies.  The reveal pass normally has one column group, and the
    // score kernels with at most four column tiles per wavefront always have: a token row is read
    // once and should not push other lines out of L2 - above all those of the (sum, M2) array,
    // which fill up over several documents; such copies carry the non-temporal hint (bit 1).
    constexpr int LOAD_POLICY = (REVEAL || NT <= 4) ? 2 : 0;
    // Swizzle key of a ring row: rows whose 16-byte pieces would fall on the same banks
    // (row stride ROWB against the 256-byte bank window) get different keys.
    constexpr int KEY_SHIFT = NCH >= 16 ? 0 : (NCH == 8 ? 1 : 2);
    __shared__ __attribute__((aligned(16))) char ring[RING_ROWS * ROWB];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, in an SGPR
    const int col = lane & 15;
    const int kg = lane >> 4;

    // workgroup -> (token chunk, column group); chunks of one XCD are contiguous in `slot`
    const int b = blockIdx.x;
    const int xcd = b & 7, slot = b >> 3;
    const int group = slot % A.n_groups;
    // Eight consecutive chunks go to the eight XCDs, rotated from one eight to the next by a
    // mix of its number: documents much longer than a chunk leave all but every 2^k-th chunk
    // empty, and a fixed chunk -> XCD map would then put all the work on a few XCDs.
    const int k8 = slot / A.n_groups;
    const int chunk = k8 * 8 + ((xcd + k8 + (k8 >> 3) + (k8 >> 6) + (k8 >> 9)) & 7);
    if (chunk >= A.n_chunks) return;
    if constexpr (REVEAL) {
        if (A.pairs_r && !dense_round(A.pairs_r, A.dense_thr)) return;
    }
    int i0 = A.chunk_doc[chunk], i1 = A.chunk_doc[chunk + 1];
    i0 = i0 < 0 ? 0 : (i0 > (int)A.N ? (int)A.N : i0);
    i1 = i1 < i0 ? i0 : (i1 > (int)A.N ? (int)A.N : i1);
    if (i0 >= i1) return;
    int64_t tok_begin = A.off[i0], tok_end = A.off[i1];
    tok_begin = tok_begin < 0 ? 0 : (tok_begin > A.total ? A.total : tok_begin);
    tok_end = tok_end < tok_begin ? tok_begin : (tok_end > A.total ? A.total : tok_end);
    const int ntok = (int)(tok_end - tok_begin);
    if (ntok <= 0) return;

    const int lgG = REVEAL ? 31 - __builtin_clz(A.G > 0 ? A.G : 1) : 0;   // G is a power of two
    // ---- query rows of this wavefront's column tiles -> B fragments (registers)
    // When the column tiles of the launch fit into one or two of the four wavefronts (one or two
    // queries), the others would only repeat their work.  Instead SPLIT_DOCS (4 or 2) wavefronts
    // take the same tiles and split the chunk's DOCUMENTS among themselves: a wavefront
    // multiplies the blocks inside its own documents (every fourth, or every second) and every
    // block in which a document ends, and writes the scores of its own documents only.  All four
    // still walk the same block stream, so the stage barriers match up.  (SPLIT_DOCS: the launch
    // has one column group.)
    static_assert(SPLIT_DOCS == 0 || ((SPLIT_DOCS == 2 || SPLIT_DOCS == 4) && !REVEAL && NT <= 2),
                  "document splitting is for the smallest score kernels");
    constexpr int TILE_WAVES = SPLIT_DOCS ? 4 / SPLIT_DOCS : 4;      // wavefronts with tiles of their own
    const int tile0 = SPLIT_DOCS ? (wave % TILE_WAVES) * NT : (group * 4 + wave) * NT;
    auto mine = [&](int doc) {
        return SPLIT_DOCS == 0 || ((doc - i0) & (SPLIT_DOCS ? SPLIT_DOCS - 1 : 0)) == wave / TILE_WAVES;
    };
    F bq[NT];
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
        const int g = tile0 + tt;
        int q, trow;
        if (REVEAL) {
            const int x = g * 16 + col;
            q = x >> lgG;
            const int sl = x & (A.G - 1);
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

    // ---- stage loader: 64 rows x ROWB bytes, copied global -> LDS without passing through
    // registers (global_load_lds_dwordx4: every lane names its 16 global bytes, the wavefront's
    // 64 pieces land in 1 KB of consecutive LDS).  One instruction fills 64/NCH ring rows; the
    // lane at physical piece position p of LDS row r fetches the logical piece p ^ (r & (NCH-1)).
    const char* src = (const char*)A.docs + (size_t)tok_begin * ROWB;
    constexpr int ROWS_PER_LOAD = 64 / NCH;
    constexpr int LOADS_PER_WAVE = STAGE_ROWS / ROWS_PER_LOAD / 4;
    // A lane's place inside a load does not depend on the stage or on the load's number (both
    // move the row by multiples of the swizzle period): row wave*ROWS_PER_LOAD + lane/NCH of the
    // load group, piece (lane % NCH) ^ key(row).  A complete stage therefore needs no per-lane
    // address arithmetic at all: uniform base + this constant offset.
    const int lrow0 = wave * ROWS_PER_LOAD + lane / NCH;
    const unsigned fetch_off =
        (unsigned)(lrow0 * ROWB + (((lane & (NCH - 1)) ^ ((lrow0 >> KEY_SHIFT) & (NCH - 1))) * 16));
    auto stage_fetch = [&](int s) {
        if ((s + 1) * STAGE_ROWS <= ntok) {
#pragma unroll
            for (int i = 0; i < LOADS_PER_WAVE; ++i) {
                const int r0 = s * STAGE_ROWS + i * 4 * ROWS_PER_LOAD;               // uniform
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(src + (size_t)r0 * ROWB + fetch_off),
                    (__attribute__((address_space(3))) void*)(ring + ((r0 + wave * ROWS_PER_LOAD) & (RING_ROWS - 1)) * ROWB),
                    16, 0, LOAD_POLICY);
            }
            return;
        }
        // the chunk's last, incomplete stage: rows past the end are clamped (they are never read)
#pragma unroll
        for (int i = 0; i < LOADS_PER_WAVE; ++i) {
            const int rbase = s * STAGE_ROWS + (i * 4 + wave) * ROWS_PER_LOAD;   // wave-uniform
            if (rbase < ntok) {
                const int lrow = rbase + lane / NCH;                  // the LDS row this lane fills
                const int grow = lrow < ntok ? lrow : ntok - 1;
                const int c = (lane & (NCH - 1)) ^ ((lrow >> KEY_SHIFT) & (NCH - 1));
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(src + (size_t)grow * ROWB + c * 16),
                    (__attribute__((address_space(3))) void*)(ring + (rbase & (RING_ROWS - 1)) * ROWB),
                    16, 0, LOAD_POLICY);
            }
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

    V h[NT];
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) h[tt] = lowest_val<V>();

    // int8 codes: decode scale of the query behind each of this lane's packed results
    float cscale[Pack<NT>::NW];
    if constexpr (CODES) {
        const float ds = A.dscale[0];
#pragma unroll
        for (int j = 0; j < Pack<NT>::NW; ++j) {
            const int g = tile0 + Pack<NT>::tile_of_row(j, lane >> 4);
            int q = REVEAL ? (g * 16 + col) >> lgG : g / TQ;
            q = q < A.nq ? q : 0;
            cscale[j] = A.qscale[q] * ds;
        }
    }

    // reveal: which of this lane's result registers belong to a query that takes the batch
    unsigned qmask = ~0u;
    if constexpr (REVEAL) {
        if (A.ctl) {
            using P = Pack<NT>;
            qmask = 0u;
#pragma unroll
            for (int j = 0; j < P::NW; ++j) {
                const int x = (tile0 + P::tile_of_row(j, lane >> 4)) * 16 + col;
                const int q = x >> lgG;
                if (q < A.nq) {
                    const QueryCtl c = A.ctl[q];
                    if (c.active && c.mode == 0) qmask |= 1u << j;
                }
            }
        }
    }

    // per-document epilogue: cross-lane maxima, then the row sum (score) or the batch
    // statistics (reveal), written by the lanes that own a query
    auto finalize = [&](int doc) {
        using P = Pack<NT>;
        if (!mine(doc)) {                       // another wavefront's document: nothing to write
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) h[tt] = lowest_val<V>();
            return;
        }
        // cross-lane column maxima, decoded to float cells
        float w[P::NW];
        if constexpr (CODES) {
            V wi[P::NW];
            P::colmax(h, wi);
#pragma unroll
            for (int j = 0; j < P::NW; ++j) w[j] = (float)wi[j] * cscale[j];
        } else {
            P::colmax(h, w);
        }
        if constexpr (REVEAL) {
            const int row = lane >> 4;
#pragma unroll
            for (int j = 0; j < P::NW; ++j) {
                const int x = (tile0 + P::tile_of_row(j, row)) * 16 + col;
                const int q = x >> lgG, sl = x & (A.G - 1);
                float sb, m2b;
                batch_stats(w[j], sl, A.nb, A.G, sb, m2b);
                if (sl == 0 && q < A.nq && P::row_is_primary(row) && ((qmask >> j) & 1u))
                    A.stat[(size_t)q * A.N + doc] = make_float2(sb, m2b);
            }
        } else {
            using SC = Score<NT, TQ>;
            float sc[SC::NS];
            SC::finish(w, A.T, col, sc);
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
        for (int tt = 0; tt < NT; ++tt) h[tt] = lowest_val<V>();
    };

    // ---- stage bookkeeping.  The reader walks the chunk stage by stage; when it enters stage st
    // the stages up to st+1 are visible to every wavefront (the first block of st+1 is read as
    // the "next block" while the last block of st is multiplied) and the following stage is in
    // flight.  All four wavefronts walk the same blocks, so they reach stage_enter at
    // the same points and its barrier matches up.
    // Slot safety: a stage is requested into the slot of a stage at least two behind the
    // reader, which no wavefront reads any more once all have passed the barrier.
    const int nst = (ntok + STAGE_ROWS - 1) / STAGE_ROWS;
    const int nfull = ntok / STAGE_ROWS;            // stages with all their rows
    // wait until this wavefront's copies have landed (keeping a second stage in flight across
    // the barrier was measured and gained nothing)
    auto wait_copies = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0) */ };
    // Workgroup barrier without a memory fence: the copies a wavefront is responsible for have
    // been awaited explicitly just before and every ring read of the slot that is about to be
    // overwritten has been consumed by its MFMAs.  The empty asm statements keep the compiler from moving ring accesses across.
    auto ring_barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    stage_fetch(0);
    if (nst > 1) stage_fetch(1);
    wait_copies();
    ring_barrier();
    if (nst > 2) stage_fetch(2);
    // the reader enters stage st >= 1: publish stage st+1, request the next one
    auto stage_enter = [&](int st) {
        if (st + 1 >= nst) return;                  // everything is visible already
        wait_copies();
        ring_barrier();
        if (st + 2 < nst) stage_fetch(st + 2);
    };

    // ---- block stream.  The chunk's tokens are one stream cut into aligned blocks of 16 rows,
    // whatever the document boundaries: no row is multiplied twice.  A block that lies inside
    // one document (most do) folds into the running maxima as it is; a block in which a
    // document ends is folded in two parts, rows before the boundary into the ending document
    // and the rows after it into fresh maxima for the next one (block_mma_split); further
    // boundaries in the same block repeat the block's MFMAs for the next part.  The rows past
    // the chunk's end in its last block repeat the last token.
    // a lane's operand pieces inside an aligned block: row `col` of the block, piece
    // (ks*4 + kg) ^ key(row); the key does not depend on the block (blocks start at multiples
    // of 16 rows)
    unsigned blk_off[F::KS];
#pragma unroll
    for (int ks = 0; ks < F::KS; ++ks)
        blk_off[ks] = (unsigned)(col * ROWB + (((ks * 4 + kg) ^ ((col >> KEY_SHIFT) & (NCH - 1))) * 16));
    // a complete block (bs + 16 <= ntok) of a visible stage
    auto load_aligned = [&](F& a, int bs) {
        using piece_t = __remove_reference_t(decltype(a.v[0]));
        const char* rp = ring + (bs & (RING_ROWS - 1)) * ROWB;       // uniform
#pragma unroll
        for (int ks = 0; ks < F::KS; ++ks) a.v[ks] = *(const piece_t*)(rp + blk_off[ks]);
    };
    // any block of a visible stage; the chunk's last block repeats the last token
    auto load_block = [&](F& a, int bs) {
        using piece_t = __remove_reference_t(decltype(a.v[0]));
        if (bs + 16 <= ntok) {
            load_aligned(a, bs);
            return;
        }
        int row = bs + col;
        row = row < ntok ? row : ntok - 1;
        const char* rp = ring + (row & (RING_ROWS - 1)) * ROWB;
        const int sw = (row >> KEY_SHIFT) & (NCH - 1);
#pragma unroll
        for (int ks = 0; ks < F::KS; ++ks) a.v[ks] = *(const piece_t*)(rp + (((ks * 4 + kg) ^ sw) * 16));
    };
    int doc = i0;                   // document whose maxima are being accumulated
    int dend = rel_off(i0 + 1);     // its end, relative to the chunk
    const int rowbase = 4 * kg;
    auto process = [&](const F& a, int bs) {
        int b = dend - bs;
        if (b > 16 || doc >= i1) {              // the block lies inside the current document
            if (mine(doc)) block_mma<NT>(a, bq, h);
            return;
        }
        int lo = 0;
        if (b == 16) {                          // it ends exactly with the block: no split needed
            block_mma<NT>(a, bq, h);
            finalize(doc);
            ++doc;
            if (doc >= i1) return;
            dend = rel_off(doc + 1);
            b = dend - bs;
            if (b > 16) return;                 // the usual case: the next document has tokens
            lo = 16;
        }
        for (;;) {
            V hB[NT];
#pragma unroll
            for (int tt = 0; tt < NT; ++tt) hB[tt] = lowest_val<V>();
            const int bb = b < lo ? lo : b;     // offsets that run backwards: an empty part
            // the usual case - one document end in the block - takes the fold specialised by the
            // row of the end (the wide kernels only: it is 15 copies of the block's code)
            if (NT >= 8 && lo == 0 && bb >= 1 && bb <= 15) block_mma_split_rows<NT>(a, bq, h, hB, bb);
            else block_mma_split<NT>(a, bq, h, hB, lo, bb, rowbase);
            finalize(doc);
            ++doc;
            if (doc >= i1) return;
            lo = bb;
            dend = rel_off(doc + 1);
            b = dend - bs;
            if (b > 16) {                       // the rest of the block starts the next document
#pragma unroll
                for (int tt = 0; tt < NT; ++tt) h[tt] = hB[tt];
                return;
            }
        }
    };

    // ---- consumer: the MFMAs of block k overlap the operand reads of block k+1.  a0 always
    // holds the block at bs; the stage that begins at bs (if one does) is entered just before
    // block bs is multiplied.  Runs of blocks that lie inside one document go through a loop
    // that holds nothing but the operand reads and the MFMAs of two blocks (and, every fourth
    // block, the stage entry); it covers the rows below tight_end, where every block has a
    // complete successor and every stage entered requests a complete stage.  A block in which a
    // document ends, and the chunk's last stages, take the general path.  Kernels with fewer
    // than eight column tiles per wavefront are bound by memory, not by the matrix pipes, and run
    // at a higher occupancy with fewer registers: they keep to the general path.
    constexpr bool TIGHT_RUNS = NT >= 8;
    const int tight_end = TIGHT_RUNS ? (nfull - 2) * STAGE_ROWS : 0;
    auto stage_enter_full = [&](int bs) {        // bs < tight_end is a stage boundary
        wait_copies();
        ring_barrier();
#pragma unroll
        for (int i = 0; i < LOADS_PER_WAVE; ++i) {
            const int r0 = bs + 2 * STAGE_ROWS + i * 4 * ROWS_PER_LOAD;               // uniform
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(src + (size_t)r0 * ROWB + fetch_off),
                (__attribute__((address_space(3))) void*)(ring + ((r0 + wave * ROWS_PER_LOAD) & (RING_ROWS - 1)) * ROWB),
                16, 0, LOAD_POLICY);
        }
    };
    auto at_boundary = [&](int bs) { return (bs & (STAGE_ROWS - 1)) == 0 && bs > 0; };
    F a0, a1;
    int bs = 0;
    load_block(a0, 0);
    while (bs < ntok) {
        if (TIGHT_RUNS && bs < tight_end) {
            // blocks from bs on that end before the current document does
            int run = doc < i1 ? (dend - bs - 1) >> 4 : RING_ROWS;
            const int left = (tight_end - bs) >> 4;
            run = run < 0 ? 0 : (run > left ? left : run);
            if (run >= 1 && (bs & 16)) {        // to an even block: pairs never straddle a stage
                load_aligned(a1, bs + 16);
                __builtin_amdgcn_sched_barrier(0);
                block_mma<NT>(a0, bq, h);
                a0 = a1;
                bs += 16;
                --run;
            }
#pragma unroll 1
            for (; run >= 2; run -= 2) {
                if (at_boundary(bs)) stage_enter_full(bs);
                load_aligned(a1, bs + 16);
                block_mma<NT>(a0, bq, h);
                load_aligned(a0, bs + 32);
                block_mma<NT>(a1, bq, h);
                bs += 32;
            }
            if (run == 1) {
                if (at_boundary(bs)) stage_enter_full(bs);
                load_aligned(a1, bs + 16);
                __builtin_amdgcn_sched_barrier(0);
                block_mma<NT>(a0, bq, h);
                a0 = a1;
                bs += 16;
            }
        }
        if (at_boundary(bs)) stage_enter(bs / STAGE_ROWS);
        if (bs + 16 < ntok) load_block(a1, bs + 16);
        __builtin_amdgcn_sched_barrier(0);      // keep the reads of the next block up here
        process(a0, bs);
        a0 = a1;
        bs += 16;
    }
    while (doc < i1) finalize(doc++);           // documents without tokens at the chunk's end
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

bool dense_supported(const Problem& P, const Coarse* co) {
    // the streaming kernel reads bf16 embeddings or int8 codes
    return (P.dt == DT_BF16 || co != nullptr) && (P.d == 64 || P.d == 128) &&
           P.total / 4096 < 0x7fffff00;
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

template <typename Tag, int D, int NT, int TQ, bool REVEAL, int SPLIT_DOCS = 0>
static hipError_t dense_go(DenseArgs& A, int tiles, hipStream_t st) {
    A.n_groups = SPLIT_DOCS ? 1 : (tiles + 4 * NT - 1) / (4 * NT);
    const int chunks8 = (A.n_chunks + 7) / 8 * 8;
    const long long blocks = (long long)chunks8 * A.n_groups;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    k_dense<Tag, D, NT, TQ, REVEAL, SPLIT_DOCS><<<(unsigned)blocks, DENSE_THREADS, 0, st>>>(A);
    return hipGetLastError();
}

template <typename Tag, int D, int TQ>
static hipError_t dense_score_nt(DenseArgs& A, int tiles, hipStream_t st) {
    // one or two queries (twice as many of at most 16 tokens): the tiles fit one or two
    // wavefronts, and four or two wavefronts split the documents
    if constexpr (TQ <= 2) {
        if (tiles <= 2) return dense_go<Tag, D, 2, TQ, false, 4>(A, tiles, st);
        if (tiles <= 4) return dense_go<Tag, D, 2, TQ, false, 2>(A, tiles, st);
    }
    if constexpr (TQ <= 2) {
        if (tiles <= 8) return dense_go<Tag, D, 2, TQ, false>(A, tiles, st);
    }
    if constexpr (TQ <= 4) {
        if (tiles <= 16) return dense_go<Tag, D, 4, TQ, false>(A, tiles, st);
    }
    return dense_go<Tag, D, 8, TQ, false>(A, tiles, st);
}

template <typename Tag, int D>
static hipError_t dense_score_d(DenseArgs& A, hipStream_t st) {
    const int tq = (A.T + 15) / 16;
    if (tq <= 1) return dense_score_nt<Tag, D, 1>(A, A.nq * 1, st);
    if (tq <= 2) return dense_score_nt<Tag, D, 2>(A, A.nq * 2, st);
    if (tq <= 4) return dense_score_nt<Tag, D, 4>(A, A.nq * 4, st);
    return dense_score_nt<Tag, D, 8>(A, A.nq * 8, st);
}

// int8 codes instead of the stored embeddings
static void use_codes(DenseArgs& A, const Coarse* co) {
    A.Q = co->Q8;
    A.docs = co->docs8;
    A.qscale = co->qscale;
    A.dscale = co->dscale;
}

hipError_t launch_dense_score(const Problem& P, const Work& W, int C, int n_chunks, float* out,
                              float* cells, const Coarse* co, hipStream_t st) {
    (void)C;
    DenseArgs A{};
    fill_dense(A, P, W, n_chunks);
    A.out = out;
    A.cells = cells;
    if (co) {
        use_codes(A, co);
        return P.d == 128 ? dense_score_d<i8_tag, 128>(A, st) : dense_score_d<i8_tag, 64>(A, st);
    }
    return P.d == 128 ? dense_score_d<bf16_tag, 128>(A, st) : dense_score_d<bf16_tag, 64>(A, st);
}

template <typename Tag, int D>
static hipError_t dense_reveal_d(DenseArgs& A, hipStream_t st) {
    const int tiles = (A.nq * A.G + 15) / 16;
    if (tiles <= 4) return dense_go<Tag, D, 1, 1, true>(A, tiles, st);
    if (tiles <= 8) return dense_go<Tag, D, 2, 1, true>(A, tiles, st);
    if (tiles <= 16) return dense_go<Tag, D, 4, 1, true>(A, tiles, st);
    return dense_go<Tag, D, 8, 1, true>(A, tiles, st);
}

static hipError_t dense_reveal_any(DenseArgs& A, const Problem& P, const Coarse* co, hipStream_t st) {
    if (co) {
        use_codes(A, co);
        return P.d == 128 ? dense_reveal_d<i8_tag, 128>(A, st) : dense_reveal_d<i8_tag, 64>(A, st);
    }
    return P.d == 128 ? dense_reveal_d<bf16_tag, 128>(A, st) : dense_reveal_d<bf16_tag, 64>(A, st);
}

hipError_t launch_dense_reveal(const Problem& P, const Work& W, int C, int n_chunks,
                               const RevealRound& rr, int G, const Coarse* co, hipStream_t st) {
    (void)C;
    DenseArgs A{};
    fill_dense(A, P, W, n_chunks);
    A.lo = rr.lo;
    A.nb = rr.nb;
    A.G = G;
    return dense_reveal_any(A, P, co, st);
}

hipError_t launch_dense_reveal_later(const Problem& P, const Work& W, int C, int n_chunks,
                                     const RevealRound& rr, int G, const Coarse* co,
                                     hipStream_t st) {
    (void)C;
    if (rr.dense_thr == ~0ull) return hipSuccess;
    DenseArgs A{};
    fill_dense(A, P, W, n_chunks);
    A.lo = rr.lo;
    A.nb = rr.nb;
    A.G = G;
    A.stat = W.stat2;
    A.pairs_r = W.pairs + rr.r;
    A.dense_thr = rr.dense_thr;
    A.ctl = W.ctl;
    return dense_reveal_any(A, P, co, st);
}

}  // namespace cb
