// Device-side building blocks shared by all kernels of the library: MFMA operand
// fragments, the per-document epilogues (score, batch statistics) and the
// Bernstein-Serfling interval.  Written for gfx950 (64-lane wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// No fused multiply-add contraction anywhere in this library's device code: the same
// formula must give the same bits in every kernel it is inlined into (the bound updates run
// in a cross-lane form and in a one-thread form).
#pragma clang fp contract(off)

namespace cb {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// `wide`: up to 8 column tiles (T <= 128) fit the register file; fp32 stops at 4.
struct bf16_tag { static constexpr bool wide = true; };
struct f32_tag { static constexpr bool wide = false; };
// int8 codes of the coarse elimination pass (implementation appendix, quantized layout)
struct i8_tag { static constexpr bool wide = true; };

// Per-query round control, resident in the workspace.  `implicit` means the active set
// is still all N documents in index order (no list has been written yet).
struct QueryCtl {
    int count;     // |A| of the query
    int cur;       // which of the two id lists holds A
    int implicit;  // 1: A = [0,N) and no list exists
    int active;    // 1: the query still takes part in elimination rounds
    int mode;      // 0: list entries are document ids; 1: they are slots of the cell cache
    int pad0, pad1, pad2;
};

// Device-side choice of a later round's reveal path (uniform over the launch): true = the
// corpus-streaming pass serves every active ids-mode query, false = per-pair gather.
__device__ __forceinline__ bool dense_round(const unsigned long long* pairs_r,
                                            unsigned long long thr) {
    return pairs_r != nullptr && *pairs_r > thr;
}


// ---------------------------------------------------------------------------------
// Operand fragments for the 16x16 MFMA family.  One fragment holds, for the lane's row
// (lane & 15) of a 16-row operand block, the d/4 elements that the lane's k-group
// (lane >> 4) contributes.  A (document tokens) and B (query rows) use the same
// k mapping, so every product q[k]*e[k] is formed exactly once.
//   bf16: v_mfma_f32_16x16x32_bf16, k-step s covers k in [32s, 32s+32); the lane
//         holds k = 32s + 8*(lane>>4) .. +7 (one 16-byte load).
//   fp32: v_mfma_f32_16x16x4_f32; the lane loads 16 bytes = k in
//         [16j + 4*(lane>>4), +4) and feeds component e to the e-th instruction of
//         group j, i.e. instruction (j,e) contracts k = 16j + 4g + e over g = 0..3.
//   int8: v_mfma_i32_16x16x64_i8, k-step s covers k in [64s, 64s+64); the lane holds
//         k = 64s + 16*(lane>>4) .. +15 (one 16-byte load); int32 accumulation is exact.
// acc_t / val_t: accumulator vector and the scalar type of a cell before decoding.
// ---------------------------------------------------------------------------------
template <typename Tag, int D> struct Frag;

template <int D> struct Frag<bf16_tag, D> {
    static constexpr int KS = D / 32;
    static constexpr int ELEM_BYTES = 2;
    using acc_t = f32x4_t;
    using val_t = float;
    bf16x8_t v[KS];
    __device__ __forceinline__ void load(const void* row, int kgroup) {
        const char* p = (const char*)row + kgroup * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) v[s] = *(const bf16x8_t*)(p + s * 64);
    }
    __device__ __forceinline__ static void mma(f32x4_t& acc, const Frag& a, const Frag& b) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v[s], b.v[s], acc, 0, 0, 0);
    }
    // two independent accumulation chains, interleaved step by step
    __device__ __forceinline__ static void mma2(f32x4_t& c0, f32x4_t& c1, const Frag& a,
                                                const Frag& b0, const Frag& b1) {
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            c0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v[s], b0.v[s], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v[s], b1.v[s], c1, 0, 0, 0);
        }
    }
};

template <int D> struct Frag<f32_tag, D> {
    static constexpr int KS = D / 16;
    static constexpr int ELEM_BYTES = 4;
    using acc_t = f32x4_t;
    using val_t = float;
    f32x4_t v[KS];
    __device__ __forceinline__ void load(const void* row, int kgroup) {
        const char* p = (const char*)row + kgroup * 16;
#pragma unroll
        for (int j = 0; j < KS; ++j) v[j] = *(const f32x4_t*)(p + j * 64);
    }
    __device__ __forceinline__ static void mma(f32x4_t& acc, const Frag& a, const Frag& b) {
#pragma unroll
        for (int j = 0; j < KS; ++j) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[j][e], b.v[j][e], acc, 0, 0, 0);
        }
    }
    __device__ __forceinline__ static void mma2(f32x4_t& c0, f32x4_t& c1, const Frag& a,
                                                const Frag& b0, const Frag& b1) {
#pragma unroll
        for (int j = 0; j < KS; ++j) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                c0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[j][e], b0.v[j][e], c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[j][e], b1.v[j][e], c1, 0, 0, 0);
            }
        }
    }
};

template <int D> struct Frag<i8_tag, D> {
    static constexpr int KS = D / 64;
    static constexpr int ELEM_BYTES = 1;
    using acc_t = i32x4_t;
    using val_t = int;
    i32x4_t v[KS];
    __device__ __forceinline__ void load(const void* row, int kgroup) {
        const char* p = (const char*)row + kgroup * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) v[s] = *(const i32x4_t*)(p + s * 64);
    }
    __device__ __forceinline__ static void mma(i32x4_t& acc, const Frag& a, const Frag& b) {
#pragma unroll
        for (int s = 0; s < KS; ++s)
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.v[s], b.v[s], acc, 0, 0, 0);
    }
    __device__ __forceinline__ static void mma2(i32x4_t& c0, i32x4_t& c1, const Frag& a,
                                                const Frag& b0, const Frag& b1) {
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            c0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.v[s], b0.v[s], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a.v[s], b1.v[s], c1, 0, 0, 0);
        }
    }
};

// "no token seen yet" for a running maximum
template <class V> __device__ __forceinline__ V lowest_val();
template <> __device__ __forceinline__ float lowest_val<float>() { return -__builtin_inff(); }
template <> __device__ __forceinline__ int lowest_val<int>() { return (int)0x80000000; }
__device__ __forceinline__ int imax(int a, int b) { return a > b ? a : b; }
__device__ __forceinline__ float vmax(float a, float b) { return fmaxf(a, b); }
__device__ __forceinline__ int vmax(int a, int b) { return a > b ? a : b; }

// Accumulator layout of the 16x16 MFMAs: lane holds column (lane & 15) and rows
// 4*(lane >> 4) + {0,1,2,3}.  Rows are document tokens, columns are query rows.
__device__ __forceinline__ float max4(const f32x4_t& c) {
    return fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3]));
}
// running maximum h <- max(h, c0..c3), two three-input maxima
__device__ __forceinline__ float fold_max(float h, const f32x4_t& c) {
    const float t = fmaxf(fmaxf(c[0], c[1]), c[2]);
    return fmaxf(fmaxf(h, t), c[3]);
}

__device__ __forceinline__ int fold_max(int h, const i32x4_t& c) {
    const int t = imax(imax(c[0], c[1]), c[2]);
    return imax(imax(h, t), c[3]);
}

// One block of 16 document tokens against NT column tiles, folded into the running
// maxima h.  Tiles go in pairs: the two accumulation chains of a pair are interleaved
// (no back-to-back dependent MFMAs) and a pair's maxima are taken while the next pair's
// MFMAs run.
template <int NT, class F>
__device__ __forceinline__ void block_mma(const F& a, const F (&bq)[NT],
                                          typename F::val_t (&h)[NT]) {
    using acc_t = typename F::acc_t;
    if constexpr (NT == 1) {
        acc_t acc = {0, 0, 0, 0};
        F::mma(acc, a, bq[0]);
        h[0] = fold_max(h[0], acc);
    } else {
        acc_t p0 = {0, 0, 0, 0}, p1 = p0;
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) {
            acc_t c0 = {0, 0, 0, 0}, c1 = c0;
            F::mma2(c0, c1, a, bq[2 * p], bq[2 * p + 1]);
            if (p > 0) {
                h[2 * p - 2] = fold_max(h[2 * p - 2], p0);
                h[2 * p - 1] = fold_max(h[2 * p - 1], p1);
            }
            p0 = c0;
            p1 = c1;
        }
        h[NT - 2] = fold_max(h[NT - 2], p0);
        h[NT - 1] = fold_max(h[NT - 1], p1);
    }
}

// The same block when a document ends inside it: rows [lo, b) of the block still belong to the
// current document and go into hA, rows [b, 16) into hB (the start of the next document); rows
// below lo were consumed by earlier documents.  inA[i] / inB[i]: membership of this lane's
// accumulator row 4*(lane>>4)+i.
template <class V, class ACC>
__device__ __forceinline__ void fold_split(V& hA, V& hB, const ACC& c, const bool (&inA)[4],
                                           const bool (&inB)[4]) {
    const V low = lowest_val<V>();
    V va[4], vb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        va[i] = inA[i] ? c[i] : low;
        vb[i] = inB[i] ? c[i] : low;
    }
    // three-input maxima, as in fold_max
    hA = vmax(vmax(hA, vmax(vmax(va[0], va[1]), va[2])), va[3]);
    hB = vmax(vmax(hB, vmax(vmax(vb[0], vb[1]), vb[2])), vb[3]);
}
template <int NT, class F>
__device__ __forceinline__ void block_mma_split(const F& a, const F (&bq)[NT],
                                                typename F::val_t (&hA)[NT],
                                                typename F::val_t (&hB)[NT], int lo, int b,
                                                int rowbase) {
    using acc_t = typename F::acc_t;
    bool inA[4], inB[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = rowbase + i;
        inA[i] = r >= lo && r < b;
        inB[i] = r >= b;
    }
    if constexpr (NT == 1) {
        acc_t acc = {0, 0, 0, 0};
        F::mma(acc, a, bq[0]);
        fold_split(hA[0], hB[0], acc, inA, inB);
    } else {
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) {
            acc_t c0 = {0, 0, 0, 0}, c1 = c0;
            F::mma2(c0, c1, a, bq[2 * p], bq[2 * p + 1]);
            fold_split(hA[2 * p], hB[2 * p], c0, inA, inB);
            fold_split(hA[2 * p + 1], hB[2 * p + 1], c1, inA, inB);
        }
    }
}

// ---------------------------------------------------------------------------------
// The split fold with the boundary known at compile time.  A block's 16 rows are four row
// groups of four (row group = lane >> 4 = a DPP row); rows [0, b) belong to the ending
// document, rows [b, 16) to the next one.  With KB = b / 4 and KR = b % 4 fixed, whole row
// groups are folded by one maximum that writes only the DPP rows named by an immediate row
// mask, and the one group that straddles the boundary (KR > 0) takes the maxima of its first
// KR and its last 4 - KR rows.  dpp_max<RM>(h, x): h <- max(h, x) in the rows of RM, h elsewhere
// (a DPP move whose disabled rows keep the identity of the maximum, then the maximum: the
// compiler merges the two into one v_max_*_dpp).
// ---------------------------------------------------------------------------------
template <int RM> __device__ __forceinline__ float dpp_max(float h, float x) {
    if constexpr (RM == 0) return h;
    else if constexpr (RM == 0xF) return fmaxf(h, x);
    else {
        const int low = __builtin_bit_cast(int, -__builtin_inff());
        const int y = __builtin_amdgcn_update_dpp(low, __builtin_bit_cast(int, x), 0xE4, RM, 0xF, false);
        return fmaxf(h, __builtin_bit_cast(float, y));
    }
}
template <int RM> __device__ __forceinline__ int dpp_max(int h, int x) {
    if constexpr (RM == 0) return h;
    else if constexpr (RM == 0xF) return h > x ? h : x;
    else {
        const int y = __builtin_amdgcn_update_dpp((int)0x80000000, x, 0xE4, RM, 0xF, false);
        return h > y ? h : y;
    }
}
template <int KB, int KR, class V, class ACC>
__device__ __forceinline__ void fold_split_at(V& hA, V& hB, const ACC& c) {
    constexpr int RM_A = (1 << KB) - 1;                         // row groups wholly before b
    constexpr int RM_S = KR > 0 ? (1 << KB) : 0;                // the straddling row group
    constexpr int RM_B = 0xF & ~(RM_A | RM_S);                  // row groups wholly from b on
    V sA, sB, all;
    if constexpr (KR == 0) {
        all = vmax(vmax(vmax(c[0], c[1]), c[2]), c[3]);
        sA = sB = all;
    } else if constexpr (KR == 1) {
        sA = c[0];
        sB = vmax(vmax(c[1], c[2]), c[3]);
        all = vmax(sA, sB);
    } else if constexpr (KR == 2) {
        sA = vmax(c[0], c[1]);
        sB = vmax(c[2], c[3]);
        all = vmax(sA, sB);
    } else {
        sA = vmax(vmax(c[0], c[1]), c[2]);
        sB = c[3];
        all = vmax(sA, sB);
    }
    if constexpr (__is_same(V, float)) {
        // Written out: the compiler merges the move and the maximum only for integers.  sA, sB
        // and `all` were written by vector instructions just before; a DPP operand may be read
        // two wait states after such a write at the earliest, hence the leading s_nop; the
        // trailing one gives whatever the compiler places next (it does not see these writes)
        // the same distance to hA and hB.  Row masks of zero (no such row group) make the
        // instruction a no-op.
        if constexpr (KR > 0) {
            asm("s_nop 1\n\t"
                "v_max_f32_dpp %0, %2, %0 quad_perm:[0,1,2,3] row_mask:%5 bank_mask:0xf\n\t"
                "v_max_f32_dpp %1, %2, %1 quad_perm:[0,1,2,3] row_mask:%6 bank_mask:0xf\n\t"
                "v_max_f32_dpp %0, %3, %0 quad_perm:[0,1,2,3] row_mask:%7 bank_mask:0xf\n\t"
                "v_max_f32_dpp %1, %4, %1 quad_perm:[0,1,2,3] row_mask:%7 bank_mask:0xf\n\t"
                "s_nop 1"
                : "+v"(hA), "+v"(hB)
                : "v"(all), "v"(sA), "v"(sB), "n"(RM_A), "n"(RM_B), "n"(RM_S));
        } else {
            asm("s_nop 1\n\t"
                "v_max_f32_dpp %0, %2, %0 quad_perm:[0,1,2,3] row_mask:%3 bank_mask:0xf\n\t"
                "v_max_f32_dpp %1, %2, %1 quad_perm:[0,1,2,3] row_mask:%4 bank_mask:0xf\n\t"
                "s_nop 1"
                : "+v"(hA), "+v"(hB)
                : "v"(all), "n"(RM_A), "n"(RM_B));
        }
    } else {
        hA = dpp_max<RM_A>(hA, all);
        hB = dpp_max<RM_B>(hB, all);
        if constexpr (KR > 0) {
            hA = dpp_max<RM_S>(hA, sA);
            hB = dpp_max<RM_S>(hB, sB);
        }
    }
}
// block_mma_split for rows [0, b) / [b, 16), b = 4 * KB + KR in 1..15
template <int NT, int KB, int KR, class F>
__device__ __forceinline__ void block_mma_split_at(const F& a, const F (&bq)[NT],
                                                   typename F::val_t (&hA)[NT],
                                                   typename F::val_t (&hB)[NT]) {
    using acc_t = typename F::acc_t;
    if constexpr (NT == 1) {
        acc_t acc = {0, 0, 0, 0};
        F::mma(acc, a, bq[0]);
        fold_split_at<KB, KR>(hA[0], hB[0], acc);
    } else {
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) {
            acc_t c0 = {0, 0, 0, 0}, c1 = c0;
            F::mma2(c0, c1, a, bq[2 * p], bq[2 * p + 1]);
            fold_split_at<KB, KR>(hA[2 * p], hB[2 * p], c0);
            fold_split_at<KB, KR>(hA[2 * p + 1], hB[2 * p + 1], c1);
        }
    }
}
template <int NT, class F>
__device__ __forceinline__ void block_mma_split_rows(const F& a, const F (&bq)[NT],
                                                     typename F::val_t (&hA)[NT],
                                                     typename F::val_t (&hB)[NT], int b) {
    switch (b) {
#define CB_SPLIT_CASE(B) case B: block_mma_split_at<NT, (B) / 4, (B) % 4>(a, bq, hA, hB); break;
        CB_SPLIT_CASE(1) CB_SPLIT_CASE(2) CB_SPLIT_CASE(3) CB_SPLIT_CASE(4) CB_SPLIT_CASE(5)
        CB_SPLIT_CASE(6) CB_SPLIT_CASE(7) CB_SPLIT_CASE(8) CB_SPLIT_CASE(9) CB_SPLIT_CASE(10)
        CB_SPLIT_CASE(11) CB_SPLIT_CASE(12) CB_SPLIT_CASE(13) CB_SPLIT_CASE(14) CB_SPLIT_CASE(15)
#undef CB_SPLIT_CASE
        default: break;
    }
}

// ---------------------------------------------------------------------------------
// Cross-lane helpers.  A wavefront is four rows of 16 lanes; row = lane >> 4 is the
// accumulator's row group, col = lane & 15 its column.  DPP moves data inside a row,
// v_permlane32_swap / v_permlane16_swap exchange rows between two registers:
//   swap32(a,b): a' = [a.r0 a.r1 b.r0 b.r1]   b' = [a.r2 a.r3 b.r2 b.r3]
//   swap16(a,b): a' = [a.r0 b.r0 a.r2 b.r2]   b' = [a.r1 b.r1 a.r3 b.r3]
// ---------------------------------------------------------------------------------
constexpr int DPP_QUAD_XOR1 = 0xB1;    // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;    // quad_perm [2,3,0,1]
constexpr int DPP_ROW_MIRROR = 0x140;
constexpr int DPP_ROW_HALF_MIRROR = 0x141;
constexpr int DPP_ROW_ROR = 0x120;     // + n: lane c reads lane (c - n) mod 16 of its row

template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ void swap32(float& a, float& b) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    const unsigned r0 = r[0], r1 = r[1];   // copy the elements out before reinterpreting them
    a = __uint_as_float(r0);
    b = __uint_as_float(r1);
}
__device__ __forceinline__ void swap16(float& a, float& b) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    const unsigned r0 = r[0], r1 = r[1];   // copy the elements out before reinterpreting them
    a = __uint_as_float(r0);
    b = __uint_as_float(r1);
}
// rows 0,1 <- max over (r0,r2),(r1,r3) of a; rows 2,3 <- the same of b
__device__ __forceinline__ float maxpack32(float a, float b) {
    swap32(a, b);
    return fmaxf(a, b);
}
// rows 0,2 <- max over (r0,r1),(r2,r3) of a; rows 1,3 <- the same of b
__device__ __forceinline__ float maxpack16(float a, float b) {
    swap16(a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ int maxpack32(int a, int b) {
    auto r = __builtin_amdgcn_permlane32_swap((unsigned)a, (unsigned)b, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    return imax((int)r0, (int)r1);
}
__device__ __forceinline__ int maxpack16(int a, int b) {
    auto r = __builtin_amdgcn_permlane16_swap((unsigned)a, (unsigned)b, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    return imax((int)r0, (int)r1);
}
// every lane <- w[lane] + w[lane ^ 32] (lower-row operand first in every lane)
__device__ __forceinline__ float addswap32(float w) {
    float a = w, b = w;
    swap32(a, b);
    return a + b;
}
// every lane <- w[lane] + w[lane ^ 16] (even-row operand first in every lane)
__device__ __forceinline__ float addswap16(float w) {
    float a = w, b = w;
    swap16(a, b);
    return a + b;
}
// Sum of the 16 columns of a row by four rotations.  The association order depends on
// the lane, so only column 0's value is the canonical one (it is the only one stored).
__device__ __forceinline__ float rowsum16(float v) {
    v += dpp_mov<DPP_ROW_ROR + 8>(v);
    v += dpp_mov<DPP_ROW_ROR + 4>(v);
    v += dpp_mov<DPP_ROW_ROR + 2>(v);
    v += dpp_mov<DPP_ROW_ROR + 1>(v);
    return v;
}
// Sum over aligned groups of G consecutive columns, G in {1,2,4,8,16}; slot 0 of the group
// holds the canonical value.
template <int G> __device__ __forceinline__ float sum_group(float v) {
    if (G >= 16) v += dpp_mov<DPP_ROW_MIRROR>(v);
    if (G >= 8) v += dpp_mov<DPP_ROW_HALF_MIRROR>(v);
    if (G >= 4) v += dpp_mov<DPP_QUAD_XOR2>(v);
    if (G >= 2) v += dpp_mov<DPP_QUAD_XOR1>(v);
    return v;
}

// Packing of NT per-tile running maxima (each lane: its column, its row group's 4 rows)
// into registers whose ROWS are tiles: after pack_colmax every lane of row r of w[j]
// holds the maximum over all 16 accumulator rows of column col of tile tile_of_row(j, r).
template <int NT> struct Pack {
    static constexpr int NW = NT >= 4 ? NT / 4 : 1;
    // which tile sits in row `row` of packed register j
    __device__ __forceinline__ static int tile_of_row(int j, int row) {
        if (NT >= 4) return 4 * j + (((row & 1) << 1) | (row >> 1));
        if (NT == 2) return row >> 1;
        return 0;
    }
    // a row that holds tile `tile` of its packed register (tile taken modulo 4)
    __device__ __forceinline__ static int row_of_tile(int tile) {
        const int k = tile & 3;
        if (NT >= 4) return ((k & 1) << 1) | (k >> 1);
        if (NT == 2) return (k & 1) << 1;
        return 0;
    }
    // rows that hold a tile not already held by a lower row
    __device__ __forceinline__ static bool row_is_primary(int row) {
        if (NT >= 4) return true;
        if (NT == 2) return (row & 1) == 0;
        return row == 0;
    }
    template <class V>
    __device__ __forceinline__ static void colmax(const V (&h)[NT], V (&w)[NW]) {
        if constexpr (NT == 1) {
            const V m = maxpack32(h[0], h[0]);
            w[0] = maxpack16(m, m);
        } else if constexpr (NT == 2) {
            const V m = maxpack32(h[0], h[1]);
            w[0] = maxpack16(m, m);
        } else {
#pragma unroll
            for (int j = 0; j < NW; ++j) {
                const V m0 = maxpack32(h[4 * j], h[4 * j + 1]);
                const V m1 = maxpack32(h[4 * j + 2], h[4 * j + 3]);
                w[j] = maxpack16(m0, m1);
            }
        }
    }
};

// Late-interaction scores from NT tile maxima, TQ consecutive tiles per query (column c of
// a query's tile k is query token 16k + c; tokens >= T count as 0).  Fixed order: tiles are
// added pairwise (t0+t1), then ((t0+t1)+(t2+t3)), then the two halves of 8, then the 16
// columns by rowsum16.  Every kernel that produces a score goes through here, so equal
// cells give equal bits.  Outputs: w = packed cells (masked), s[j] = score register j.
// Use score_writer() to find the lanes that own a query's score.
template <int NT, int TQ> struct Score {
    using P = Pack<NT>;
    static constexpr int NW = P::NW;
    static constexpr int NS = TQ == 8 ? 1 : NW;
    __device__ __forceinline__ static void run(float (&h)[NT], int T, int col, float (&w)[NW],
                                               float (&s)[NS]) {
        P::colmax(h, w);
        finish(w, T, col, s);
    }
    // the same from packed cells (row r of w[j] = tile tile_of_row(j, r)); columns that are
    // not query tokens are zeroed in w
    __device__ __forceinline__ static void finish(float (&w)[NW], int T, int col, float (&s)[NS]) {
        if (T != TQ * 16) {
            const int row = (int)(threadIdx.x & 63) >> 4;
#pragma unroll
            for (int j = 0; j < NW; ++j)
                if ((P::tile_of_row(j, row) % TQ) * 16 + col >= T) w[j] = 0.f;
        }
        if constexpr (TQ == 1) {
#pragma unroll
            for (int j = 0; j < NW; ++j) s[j] = rowsum16(w[j]);
        } else if constexpr (TQ == 2) {
#pragma unroll
            for (int j = 0; j < NW; ++j) s[j] = rowsum16(addswap32(w[j]));
        } else if constexpr (TQ == 4) {
#pragma unroll
            for (int j = 0; j < NW; ++j) s[j] = rowsum16(addswap16(addswap32(w[j])));
        } else {
            const float y0 = addswap16(addswap32(w[0]));
            const float y1 = addswap16(addswap32(w[1]));
            s[0] = rowsum16(y0 + y1);
        }
    }
    // local query index (0 .. NT/TQ-1) whose score lane `lane` holds in s[j], or -1
    __device__ __forceinline__ static int writer(int j, int lane) {
        const int row = lane >> 4;
        if ((lane & 15) != 0) return -1;
        if (TQ == 1) return P::row_is_primary(row) ? P::tile_of_row(j, row) : -1;
        if (TQ == 2) {
            if (NT >= 4) return row < 2 ? 2 * j + row : -1;
            return row == 0 ? 0 : -1;
        }
        return row == 0 ? j : -1;
    }
};

// x / n for a small positive count n.  A power of two divides exactly by multiplying with its
// reciprocal (same bits as the division), which spares the long division sequence in the
// common case of 4 cells per batch.
__device__ __forceinline__ float div_count(float x, int n) {
    if ((n & (n - 1)) == 0) return x * (1.0f / (float)n);
    return x / (float)n;
}

// Statistics of one reveal batch held in a group of G columns (slot = column % G, the
// first nb slots are real): sum and centred sum of squares of the nb cells; canonical at
// slot 0.
template <int G>
__device__ __forceinline__ void batch_stats_g(float h, int slot, int nb, float& s, float& m2) {
    const bool valid = slot < nb;
    s = sum_group<G>(valid ? h : 0.f);
    const float mean = div_count(s, nb);
    const float dv = valid ? (h - mean) : 0.f;
    m2 = sum_group<G>(dv * dv);
}
__device__ __forceinline__ void batch_stats(float h, int slot, int nb, int G, float& s, float& m2) {
    switch (G) {
        case 1: batch_stats_g<1>(h, slot, nb, s, m2); break;
        case 2: batch_stats_g<2>(h, slot, nb, s, m2); break;
        case 4: batch_stats_g<4>(h, slot, nb, s, m2); break;
        case 8: batch_stats_g<8>(h, slot, nb, s, m2); break;
        default: batch_stats_g<16>(h, slot, nb, s, m2); break;
    }
}

// Merge a batch (nb cells: sum sb, centred squares m2b) into a document's running
// (sum S, centred squares M2 over n_prev cells); pairwise update of Chan et al.
__device__ __forceinline__ void merge_stats(float& S, float& M2, int n_prev, float sb, float m2b,
                                            int nb) {
    if (n_prev == 0) {
        S = sb;
        M2 = m2b;
        return;
    }
    const float dm = sb / (float)nb - S / (float)n_prev;
    M2 = M2 + m2b + dm * dm * ((float)n_prev * (float)nb / (float)(n_prev + nb));
    S += sb;
}

// NaN test on the bit pattern: device code is compiled under the assumption that floating-point
// comparisons never see a NaN, so a comparison cannot be trusted to detect one.
__device__ __forceinline__ bool is_nan_bits(float x) {
    return (__float_as_uint(x) & 0x7fffffffu) > 0x7f800000u;
}

// Hybrid decision interval (paper Eq. (8)) from a document's revealed sum S and centred
// squares M2 after n cells: hard bounds S + (T-n)[a,b], estimator T*S/n, radius
// kappa*sigma_hat with sigma_hat^2 = M2/(n-1) (Appendix A).  n <= 1: hard bounds only;
// n == T: the interval is the exact sum.
// Inputs outside the contract (a document without tokens has cells -inf and M2 = NaN; NaN
// embeddings give NaN cells) yield the interval [-inf, -inf]: such a document is dropped as soon
// as K others exist and never disturbs the threshold of the rest.
__device__ __forceinline__ void interval(float S, float M2, int n, int T, float kappa, float a,
                                         float b, float& lcb, float& ucb) {
    const float rest = (float)(T - n);
    const float lb = S + rest * a, ub = S + rest * b;
    if (n <= 1) {
        lcb = lb;
        ucb = ub;
    } else if (n >= T) {
        lcb = S;
        ucb = S;
    } else {
        const float shat = (float)T * (S / (float)n);
        const float sigma = sqrtf(fmaxf(M2, 0.f) / (float)(n - 1));
        const float r = kappa * sigma;
        lcb = fmaxf(lb, shat - r);
        ucb = fminf(ub, shat + r);
    }
    if (is_nan_bits(S) || is_nan_bits(M2) || is_nan_bits(lcb) || is_nan_bits(ucb)) {
        lcb = -__builtin_inff();
        ucb = -__builtin_inff();
    }
}

// Order-preserving map float -> uint32 (larger float, larger key); NaN maps below everything.
__device__ __forceinline__ uint32_t float_key(float f) {
    if (is_nan_bits(f)) return 0u;
    uint32_t u = __float_as_uint(f + 0.0f);   // -0 and +0 share a key
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k) {
    if (k < 0x007fffffu) return -__builtin_inff();      // below the key of -inf: NaN's key
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

}  // namespace cb
