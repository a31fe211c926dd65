// Device-side building blocks shared by all kernels of the library: MFMA operand
// fragments, the per-document epilogues (score, batch statistics) and the
// Bernstein-Serfling interval.  Written for gfx950 (64-lane wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cb {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// `wide`: up to 8 column tiles (T <= 128) fit the register file; fp32 stops at 4.
struct bf16_tag { static constexpr bool wide = true; };
struct f32_tag { static constexpr bool wide = false; };

// Per-query round control, resident in the workspace.  `implicit` means the active set
// is still all N documents in index order (no list has been written yet).
struct QueryCtl {
    int count;     // |A| of the query
    int cur;       // which of the two id lists holds A
    int implicit;  // 1: A = [0,N) and no list exists
    int active;    // 1: the query still takes part in elimination rounds
};

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
// ---------------------------------------------------------------------------------
template <typename Tag, int D> struct Frag;

template <int D> struct Frag<bf16_tag, D> {
    static constexpr int KS = D / 32;
    static constexpr int ELEM_BYTES = 2;
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
};

template <int D> struct Frag<f32_tag, D> {
    static constexpr int KS = D / 16;
    static constexpr int ELEM_BYTES = 4;
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
};

// Accumulator layout of the 16x16 MFMAs: lane holds column (lane & 15) and rows
// 4*(lane >> 4) + {0,1,2,3}.  Rows are document tokens, columns are query rows.
__device__ __forceinline__ float max4(const f32x4_t& c) {
    return fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3]));
}

// Max over the four row groups of a column: afterwards every lane of a column holds
// the column's maximum over all 16 rows.
__device__ __forceinline__ float colmax_rows(float v) {
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

// Sum over the 16 columns (lanes sharing lane >> 4); fixed butterfly order.
__device__ __forceinline__ float sum_cols16(float v) {
    v += __shfl_xor(v, 8);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 1);
    return v;
}

// Sum over aligned groups of G consecutive columns (G a power of two <= 16).
__device__ __forceinline__ float sum_group(float v, int G) {
    for (int o = G >> 1; o >= 1; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Late-interaction score from the per-column maxima of one query (TQ column tiles,
// column c of tile tt is query token 16*tt + c): tokens >= T contribute 0, tiles are
// added in ascending order, then the 16 columns by butterfly.  Every kernel that
// produces a score goes through here, so equal cells give equal bits.
template <int TQ>
__device__ __forceinline__ float score_from_colmax(const float (&h)[TQ], int T, int col) {
    float s = 0.f;
#pragma unroll
    for (int tt = 0; tt < TQ; ++tt) s += (tt * 16 + col < T) ? h[tt] : 0.f;
    return sum_cols16(s);
}

// Statistics of one reveal batch held in a group of G columns (slot = col % G, the
// first nb slots are real): sum and centred sum of squares of the nb cells.
__device__ __forceinline__ void batch_stats(float h, int slot, int nb, int G, float& s,
                                            float& m2) {
    const bool valid = slot < nb;
    s = sum_group(valid ? h : 0.f, G);
    const float mean = s / (float)nb;
    const float dv = valid ? (h - mean) : 0.f;
    m2 = sum_group(dv * dv, G);
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

// Hybrid decision interval (paper Eq. (8)) from a document's revealed sum S and centred
// squares M2 after n cells: hard bounds S + (T-n)[a,b], estimator T*S/n, radius
// kappa*sigma_hat with sigma_hat^2 = M2/(n-1) (Appendix A).  n <= 1: hard bounds only;
// n == T: the interval is the exact sum.
__device__ __forceinline__ void interval(float S, float M2, int n, int T, float kappa, float a,
                                         float b, float& lcb, float& ucb) {
    const float rest = (float)(T - n);
    const float lb = S + rest * a, ub = S + rest * b;
    if (n <= 1) {
        lcb = lb;
        ucb = ub;
        return;
    }
    if (n >= T) {
        lcb = S;
        ucb = S;
        return;
    }
    const float shat = (float)T * (S / (float)n);
    const float sigma = sqrtf(fmaxf(M2, 0.f) / (float)(n - 1));
    const float r = kappa * sigma;
    lcb = fmaxf(lb, shat - r);
    ucb = fminf(ub, shat + r);
}

// Order-preserving map float -> uint32 (larger float, larger key).
__device__ __forceinline__ uint32_t float_key(float f) {
    uint32_t u = __float_as_uint(f + 0.0f);   // -0 and +0 share a key
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

}  // namespace cb
