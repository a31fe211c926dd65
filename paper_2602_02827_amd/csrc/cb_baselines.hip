// The paper's two non-adaptive baselines (appendix "Compared Methods"), on the library's own
// scoring kernels:
//   Doc-Uniform   every (query, document) pair is scored on its own random subset of m query
//                 tokens.  Subsets that differ from document to document leave no query column
//                 that a matrix tile could share, so the MaxSim matrix is computed whole by the
//                 exhaustive kernel and k_uniform_score sums each row over its subset.
//   Ball-carving  the T query tokens are clustered greedily around pivots (k_ball_carve), each
//                 cluster is replaced by the sum of its members, and every document is scored
//                 by exhaustive MaxSim over the k centroids.  For bf16 the centroids of the whole
//                 batch are packed four to a group (k_ball_groups) and go through the corpus-
//                 streaming reveal kernel, whose cost follows the number of query columns, so
//                 the saving k/T shows up in time; k_ball_reduce adds a query's group sums.
#include "cb_launch.h"

namespace cb {

namespace {

__device__ __forceinline__ uint64_t mix_next(uint64_t& s) {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Subset of m of the T query tokens for (query key, document i): Floyd's sampling, driven by a
// SplitMix64 stream that starts at key + (i+1) * 0xD1B54A32D192ED03.
__device__ __forceinline__ uint64_t uniform_subset(uint64_t key, int64_t i, int T, int m) {
    uint64_t st = key + ((uint64_t)i + 1ull) * 0xD1B54A32D192ED03ull;
    uint64_t mask = 0;
    for (int j = T - m; j < T; ++j) {
        const uint32_t t = (uint32_t)__umul64hi(mix_next(st), (uint64_t)(j + 1));   // uniform in [0, j]
        mask |= ((mask >> t) & 1ull) ? (1ull << j) : (1ull << t);
    }
    return mask;
}

}  // namespace

// ---------------------------------------------------------------------------------------
// Doc-Uniform: scores[q][i] = sum over t in R_{q,i} of cells[q][i][t], t ascending.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_uniform_score(const float* cells, int64_t N, int T, int m,
                                                       uint64_t seed, float* scores,
                                                       uint64_t* masks) {
    const int q = blockIdx.y;
    uint64_t qs = seed + ((uint64_t)q + 1ull) * 0x9E3779B97F4A7C15ull;
    const uint64_t key = mix_next(qs);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (int64_t)gridDim.x * blockDim.x) {
        const uint64_t R = uniform_subset(key, i, T, m);
        const float* row = cells + ((size_t)q * N + i) * T;
        float s = 0.f;
        if ((T & 3) == 0) {                  // rows are 16-byte aligned
            for (int t = 0; t < T; t += 4) {
                const f32x4_t v = *(const f32x4_t*)(row + t);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if ((R >> (t + e)) & 1ull) s = s + v[e];
            }
        } else {
            for (int t = 0; t < T; ++t) {
                const float v = row[t];
                if ((R >> t) & 1ull) s = s + v;
            }
        }
        scores[(size_t)q * N + i] = s;
        if (masks) masks[(size_t)q * N + i] = R;
    }
}

hipError_t launch_uniform_score(const float* cells, int nq, int64_t N, int T, int m, uint64_t seed,
                                float* scores, uint64_t* masks, hipStream_t st) {
    int64_t bx = (N + 255) / 256;
    bx = bx > 4096 ? 4096 : bx;
    k_uniform_score<<<dim3((unsigned)bx, nq), 256, 0, st>>>(cells, N, T, m, seed, scores, masks);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Ball-carving, step 1.  One 64-thread workgroup per query, T <= 64, d <= 128.
// Token i joins pivot p iff dot > 0 and dot*dot >= ((tau*tau) * |p|^2) * |i|^2, all in double
// with sums over the components in ascending order: the test cos >= tau without a square root
// or a division, so that its outcome does not depend on how those are rounded.  The pivot always
// belongs to its own cluster.  A centroid is the single-precision sum of its members in ascending
// index, stored in the storage type (bf16: round to nearest even).
// ---------------------------------------------------------------------------------------
template <typename S> __device__ __forceinline__ float to_f32(S x) { return (float)x; }

template <typename S>
__global__ __launch_bounds__(64) void k_ball_carve(const S* Q, int T, int d, float tau, S* Cz,
                                                   int32_t* labels, int32_t* kq) {
    __shared__ float qs[64 * 128];
    __shared__ double nn[64];
    __shared__ int lab[64];
    const int q = blockIdx.x, tid = threadIdx.x;
    const S* Qq = Q + (size_t)q * T * d;
    for (int x = tid; x < T * d; x += 64) qs[x] = to_f32(Qq[x]);
    __syncthreads();
    if (tid < T) {
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += (double)qs[tid * d + c] * (double)qs[tid * d + c];
        nn[tid] = s;
        lab[tid] = -1;
    }
    __syncthreads();
    const double tau2 = (double)tau * (double)tau;
    S* Cq = Cz + (size_t)q * T * d;
    int k = 0;
    for (int p = 0; p < T; ++p) {
        if (lab[p] >= 0) continue;          // same value in every thread: p is not a pivot
        bool in = false;
        if (tid >= p && tid < T && lab[tid] < 0) {
            in = tid == p;
            if (!in) {
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += (double)qs[p * d + c] * (double)qs[tid * d + c];
                in = dot > 0.0 && dot * dot >= (tau2 * nn[p]) * nn[tid];
            }
        }
        __syncthreads();
        if (in) lab[tid] = k;
        __syncthreads();
        for (int c = tid; c < d; c += 64) {
            float acc = 0.f;
            for (int i = p; i < T; ++i)
                if (lab[i] == k) acc = acc + qs[i * d + c];
            Cq[(size_t)k * d + c] = (S)acc;
        }
        ++k;
    }
    for (int x = k * d + tid; x < T * d; x += 64) Cq[x] = (S)0.f;
    if (tid < T && labels) labels[(size_t)q * T + tid] = lab[tid];
    if (tid == 0) kq[q] = k;
}

// goff[q] = number of 4-column groups of the queries before q; goff[nq] = their total.
__global__ __launch_bounds__(1024) void k_ball_scan(const int32_t* kq, int nq, int32_t* goff) {
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int per = (nq + 1023) / 1024;
    const int b = tid * per < nq ? tid * per : nq;
    const int e = b + per < nq ? b + per : nq;
    int s = 0;
    for (int q = b; q < e; ++q) s += (kq[q] + 3) >> 2;
    part[tid] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const int v = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int base = part[tid] - s;
    for (int q = b; q < e; ++q) {
        goff[q] = base;
        base += (kq[q] + 3) >> 2;
    }
    if (tid == 1023) goff[nq] = part[1023];
}

// Rows of the packed query matrix: group g of query q holds centroids 4g .. 4g+3 (zero rows
// past the last centroid: a zero row's cell is 0 and adds nothing to a sum); the reveal kernel
// reads them through an identity token table.
__global__ __launch_bounds__(256) void k_ball_groups(const uint16_t* Cz, const int32_t* goff, int T,
                                                     int d, uint16_t* Qg, int32_t* ident) {
    const int q = blockIdx.x;
    const int g0 = goff[q], ng = goff[q + 1] - g0;
    const uint16_t* Cq = Cz + (size_t)q * T * d;
    for (int x = threadIdx.x; x < ng * 4 * d; x += blockDim.x) {
        const int row = x / d;
        Qg[(size_t)g0 * 4 * d + x] = row < T ? Cq[x] : (uint16_t)0;
    }
    for (int x = threadIdx.x; x < ng * 4; x += blockDim.x) ident[(size_t)g0 * 4 + x] = x & 3;
}

// scores[q][i] = sum over the query's groups, ascending, of part[g][i * stride].
__global__ __launch_bounds__(256) void k_ball_reduce(const float* part, int stride,
                                                     const int32_t* goff, int64_t N, float* scores) {
    const int q = blockIdx.y;
    const int g0 = goff[q], g1 = goff[q + 1];
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (int64_t)gridDim.x * blockDim.x) {
        float s = 0.f;
        for (int g = g0; g < g1; ++g) s = s + part[((size_t)g * N + i) * stride];
        scores[(size_t)q * N + i] = s;
    }
}

hipError_t launch_ball_carve(const Problem& P, float tau, void* Cz, int32_t* labels, int32_t* kq,
                             hipStream_t st) {
    if (P.dt == DT_BF16)
        k_ball_carve<__bf16><<<P.nq, 64, 0, st>>>((const __bf16*)P.Q, P.T, P.d, tau, (__bf16*)Cz,
                                                  labels, kq);
    else
        k_ball_carve<float><<<P.nq, 64, 0, st>>>((const float*)P.Q, P.T, P.d, tau, (float*)Cz,
                                                 labels, kq);
    return hipGetLastError();
}

hipError_t launch_ball_groups(const Problem& P, const void* Cz, const int32_t* kq, int32_t* goff,
                              void* Qg, int32_t* ident, hipStream_t st) {
    k_ball_scan<<<1, 1024, 0, st>>>(kq, P.nq, goff);
    k_ball_groups<<<P.nq, 256, 0, st>>>((const uint16_t*)Cz, goff, P.T, P.d, (uint16_t*)Qg, ident);
    return hipGetLastError();
}

hipError_t launch_ball_reduce(const float* part, int stride, const int32_t* goff, int nq, int64_t N,
                              float* scores, hipStream_t st) {
    int64_t bx = (N + 255) / 256;
    bx = bx > 4096 ? 4096 : bx;
    k_ball_reduce<<<dim3((unsigned)bx, nq), 256, 0, st>>>(part, stride, goff, N, scores);
    return hipGetLastError();
}

}  // namespace cb
