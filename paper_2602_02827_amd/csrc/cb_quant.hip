// int8 codes for the coarse elimination pass (paper, implementation appendix, paragraph on the
// quantized layout: magnitudes are clipped at the 999th permille and the clipped range is coded
// linearly in 8 bits).
//
// Reading of the paper fixed here: the percentile is the nearest-rank one -- the element of
// rank ceil(n * permille / 1000) of the ascending order of |x| over one segment (the whole
// corpus matrix, or one query's T x d matrix) -- found exactly by a radix select on the bit
// pattern of |x| (for non-negative floats the bit pattern orders like the value).  A code is
// rint(x * (127 / clip)) saturated to [-127, 127], all in single precision, and decodes to
// code * (clip / 127).
//
// Everything stays on the device: three histogram passes (11 + 11 + 10 bits; bf16 inputs need
// only the first two) each followed by a one-wavefront kernel that picks the bin holding the
// rank, then the quantising pass.  Segments are independent (grid.y).
#include "cb_launch.h"

namespace cb {

constexpr int QH_BINS = 2048;
constexpr int QH_THREADS = 256;

struct SelState {                 // per segment, in the workspace
    unsigned long long rank;      // remaining 1-based ascending rank inside the current prefix
    uint32_t prefix, mask;        // key bits fixed so far
    uint32_t pad[2];
};

template <bool BF16>
__device__ __forceinline__ uint32_t abs_key(const void* x, int64_t i) {
    if (BF16) return ((uint32_t)(((const uint16_t*)x)[i] & 0x7fffu)) << 16;
    return ((const uint32_t*)x)[i] & 0x7fffffffu;
}

__global__ void k_quant_init(SelState* st, unsigned long long* hist, int64_t nseg,
                             unsigned long long rank) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nseg) {
        SelState s;
        s.rank = rank;
        s.prefix = 0;
        s.mask = 0;
        s.pad[0] = s.pad[1] = 0;
        st[i] = s;
    }
    if (i < nseg * QH_BINS) hist[i] = 0ull;
}

// VEC elements per 16-byte load
template <bool BF16> struct QVec { static constexpr int N = BF16 ? 8 : 4; };

// the VEC keys of 16 aligned bytes
template <bool BF16>
__device__ __forceinline__ void abs_keys16(const uint4& v, uint32_t (&k)[QVec<BF16>::N]) {
    if constexpr (BF16) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            k[2 * i] = (w[i] & 0x7fffu) << 16;
            k[2 * i + 1] = w[i] & 0x7fff0000u;
        }
    } else {
        k[0] = v.x & 0x7fffffffu;
        k[1] = v.y & 0x7fffffffu;
        k[2] = v.z & 0x7fffffffu;
        k[3] = v.w & 0x7fffffffu;
    }
}

// histogram of the `shift`-ed digit over the keys that match the segment's prefix.
// vec: the segment starts 16-byte aligned and holds a multiple of VEC elements.
template <bool BF16>
__global__ __launch_bounds__(QH_THREADS) void k_quant_hist(const void* x, int64_t seg_elems,
                                                           const SelState* st,
                                                           unsigned long long* hist, int shift,
                                                           int nbins, int vec) {
    __shared__ uint32_t lh[QH_BINS];
    constexpr int VEC = QVec<BF16>::N;
    const int64_t seg = blockIdx.y;
    for (int i = threadIdx.x; i < QH_BINS; i += QH_THREADS) lh[i] = 0;
    __syncthreads();
    const uint32_t prefix = st[seg].prefix, mask = st[seg].mask;
    const int64_t base = seg * seg_elems;
    // a block's share stays below 2^32 elements (the launch gives every block <= 2^32)
    if (vec) {
        const uint4* xv = (const uint4*)((const char*)x + base * (BF16 ? 2 : 4));
        const int64_t nv = seg_elems / VEC;
        for (int64_t i = (int64_t)blockIdx.x * QH_THREADS + threadIdx.x; i < nv;
             i += (int64_t)gridDim.x * QH_THREADS) {
            uint32_t k[VEC];
            abs_keys16<BF16>(xv[i], k);
#pragma unroll
            for (int u = 0; u < VEC; ++u)
                if ((k[u] & mask) == prefix) atomicAdd(&lh[(k[u] >> shift) & (nbins - 1)], 1u);
        }
    } else {
        for (int64_t i = (int64_t)blockIdx.x * QH_THREADS + threadIdx.x; i < seg_elems;
             i += (int64_t)gridDim.x * QH_THREADS) {
            const uint32_t k = abs_key<BF16>(x, base + i);
            if ((k & mask) == prefix) atomicAdd(&lh[(k >> shift) & (nbins - 1)], 1u);
        }
    }
    __syncthreads();
    unsigned long long* gh = hist + seg * QH_BINS;
    for (int i = threadIdx.x; i < nbins; i += QH_THREADS)
        if (lh[i]) atomicAdd(&gh[i], (unsigned long long)lh[i]);
}

// one wavefront per segment: ascending walk to the bin that holds the rank; clears the bins
__global__ __launch_bounds__(64) void k_quant_pick(SelState* st, unsigned long long* hist,
                                                   int shift, int nbins) {
    const int64_t seg = blockIdx.x;
    unsigned long long* gh = hist + seg * QH_BINS;
    const int lane = threadIdx.x;
    const int per = nbins / 64;
    const unsigned long long rank = st[seg].rank;
    unsigned long long local = 0;
    for (int j = 0; j < per; ++j) local += gh[lane * per + j];
    unsigned long long incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    const unsigned long long excl = incl - local;
    if (excl < rank && rank <= incl) {
        unsigned long long run = excl;
        for (int j = 0; j < per; ++j) {
            const unsigned long long c = gh[lane * per + j];
            if (run + c >= rank) {
                SelState s = st[seg];
                s.prefix |= (uint32_t)(lane * per + j) << shift;
                s.mask |= (uint32_t)(nbins - 1) << shift;
                s.rank = rank - run;
                st[seg] = s;
                break;
            }
            run += c;
        }
    }
    __syncthreads();
    for (int i = lane; i < QH_BINS; i += 64) gh[i] = 0ull;
}

__device__ __forceinline__ int code_of(float v, float inv) {
    float r = rintf(v * inv);
    r = r > 127.f ? 127.f : (r < -127.f ? -127.f : r);
    return (int)r;
}

template <bool BF16>
__global__ __launch_bounds__(QH_THREADS) void k_quant_codes(const void* x, int64_t seg_elems,
                                                            const SelState* st, int8_t* out,
                                                            float* scales, int vec) {
    constexpr int VEC = QVec<BF16>::N;
    const int64_t seg = blockIdx.y;
    const float clip = __uint_as_float(st[seg].prefix);
    const float inv = clip > 0.f ? 127.0f / clip : 0.f;
    if (blockIdx.x == 0 && threadIdx.x == 0) scales[seg] = clip / 127.0f;
    const int64_t base = seg * seg_elems;
    if (vec) {
        const uint4* xv = (const uint4*)((const char*)x + base * (BF16 ? 2 : 4));
        const int64_t nv = seg_elems / VEC;
        for (int64_t i = (int64_t)blockIdx.x * QH_THREADS + threadIdx.x; i < nv;
             i += (int64_t)gridDim.x * QH_THREADS) {
            const uint4 v = xv[i];
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            uint32_t packed[VEC / 4];
#pragma unroll
            for (int j = 0; j < VEC / 4; ++j) packed[j] = 0;
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                float f;
                if constexpr (BF16) f = __uint_as_float((u & 1) ? (w[u >> 1] & 0xffff0000u) : (w[u >> 1] << 16));
                else f = __uint_as_float(w[u]);
                packed[u >> 2] |= ((uint32_t)code_of(f, inv) & 0xffu) << (8 * (u & 3));
            }
            if constexpr (BF16) ((uint2*)(out + base))[i] = make_uint2(packed[0], packed[1]);
            else ((uint32_t*)(out + base))[i] = packed[0];
        }
        return;
    }
    for (int64_t i = (int64_t)blockIdx.x * QH_THREADS + threadIdx.x; i < seg_elems;
         i += (int64_t)gridDim.x * QH_THREADS) {
        float v;
        if (BF16) v = __uint_as_float((uint32_t)((const uint16_t*)x)[base + i] << 16);
        else v = ((const float*)x)[base + i];
        out[base + i] = (int8_t)code_of(v, inv);
    }
}

// Small segments (a query's T x d matrix): the whole job in one launch, one workgroup per
// segment.  Same selection (ascending rank over the radix digits of |x|) with the histogram in
// LDS; the segment is re-read from cache in every pass.
constexpr int QS_MAX_ELEMS = 65536;
template <bool BF16>
__global__ __launch_bounds__(QH_THREADS) void k_quant_small(const void* x, int seg_elems,
                                                            unsigned long long rank0, int8_t* out,
                                                            float* scales) {
    __shared__ uint32_t lh[QH_BINS];
    __shared__ uint32_t sel[2];           // chosen bin, remaining rank
    const int64_t base = (int64_t)blockIdx.x * seg_elems;
    uint32_t prefix = 0, mask = 0;
    uint32_t rank = (uint32_t)rank0;
    const int npass = BF16 ? 2 : 3;
#pragma unroll 1
    for (int p = 0; p < npass; ++p) {
        const int shift = p == 0 ? 21 : (p == 1 ? 10 : 0);
        const int nbins = p == 2 ? 1024 : 2048;
        for (int i = threadIdx.x; i < QH_BINS; i += QH_THREADS) lh[i] = 0;
        if (threadIdx.x == 0) {
            sel[0] = 0;
            sel[1] = 1;
        }
        __syncthreads();
        for (int i = threadIdx.x; i < seg_elems; i += QH_THREADS) {
            const uint32_t k = abs_key<BF16>(x, base + i);
            if ((k & mask) == prefix) atomicAdd(&lh[(k >> shift) & (nbins - 1)], 1u);
        }
        __syncthreads();
        if (threadIdx.x < 64) {
            const int lane = threadIdx.x;
            const int per = nbins / 64;
            uint32_t local = 0;
            for (int j = 0; j < per; ++j) local += lh[lane * per + j];
            uint32_t incl = local;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t t = __shfl_up(incl, o);
                if (lane >= o) incl += t;
            }
            const uint32_t excl = incl - local;
            if (excl < rank && rank <= incl) {
                uint32_t run = excl;
                for (int j = 0; j < per; ++j) {
                    const uint32_t c = lh[lane * per + j];
                    if (run + c >= rank) {
                        sel[0] = (uint32_t)(lane * per + j);
                        sel[1] = rank - run;
                        break;
                    }
                    run += c;
                }
            }
        }
        __syncthreads();
        prefix |= sel[0] << shift;
        mask |= (uint32_t)(nbins - 1) << shift;
        rank = sel[1];
        __syncthreads();
    }
    const float clip = __uint_as_float(prefix);
    const float inv = clip > 0.f ? 127.0f / clip : 0.f;
    if (threadIdx.x == 0) scales[blockIdx.x] = clip / 127.0f;
    for (int i = threadIdx.x; i < seg_elems; i += QH_THREADS) {
        float v;
        if (BF16) v = __uint_as_float((uint32_t)((const uint16_t*)x)[base + i] << 16);
        else v = ((const float*)x)[base + i];
        out[base + i] = (int8_t)code_of(v, inv);
    }
}

size_t quantize_scratch_bytes(int64_t n_segments) {
    return (size_t)n_segments * (sizeof(SelState) + sizeof(unsigned long long) * QH_BINS);
}

// x: [n_segments][seg_elems] of dt; codes: same shape; scales: [n_segments].
hipError_t launch_quantize_i8(const void* x, int dt, int64_t n_segments, int64_t seg_elems,
                              int permille, int8_t* codes, float* scales, void* scratch,
                              hipStream_t st) {
    const unsigned long long rank_all =
        ((unsigned long long)seg_elems * (unsigned long long)permille + 999ull) / 1000ull;
    if (seg_elems <= QS_MAX_ELEMS) {
        const unsigned long long r1 = rank_all < 1 ? 1 : rank_all;
        if (dt == DT_BF16)
            k_quant_small<true><<<(unsigned)n_segments, QH_THREADS, 0, st>>>(x, (int)seg_elems, r1, codes, scales);
        else
            k_quant_small<false><<<(unsigned)n_segments, QH_THREADS, 0, st>>>(x, (int)seg_elems, r1, codes, scales);
        return hipGetLastError();
    }
    SelState* state = (SelState*)scratch;
    unsigned long long* hist = (unsigned long long*)(state + n_segments);
    // ceil(seg_elems * permille / 1000), exact in 64-bit integers
    const unsigned long long rank =
        ((unsigned long long)seg_elems * (unsigned long long)permille + 999ull) / 1000ull;
    const int64_t init_n = n_segments * QH_BINS;
    k_quant_init<<<(unsigned)((init_n + 255) / 256), 256, 0, st>>>(state, hist, n_segments,
                                                                  rank < 1 ? 1 : rank);
    int64_t bx = (seg_elems + (int64_t)QH_THREADS * 64 - 1) / ((int64_t)QH_THREADS * 64);
    if (bx > 8192) bx = 8192;
    if (bx < 1) bx = 1;
    while (seg_elems / bx > (1ll << 24) * QH_THREADS) bx *= 2;   // per-block counts fit 32 bits
    const dim3 grid((unsigned)bx, (unsigned)n_segments);
    const bool bf = dt == DT_BF16;
    // 16-byte accesses need every segment (and the codes, 8 or 4 per store) aligned
    const int vec_n = bf ? 8 : 4;
    const int vec = (seg_elems % vec_n == 0 && ((uintptr_t)x & 15) == 0 && ((uintptr_t)codes & 7) == 0) ? 1 : 0;
    const int npass = bf ? 2 : 3;
    for (int p = 0; p < npass; ++p) {
        const int shift = p == 0 ? 21 : (p == 1 ? 10 : 0);
        const int nbins = p == 2 ? 1024 : 2048;
        if (bf) k_quant_hist<true><<<grid, QH_THREADS, 0, st>>>(x, seg_elems, state, hist, shift, nbins, vec);
        else k_quant_hist<false><<<grid, QH_THREADS, 0, st>>>(x, seg_elems, state, hist, shift, nbins, vec);
        k_quant_pick<<<(unsigned)n_segments, 64, 0, st>>>(state, hist, shift, nbins);
    }
    if (bf) k_quant_codes<true><<<grid, QH_THREADS, 0, st>>>(x, seg_elems, state, codes, scales, vec);
    else k_quant_codes<false><<<grid, QH_THREADS, 0, st>>>(x, seg_elems, state, codes, scales, vec);
    return hipGetLastError();
}

}  // namespace cb
