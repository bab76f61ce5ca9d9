// Smooth-and-quantize pre-pass of SageAttention for gfx950 (HBM-bound kernels).
//
//   column sums of K over tokens      -> exact integer arithmetic (Section 4.2, mean(K))
//   K - mean(K), per-block absmax,    -> Section 4.2 (gamma) + Section 3.2 (per-block psi)
//   INT8 pack
//   Q * sm_scale, per-block absmax,   -> Section 4.6 (scale folded into Q) + Section 3.2
//   INT8 pack
//
// Every fp16 value is an integer multiple of 2^-24, so the column sum is accumulated as an
// integer count of 2^-24 units; the result does not depend on how tokens are split over
// threads, workgroups or atomics.  One fp64 division and one rounding to fp32 give the mean.
#include "sage_internal.h"
#include <hip/hip_fp16.h>

namespace sage {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

__global__ void __launch_bounds__(256) zero_sums_kernel(long long* sums, int n) {
    int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) sums[i] = 0;
}

// grid (ceil(N / CHUNK), BH); CHUNK = 32 rows per thread * (256 / (D/8)) row groups.
template <int D>
__global__ void __launch_bounds__(256) k_colsum_kernel(const _Float16* __restrict__ k,
                                                       long long* __restrict__ sums, int N) {
    constexpr int VPR = D / 8;          // 16-byte vectors per token row
    constexpr int RG = 256 / VPR;       // row groups per workgroup
    constexpr int RPT = 32;             // rows per thread: keeps the int32 partials far from overflow
    constexpr int CHUNK = RG * RPT;
    const int t = threadIdx.x, c8 = t % VPR, rg = t / VPR;
    const int bh = blockIdx.y;
    const int row_base = blockIdx.x * CHUNK + rg;
    const _Float16* base = k + ((size_t)bh * N) * D + c8 * 8;

    int acc_hi[8], acc_lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { acc_hi[e] = 0; acc_lo[e] = 0; }
#pragma unroll 8
    for (int i = 0; i < RPT; ++i) {
        int r = row_base + i * RG;
        if (r < N) {
            h8 x = *(const h8*)(base + (size_t)r * D);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)x[e];
                float hi = __builtin_truncf(f);          // integer part, |hi| <= 65504
                float lo = f - hi;                       // exact; a multiple of 2^-24 below 1
                acc_hi[e] += (int)hi;
                acc_lo[e] += (int)(lo * 16777216.0f);    // exact integer below 2^24
            }
        }
    }
    __shared__ long long part[RG][D];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        part[rg][c8 * 8 + e] = (long long)acc_hi[e] * 16777216ll + (long long)acc_lo[e];
    __syncthreads();
    if (t < D) {
        long long s = 0;
#pragma unroll 4
        for (int g = 0; g < RG; ++g) s += part[g][t];
        atomicAdd((unsigned long long*)(sums + (size_t)bh * D + t), (unsigned long long)s);
    }
}

__device__ __forceinline__ float wg_max(float v, float* red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = __builtin_fmaxf(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return __builtin_fmaxf(__builtin_fmaxf(red[0], red[1]), __builtin_fmaxf(red[2], red[3]));
}

// One workgroup per quantization block of `block` tokens x D channels; block * D = 2048 * LPT.
// IS_K: x - mean (mean derived from the exact sums); else x * sm_scale.
template <int D, int LPT, bool IS_K>
__global__ void __launch_bounds__(256) quant_block_kernel(const _Float16* __restrict__ x,
                                                          int8_t* __restrict__ xq,
                                                          float* __restrict__ scale,
                                                          float* __restrict__ k_mean,
                                                          const long long* __restrict__ sums,
                                                          int N, int block, float sm_scale) {
    constexpr int VPR = D / 8;
    constexpr int RSTEP = 256 / VPR;
    const int t = threadIdx.x, c8 = t % VPR, rbase = t / VPR;
    const int g = blockIdx.x, bh = blockIdx.y, nblk = gridDim.x;
    const int row0 = g * block;
    const int rows = (N - row0 < block) ? (N - row0) : block;

    __shared__ float s_mean[D];
    __shared__ float s_red[4];
    float mean[8];
    if (IS_K) {
        if (t < D) {
            long long s = sums[(size_t)bh * D + t];
            double avg = (double)s / (double)N;
            float m = (float)(avg * 0x1p-24);
            s_mean[t] = m;
            if (g == 0) k_mean[(size_t)bh * D + t] = m;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) mean[e] = s_mean[c8 * 8 + e];
    }

    const size_t slab = ((size_t)bh * N + row0) * D + c8 * 8;
    h8 raw[LPT];
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        int r = rbase + i * RSTEP;
        if (r < rows) {
            raw[i] = *(const h8*)(x + slab + (size_t)r * D);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)raw[i][e];
                f = IS_K ? (f - mean[e]) : (f * sm_scale);
                amax = __builtin_fmaxf(amax, __builtin_fabsf(f));
            }
        }
    }
    amax = wg_max(amax, s_red);
    const float delta = amax / 127.0f;
    const float rcp = amax > 0.0f ? 127.0f / amax : 0.0f;
    if (t == 0) scale[(size_t)bh * nblk + g] = delta;

#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        int r = rbase + i * RSTEP;
        if (r < rows) {
            unsigned w[2] = {0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f = (float)raw[i][e];
                f = IS_K ? (f - mean[e]) : (f * sm_scale);
                float q = __builtin_rintf(f * rcp);                 // round half to even
                q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
                w[e >> 2] |= ((unsigned)((int)q) & 0xffu) << (8 * (e & 3));
            }
            *(uint2*)(xq + slab + (size_t)r * D) = make_uint2(w[0], w[1]);
        }
    }
}

// Per-token quantizer (Section 3.2): one scale per token row.  D/8 adjacent lanes own a row
// (16 bytes each); the row's absmax is a butterfly over those lanes.  A workgroup covers
// TOK_ROWS consecutive tokens, TOK_LPT rows per thread, all loads issued before the first use.
constexpr int TOK_LPT = 8;
template <int D, bool IS_K>
__global__ void __launch_bounds__(256) quant_token_kernel(const _Float16* __restrict__ x,
                                                          int8_t* __restrict__ xq,
                                                          float* __restrict__ scale,
                                                          float* __restrict__ k_mean,
                                                          const long long* __restrict__ sums,
                                                          int N, float sm_scale) {
    constexpr int VPR = D / 8;
    constexpr int RSTEP = 256 / VPR;
    constexpr int ROWS = RSTEP * TOK_LPT;
    const int t = threadIdx.x, c8 = t % VPR, rbase = t / VPR;
    const int bh = blockIdx.y;
    const int row0 = blockIdx.x * ROWS;

    __shared__ float s_mean[D];
    float mean[8];
    if (IS_K) {
        if (t < D) {
            long long s = sums[(size_t)bh * D + t];
            double avg = (double)s / (double)N;
            float m = (float)(avg * 0x1p-24);
            s_mean[t] = m;
            if (blockIdx.x == 0) k_mean[(size_t)bh * D + t] = m;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) mean[e] = s_mean[c8 * 8 + e];
    }

    const size_t slab = ((size_t)bh * N + row0) * D + c8 * 8;
    h8 raw[TOK_LPT];
#pragma unroll
    for (int i = 0; i < TOK_LPT; ++i) {
        int r = rbase + i * RSTEP;
        raw[i] = (h8){0, 0, 0, 0, 0, 0, 0, 0};
        if (row0 + r < N) raw[i] = *(const h8*)(x + slab + (size_t)r * D);
    }
#pragma unroll
    for (int i = 0; i < TOK_LPT; ++i) {
        const int r = rbase + i * RSTEP;
        float f[8];
        float amax = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            f[e] = (float)raw[i][e];
            f[e] = IS_K ? (f[e] - mean[e]) : (f[e] * sm_scale);
            amax = __builtin_fmaxf(amax, __builtin_fabsf(f[e]));
        }
#pragma unroll
        for (int off = VPR / 2; off >= 1; off >>= 1) amax = __builtin_fmaxf(amax, __shfl_xor(amax, off, 64));
        const float delta = amax / 127.0f;
        const float rcp = amax > 0.0f ? 127.0f / amax : 0.0f;
        if (row0 + r < N) {
            if (c8 == 0) scale[(size_t)bh * N + row0 + r] = delta;
            unsigned w[2] = {0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float q = __builtin_rintf(f[e] * rcp);                 // round half to even
                q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
                w[e >> 2] |= ((unsigned)((int)q) & 0xffu) << (8 * (e & 3));
            }
            *(uint2*)(xq + slab + (size_t)r * D) = make_uint2(w[0], w[1]);
        }
    }
}

template <int D, bool IS_K>
static hipError_t launch_quant(const void* x, int8_t* xq, float* scale, float* mean, const long long* sums,
                               int BH, int N, int block, float sm_scale, hipStream_t st) {
    const _Float16* xp = (const _Float16*)x;
    if (block == 1) {
        constexpr int ROWS = (256 / (D / 8)) * TOK_LPT;
        quant_token_kernel<D, IS_K><<<dim3((N + ROWS - 1) / ROWS, BH), 256, 0, st>>>(xp, xq, scale, mean, sums, N, sm_scale);
        return hipGetLastError();
    }
    dim3 grid((N + block - 1) / block, BH);
    switch (block * D / 2048) {
        case 1: quant_block_kernel<D, 1, IS_K><<<grid, 256, 0, st>>>(xp, xq, scale, mean, sums, N, block, sm_scale); break;
        case 2: quant_block_kernel<D, 2, IS_K><<<grid, 256, 0, st>>>(xp, xq, scale, mean, sums, N, block, sm_scale); break;
        case 4: quant_block_kernel<D, 4, IS_K><<<grid, 256, 0, st>>>(xp, xq, scale, mean, sums, N, block, sm_scale); break;
        case 8: quant_block_kernel<D, 8, IS_K><<<grid, 256, 0, st>>>(xp, xq, scale, mean, sums, N, block, sm_scale); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_quant_q(const void* q, int8_t* qq, float* qscale, int BH, int N, int D,
                          float sm_scale, int block, hipStream_t st) {
    if (D == 64) return launch_quant<64, false>(q, qq, qscale, nullptr, nullptr, BH, N, block, sm_scale, st);
    return launch_quant<128, false>(q, qq, qscale, nullptr, nullptr, BH, N, block, sm_scale, st);
}

hipError_t launch_smooth_quant_k(const void* k, int8_t* kq, float* kscale, float* kmean,
                                 long long* sums, int BH, int N, int D, int block, hipStream_t st) {
    int n = BH * D;
    zero_sums_kernel<<<(n + 255) / 256, 256, 0, st>>>(sums, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (D == 64) {
        constexpr int CHUNK = (256 / 8) * 32;
        k_colsum_kernel<64><<<dim3((N + CHUNK - 1) / CHUNK, BH), 256, 0, st>>>((const _Float16*)k, sums, N);
    } else {
        constexpr int CHUNK = (256 / 16) * 32;
        k_colsum_kernel<128><<<dim3((N + CHUNK - 1) / CHUNK, BH), 256, 0, st>>>((const _Float16*)k, sums, N);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (D == 64) return launch_quant<64, true>(k, kq, kscale, kmean, sums, BH, N, block, 1.0f, st);
    return launch_quant<128, true>(k, kq, kscale, kmean, sums, BH, N, block, 1.0f, st);
}

}  // namespace sage
