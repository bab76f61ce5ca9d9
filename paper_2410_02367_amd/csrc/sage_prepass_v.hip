// Per-channel INT8 quantizer of V for the kernels with an INT8 second product (Section 4.3:
// psi_V per channel; Section 3.2 gives the per-channel quantizer) -- HBM-bound kernels for gfx950.
//
//   per-channel absolute maximum over all tokens of a (batch, head) slab  -> delta_V[c] = amax / 127
//   V^[t,c] = clamp(rne(V[t,c] * fl32(127 / amax_c)), -127, 127)          -> stored TRANSPOSED,
//   channel-major [D][Np] with Np = 64 * ceil(N / 64), tokens past N as code 0
//
// Channel-major is what the attention kernel wants: the A operand of the INT8 matrix instruction
// of O^T = V^^T P^^T is 16 consecutive TOKENS of one channel, i.e. one 16-byte read of a row of V^^T.
// The maximum of non-negative floats is the maximum of their bit patterns, so it is order-free and
// atomicMax on the bits gives the same result however the tokens are split over workgroups.
#include "sage_internal.h"
#include <hip/hip_fp16.h>

namespace sage {

typedef _Float16 vh8 __attribute__((ext_vector_type(8)));

__global__ void __launch_bounds__(256) zero_words_kernel(unsigned* w, int n) {
    int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) w[i] = 0u;
}

// grid (ceil(N / CHUNK), BH); CHUNK = 32 rows per thread * (256 / (D/8)) row groups.
template <int D>
__global__ void __launch_bounds__(256) v_absmax_kernel(const _Float16* __restrict__ v,
                                                       unsigned* __restrict__ amax_bits, int N) {
    constexpr int VPR = D / 8, RG = 256 / VPR, RPT = 32, CHUNK = RG * RPT;
    const int t = threadIdx.x, c8 = t % VPR, rg = t / VPR;
    const int bh = blockIdx.y;
    const int row_base = blockIdx.x * CHUNK + rg;
    const _Float16* base = v + ((size_t)bh * N) * D;
    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = 0.0f;
#pragma unroll 8
    for (int i = 0; i < RPT; ++i) {
        const int r = row_base + i * RG;
        if (r < N) {
            const vh8 x = *(const vh8*)(base + (size_t)r * D + c8 * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) m[e] = __builtin_fmaxf(m[e], __builtin_fabsf((float)x[e]));
        }
    }
    __shared__ float part[RG][D];
#pragma unroll
    for (int e = 0; e < 8; ++e) part[rg][c8 * 8 + e] = m[e];
    __syncthreads();
    if (t < D) {
        float s = 0.0f;
#pragma unroll 4
        for (int g = 0; g < RG; ++g) s = __builtin_fmaxf(s, part[g][t]);
        atomicMax(amax_bits + (size_t)bh * D + t, __float_as_uint(s));
    }
}

// grid (Np / 64, BH): one workgroup quantizes 64 tokens x D channels and writes them transposed.
template <int D>
__global__ void __launch_bounds__(256) v_quant_transpose_kernel(const _Float16* __restrict__ v,
                                                                const unsigned* __restrict__ amax_bits,
                                                                int8_t* __restrict__ vt, float* __restrict__ vscale,
                                                                int N, int Np) {
    constexpr int VPR = D / 8, RG = 256 / VPR, ROWS = 64, PITCH = 80;      // LDS bytes per channel row (16-byte aligned)
    const int t = threadIdx.x, c8 = t % VPR, rg = t / VPR;
    const int bh = blockIdx.y, tile = blockIdx.x;
    const _Float16* base = v + ((size_t)bh * N) * D;
    __shared__ __attribute__((aligned(16))) int8_t tr[D * PITCH];

    float r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float amax = __uint_as_float(amax_bits[(size_t)bh * D + c8 * 8 + e]);
        r[e] = amax > 0.0f ? 127.0f / amax : 0.0f;
        if (tile == 0 && rg == 0) vscale[(size_t)bh * D + c8 * 8 + e] = amax / 127.0f;
    }
#pragma unroll
    for (int i = 0; i < ROWS / RG; ++i) {
        const int lr = rg + i * RG, row = tile * ROWS + lr;
        vh8 x;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (_Float16)0.0f;
        if (row < N) x = *(const vh8*)(base + (size_t)row * D + c8 * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float q = __builtin_rintf((float)x[e] * r[e]);            // ties to even
            q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
            tr[(c8 * 8 + e) * PITCH + lr] = (int8_t)(int)q;
        }
    }
    __syncthreads();
    // D rows of 64 bytes = 4 * D chunks of 16 bytes
    int8_t* out = vt + ((size_t)bh * D) * Np + (size_t)tile * ROWS;
#pragma unroll
    for (int i = 0; i < (4 * D) / 256; ++i) {
        const int idx = t + 256 * i, c = idx >> 2, part = idx & 3;
        const int4 chunk = *(const int4*)(tr + c * PITCH + part * 16);
        *(int4*)(out + (size_t)c * Np + part * 16) = chunk;
    }
}

hipError_t launch_quant_v(const void* v, int8_t* vt, float* vscale, unsigned* amax_bits,
                          int BH, int N, int D, hipStream_t st) {
    const int n = BH * D, Np = 64 * ((N + 63) / 64);
    zero_words_kernel<<<(n + 255) / 256, 256, 0, st>>>(amax_bits, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const _Float16* vp = (const _Float16*)v;
    if (D == 64) {
        constexpr int CHUNK = (256 / 8) * 32;
        v_absmax_kernel<64><<<dim3((N + CHUNK - 1) / CHUNK, BH), 256, 0, st>>>(vp, amax_bits, N);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        v_quant_transpose_kernel<64><<<dim3(Np / 64, BH), 256, 0, st>>>(vp, amax_bits, vt, vscale, N, Np);
    } else {
        constexpr int CHUNK = (256 / 16) * 32;
        v_absmax_kernel<128><<<dim3((N + CHUNK - 1) / CHUNK, BH), 256, 0, st>>>(vp, amax_bits, N);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        v_quant_transpose_kernel<128><<<dim3(Np / 64, BH), 256, 0, st>>>(vp, amax_bits, vt, vscale, N, Np);
    }
    return hipGetLastError();
}

}  // namespace sage
