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

// grid (ceil(N / CHUNK), BH); CHUNK = V_RPT rows per thread * (256 / (D/8)) row groups.
constexpr int V_RPT = 16;
template <int D>
__global__ void __launch_bounds__(256) v_absmax_kernel(const _Float16* __restrict__ v,
                                                       unsigned* __restrict__ amax_bits, int N) {
    constexpr int VPR = D / 8, RG = 256 / VPR, RPT = V_RPT, CHUNK = RG * RPT;
    const int t = threadIdx.x, c8 = t % VPR, rg = t / VPR;
    const int bh = blockIdx.y;
    const int row_base = blockIdx.x * CHUNK + rg;
    const _Float16* base = v + ((size_t)bh * N) * D;
    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = 0.0f;
    // all loads of a thread are issued before the first is used; a row past the end is fetched from
    // the last row instead, which leaves the maximum unchanged
    vh8 x[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int r = row_base + i * RG;
        x[i] = *(const vh8*)(base + (size_t)(r < N ? r : N - 1) * D + c8 * 8);
    }
    __builtin_amdgcn_sched_barrier(0);       // the fence that keeps the compiler from sinking each load to its use
#pragma unroll
    for (int i = 0; i < RPT; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) m[e] = __builtin_fmaxf(m[e], __builtin_fabsf((float)x[i][e]));
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

// grid (ceil(Np / ROWS), BH), ROWS = 64 (D = 128) or 128 (D = 64): one workgroup quantizes ROWS tokens
// x D channels and writes them transposed.  A thread owns 8 channels of 4 CONSECUTIVE tokens, so that
// the four codes of a channel leave as one 32-bit LDS store; the LDS rows are padded by one word,
// which spreads those stores over the banks.
template <int D>
__global__ void __launch_bounds__(256) v_quant_transpose_kernel(const _Float16* __restrict__ v,
                                                                const unsigned* __restrict__ amax_bits,
                                                                int8_t* __restrict__ vt, float* __restrict__ vscale,
                                                                int N, int Np) {
    constexpr int VPR = D / 8, G = 256 / VPR, ROWS = 4 * G, PITCH = ROWS + 4;      // LDS bytes per channel row
    const int t = threadIdx.x, c8 = t % VPR, g = t / VPR;
    const int bh = blockIdx.y, tile = blockIdx.x;
    const _Float16* base = v + ((size_t)bh * N) * D;
    __shared__ __attribute__((aligned(16))) int8_t tr[D * PITCH];

    float r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float amax = __uint_as_float(amax_bits[(size_t)bh * D + c8 * 8 + e]);
        r[e] = amax > 0.0f ? 127.0f / amax : 0.0f;
        if (tile == 0 && g == 0) vscale[(size_t)bh * D + c8 * 8 + e] = amax / 127.0f;
    }
    vh8 x[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = tile * ROWS + 4 * g + i;
        // rows past the end: fetched from the last row, then zeroed (no load sits behind a branch)
        x[i] = *(const vh8*)(base + (size_t)(row < N ? row : N - 1) * D + c8 * 8);
    }
    __builtin_amdgcn_sched_barrier(0);       // all four loads issued before the first is touched
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (tile * ROWS + 4 * g + i >= N) {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[i][e] = (_Float16)0.0f;
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        unsigned word = 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float q = __builtin_rintf((float)x[i][e] * r[e]);            // ties to even
            q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
            word |= ((unsigned)(int)q & 0xffu) << (8 * i);
        }
        *(unsigned*)(tr + (c8 * 8 + e) * PITCH + 4 * g) = word;
    }
    __syncthreads();
    // D rows of ROWS bytes = D * ROWS / 16 chunks of 16 bytes, two per thread
    constexpr int CPR = ROWS / 16;          // chunks per channel row
    int8_t* out = vt + ((size_t)bh * D) * Np + (size_t)tile * ROWS;
#pragma unroll
    for (int i = 0; i < (D * CPR) / 256; ++i) {
        const int idx = t + 256 * i, c = idx / CPR, part = idx % CPR;
        if (tile * ROWS + part * 16 < Np) {          // D = 64: the last 128-token tile may be half outside
            const unsigned* src = (const unsigned*)(tr + c * PITCH + part * 16);
            const int4 chunk = {(int)src[0], (int)src[1], (int)src[2], (int)src[3]};
            *(int4*)(out + (size_t)c * Np + part * 16) = chunk;
        }
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
        constexpr int CHUNK = (256 / 8) * V_RPT;
        v_absmax_kernel<64><<<dim3((N + CHUNK - 1) / CHUNK, BH), 256, 0, st>>>(vp, amax_bits, N);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        v_quant_transpose_kernel<64><<<dim3((Np + 127) / 128, BH), 256, 0, st>>>(vp, amax_bits, vt, vscale, N, Np);
    } else {
        constexpr int CHUNK = (256 / 16) * V_RPT;
        v_absmax_kernel<128><<<dim3((N + CHUNK - 1) / CHUNK, BH), 256, 0, st>>>(vp, amax_bits, N);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        v_quant_transpose_kernel<128><<<dim3(Np / 64, BH), 256, 0, st>>>(vp, amax_bits, vt, vscale, N, Np);
    }
    return hipGetLastError();
}

}  // namespace sage
