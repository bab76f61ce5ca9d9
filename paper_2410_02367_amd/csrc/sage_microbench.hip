// Instruction-stream probes for gfx950: what the matrix pipe sustains, alone and next to the softmax
// arithmetic of the attention kernel.  These are the ceilings the attention kernels are measured
// against (Section 5 of the SageAttention paper quotes its kernel against the peak of its GPU's INT8
// matrix unit; the same comparison here needs the rate this chip really sustains, not only the
// data-sheet figure).  The matrix instructions are the very statements of sage_attn.hip: inline
// assembly v_mfma_i32_32x32x32_i8 (Q^ K^^T) and v_mfma_f32_32x32x16_f16 (P~ V), operands in VGPRs.
//
// Every probe is one kernel: each wavefront repeats a fixed instruction group `iters` times on
// operands loaded from memory (random bytes: the power drawn, and with it the clock the chip holds,
// depends on how many bits toggle), brackets the loop with the shader-clock counter and the
// constant-rate counter, and leaves its accumulators' checksum so that nothing is optimized away.
//
//   kind 0  INT8 stream        8 x v_mfma_i32_32x32x32_i8 per group (4 independent accumulators)
//   kind 1  FP16 stream        8 x v_mfma_f32_32x32x16_f16 per group
//   kind 2  attention mix      8 INT8 + 16 FP16 instructions per group: the matrix work of one
//                              32-query x 64-key step at D = 128, no other instruction
//   kind 3  softmax stream     24 "chunks" per group, no matrix instruction; a chunk is the softmax of
//                              two scores: 2 fma, 2 exp2, 1 packed convert to FP16
//   kind 4  interleaved        8 x (FP16 matrix instruction + one chunk) per group, in ONE stream
//   kind 5  split by wavefront even wavefronts run kind 1's group, odd wavefronts 8 chunks per group
//                              (needs an even number of wavefronts per SIMD)
//   kind 6  step-shaped        the attention step's whole mix in one stream: 8 INT8 + 16 FP16 matrix
//                              instructions, each followed by its share of the 16 chunks + 8 3-way maxima
#include "sage_internal.h"

namespace sage {

typedef int mb_v4i __attribute__((ext_vector_type(4)));
typedef int mb_v16i __attribute__((ext_vector_type(16)));
typedef float mb_v16f __attribute__((ext_vector_type(16)));
typedef _Float16 mb_v8h __attribute__((ext_vector_type(8)));

__device__ __forceinline__ void mb_i8(mb_v16i& acc, const mb_v4i& a, const mb_v4i& b) {
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mb_f16(mb_v16f& acc, const mb_v8h& a, const mb_v8h& b) {
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

// The softmax of two scores, x -> FP16(exp2(x * sc + bias)), cut into the three stages the attention
// kernel runs in consecutive slots (fma | exp2 | pack), so that no instruction waits for the one
// before it: a tick packs chunk n - 2, exponentiates chunk n - 1 and starts chunk n -- exactly five
// VALU instructions.  Inputs and results pass through empty assembly statements, which keeps every
// instruction in place without adding any.
struct SoftmaxPipe {
    float xs[3][2];
    float in0, in1, sc, bias;
    __device__ __forceinline__ void tick(int n) {
        typedef float f2 __attribute__((ext_vector_type(2)));
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const int pk = (n + 1) % 3, ex = (n + 2) % 3, fm = n % 3;
        const f2 pp = {xs[pk][0], xs[pk][1]};
        const int p = __builtin_bit_cast(int, __builtin_convertvector(pp, h2));
        asm volatile("" : : "v"(p));
        xs[ex][0] = __builtin_amdgcn_exp2f(xs[ex][0]);
        xs[ex][1] = __builtin_amdgcn_exp2f(xs[ex][1]);
        asm volatile("" : "+v"(in0), "+v"(in1));
        xs[fm][0] = __builtin_fmaf(in0, sc, bias);
        xs[fm][1] = __builtin_fmaf(in1, sc, bias);
    }
};

template <int KIND>
__global__ void __launch_bounds__(512) microbench_kernel(const int* __restrict__ data, unsigned long long* __restrict__ out,
                                                         int iters) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    // wavefronts w and w + 4 of a workgroup share a SIMD
    const bool softmax_wave = KIND == 5 && (wave >> 2) % 2 == 1;

    mb_v4i a8 = *(const mb_v4i*)(data + 4 * lane), b8 = *(const mb_v4i*)(data + 256 + 4 * lane);
    // FP16 operands: random mantissas, exponents forced into [0.5, 2) so that nothing overflows
    mb_v4i ah = *(const mb_v4i*)(data + 512 + 4 * lane), bh = *(const mb_v4i*)(data + 768 + 4 * lane);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        ah[e] = (ah[e] & 0x83FF83FF) | 0x38003800;
        bh[e] = (bh[e] & 0x83FF83FF) | 0x38003800;
    }
    const mb_v8h af = __builtin_bit_cast(mb_v8h, ah), bf = __builtin_bit_cast(mb_v8h, bh);
    mb_v16i ci[4];
    mb_v16f cf[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) { ci[n][r] = 0; cf[n][r] = 0.0f; }
    SoftmaxPipe sp;
#pragma unroll
    for (int n = 0; n < 3; ++n) { sp.xs[n][0] = -0.25f * (float)(lane & 7); sp.xs[n][1] = -0.125f * (float)(lane & 15); }
    sp.in0 = -0.5f - (float)(lane & 3); sp.in1 = -0.75f; sp.sc = 1.001f; sp.bias = -0.5f;
    int mx = lane, mu = lane ^ 5, mv = 63 - lane;       // operands of the three-way maxima (never matrix results)

    __syncthreads();
    const unsigned long long t0 = __builtin_readcyclecounter(), r0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        if constexpr (KIND == 0) {
#pragma unroll
            for (int n = 0; n < 8; ++n) mb_i8(ci[n & 3], a8, b8);
        } else if constexpr (KIND == 1) {
#pragma unroll
            for (int n = 0; n < 8; ++n) mb_f16(cf[n & 3], af, bf);
        } else if constexpr (KIND == 2) {
#pragma unroll
            for (int n = 0; n < 8; ++n) mb_i8(ci[n & 3], a8, b8);
#pragma unroll
            for (int n = 0; n < 16; ++n) mb_f16(cf[n & 3], af, bf);
        } else if constexpr (KIND == 3) {
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                sp.tick(n);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if constexpr (KIND == 4) {
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                mb_f16(cf[n & 3], af, bf);
                sp.tick(n);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if constexpr (KIND == 5) {
            if (softmax_wave) {
#pragma unroll
                for (int n = 0; n < 8; ++n) {
                    sp.tick(n);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int n = 0; n < 8; ++n) mb_f16(cf[n & 3], af, bf);
            }
        } else {
            // 24 matrix instructions; chunks behind 16 of them, three-way integer maxima behind the other 8
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                if (n % 3 == 2) mb_i8(ci[n & 3], a8, b8);
                else mb_f16(cf[n & 3], af, bf);
                if (n % 3 != 2) sp.tick(n);
                else { asm volatile("" : "+v"(mu), "+v"(mv)); mx = max(max(mx, mu), mv); asm volatile("" : "+v"(mx)); }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    const unsigned long long t1 = __builtin_readcyclecounter(), r1 = wall_clock64();

    // checksum (keeps every accumulator alive); 12 wait states after the last matrix instruction
    asm volatile("s_nop 11" : "+v"(ci[0]), "+v"(ci[1]), "+v"(ci[2]), "+v"(ci[3]));
    asm volatile("s_nop 11" : "+v"(cf[0]), "+v"(cf[1]), "+v"(cf[2]), "+v"(cf[3]));
    float sum = 0.0f;
    int isum = mx;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { sum += cf[n][r]; isum ^= ci[n][r]; }
    }
    sum += sp.xs[0][0] + sp.xs[1][1] + sp.xs[2][0] + sp.in0;
    const size_t w = (size_t)blockIdx.x * nwaves + wave;
    if (lane == 0) {
        out[4 * w + 0] = t1 - t0;                 // shader-clock counter
        out[4 * w + 1] = r1 - r0;                 // constant-rate counter
        out[4 * w + 2] = (unsigned long long)(unsigned)isum;
    }
    if (sum == 123.456f) out[4 * w + 3] = 1;      // never true in practice; ties `sum` to memory
    else if (lane == 0) out[4 * w + 3] = 0;
}

hipError_t launch_microbench(int kind, int waves_per_simd, int workgroups, int iters, const int* data,
                             unsigned long long* out, hipStream_t st) {
    const int threads = 256 * waves_per_simd;
    switch (kind) {
        case 0: microbench_kernel<0><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 1: microbench_kernel<1><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 2: microbench_kernel<2><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 3: microbench_kernel<3><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 4: microbench_kernel<4><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 5: microbench_kernel<5><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 6: microbench_kernel<6><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sage
