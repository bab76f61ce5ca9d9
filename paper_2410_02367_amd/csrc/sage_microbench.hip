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
//   kind 7  LDS reads, 16 B    24 x ds_read_b128 per group (1 KB per wavefront each: a K^ operand), no other work
//   kind 8  LDS reads, transp. 48 x ds_read_b64_tr_b16 per group (two make one 1 KB V^T operand)
//   kind 9  step + operands    kind 6 with every matrix instruction's A operand read from LDS three
//                              instructions ahead, as the attention kernel does (8 x b128, 32 x tr_b16)
//   kind 10 small matrix instr 16 x v_mfma_f32_4x4x4_16b_f16 per group (the kernel's row-sum instruction)
//   kind 11 P~V with row sums  4 x (4 FP16 32x32x16 + 2 of the 4x4x4) per group, as the kernel issues them
//   kind 12 ... 16x16x32       4 x (4 FP16 32x32x16 + 1 v_mfma_f32_16x16x32_f16) per group
//   kind 13 ... 32x32x16       4 x (4 + 1 FP16 32x32x16) per group
//   kind 14 dependent chain    8 x INT8 32x32x32 into ONE accumulator (each instruction's C is the one before's D),
//                              as the four contraction steps of a K^ Q^^T block follow each other
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

typedef float mb_v4f __attribute__((ext_vector_type(4)));
typedef int mb_v2i __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void mb_small(mb_v4f& acc, const mb_v2i& a, const mb_v2i& b) {
    asm volatile("v_mfma_f32_4x4x4_16b_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
typedef int mb_v4i32 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void mb_mid_i8(mb_v4i32& acc, const mb_v4i& a, const mb_v4i& b) {
    asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mb_mid(mb_v4f& acc, const mb_v8h& a, const mb_v8h& b) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
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

typedef short mb_v4s __attribute__((ext_vector_type(4)));
#define MB_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))

// LDS byte offsets of the attention kernel's operand reads at D = 128 (64-key tiles, rows of 128 / 256
// bytes, 16-byte chunks XOR-swizzled by the row): K^ operand of 32-key half `half`, contraction step ks;
// first of the two 8-byte transposing reads of the V^T operand of 16-key group grp_su, channel block dt
// (the second lies 8 rows = 2048 bytes further).
__device__ __forceinline__ int k_operand_at(int lane, int half, int ks) {
    const int ql = lane & 31, g = lane >> 5;
    return half * 4096 + ql * 128 + (((2 * ks + g) ^ ((ql >> 1) & 7)) << 4);
}
__device__ __forceinline__ int v_operand_at(int lane, int grp_su, int dt) {
    const int grp = lane >> 4, li = lane & 15, v_row = 4 * (grp >> 1) + (li >> 2);
    const int chunk = (4 * dt + 2 * (grp & 1) + ((li & 3) >> 1)) ^ (4 * (v_row & 3));
    return 16 * grp_su * 256 + v_row * 256 + chunk * 16 + (li & 1) * 8;
}

template <int KIND>
__global__ void __launch_bounds__(512) microbench_kernel(const int* __restrict__ data, unsigned long long* __restrict__ out,
                                                         int iters) {
    // 48 KB: a 64-key K^ tile (8 KB) and V tile (16 KB) of the attention kernel at D = 128, twice
    __shared__ __attribute__((aligned(1024))) unsigned char tile[(KIND >= 7 && KIND <= 9) || KIND == 15 || KIND == 16 || KIND == 19 || KIND == 20 ? 49152 : 16];
    if constexpr ((KIND >= 7 && KIND <= 9) || KIND == 15 || KIND == 16 || KIND == 19 || KIND == 20) {
        for (int i = threadIdx.x; i < 49152 / 4; i += blockDim.x) ((int*)tile)[i] = data[i & 1023] & 0x3BFF3BFF;
    }
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
    mb_v4f cl[2] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
    mb_v4f cm[4] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
    mb_v4i32 cmi[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    mb_v4f cm2[4] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
    mb_v4i32 cmi2[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    mb_v4f cm3[4] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
    mb_v4f cm4[4] = {{0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}, {0.0f, 0.0f, 0.0f, 0.0f}};
    mb_v4i32 cmi3[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    mb_v4i32 cmi4[4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    const mb_v2i one2 = {0x3C003C00, 0x3C003C00}, bl = {ah[0], ah[1]}, bl2 = {ah[2], ah[3]};
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
        } else if constexpr (KIND == 19) {
            // Kind 15's step with the 16x16 instructions: every operand read from LDS feeds TWO matrix
            // instructions (two 16-query blocks), 32 FP16 16x16x32 + 16 INT8 16x16x64 + 4 row-sum instructions
            // per step -- the same operations, LDS reads, maxima and chunks as kind 15.
            mb_v4i ring[4];
            auto fetch = [&](int n) {
                if (n >= 16) {
                    ring[n & 3] = *(const mb_v4i*)(tile + k_operand_at(lane, (n - 16) >> 2, n & 3));
                } else {
                    const int at = 16384 + v_operand_at(lane, n >> 2, n & 3);
                    mb_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at));
                    mb_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at + 2048));
                    ring[n & 3] = __builtin_bit_cast(mb_v4i, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
            };
            if (it == 0) { fetch(0); fetch(1); fetch(2); }
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                if (n >= 16) {
                    mb_mid_i8(cmi[n & 3], ring[n & 3], b8);
                    mb_mid_i8(cmi2[n & 3], ring[n & 3], a8);
                } else {
                    mb_mid(cm[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), bf);
                    mb_mid(cm2[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), af);
                }
                fetch((n + 3) % 24);
                __builtin_amdgcn_sched_barrier(0);
                if (n < 4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { asm volatile("" : "+v"(mu), "+v"(mv)); mx = max(max(mx, mu), mv); asm volatile("" : "+v"(mx)); }
                } else if (n < 20) {
                    sp.tick(n - 4);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (n < 16 && n % 4 == 3) { mb_mid(cl[(n >> 2) & 1], af, bf); __builtin_amdgcn_sched_barrier(0); }
            }
        } else if constexpr (KIND == 20) {
            // Kind 19 for a wavefront of 64 queries: every operand read from LDS feeds FOUR 16x16 instructions,
            // the softmax work doubles (32 chunks, 32 maxima, 8 row-sum instructions), the LDS reads stay --
            // twice kind 15's operations per group.
            mb_v4i ring[4];
            auto fetch = [&](int n) {
                if (n >= 16) {
                    ring[n & 3] = *(const mb_v4i*)(tile + k_operand_at(lane, (n - 16) >> 2, n & 3));
                } else {
                    const int at = 16384 + v_operand_at(lane, n >> 2, n & 3);
                    mb_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at));
                    mb_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at + 2048));
                    ring[n & 3] = __builtin_bit_cast(mb_v4i, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
            };
            if (it == 0) { fetch(0); fetch(1); fetch(2); }
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                if (n >= 16) {
                    mb_mid_i8(cmi[n & 3], ring[n & 3], b8);
                    mb_mid_i8(cmi2[n & 3], ring[n & 3], a8);
                } else {
                    mb_mid(cm[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), bf);
                    mb_mid(cm2[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), af);
                }
                fetch((n + 3) % 24);
                __builtin_amdgcn_sched_barrier(0);
                if (n < 4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { asm volatile("" : "+v"(mu), "+v"(mv)); mx = max(max(mx, mu), mv); asm volatile("" : "+v"(mx)); }
                } else if (n < 20) {
                    sp.tick(2 * (n - 4));
                }
                __builtin_amdgcn_sched_barrier(0);
                if (n >= 16) {
                    mb_mid_i8(cmi3[n & 3], ring[n & 3], b8);
                    mb_mid_i8(cmi4[n & 3], ring[n & 3], a8);
                } else {
                    mb_mid(cm3[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), bf);
                    mb_mid(cm4[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), af);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (n < 4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { asm volatile("" : "+v"(mu), "+v"(mv)); mx = max(max(mx, mu), mv); asm volatile("" : "+v"(mx)); }
                } else if (n < 20) {
                    sp.tick(2 * (n - 4) + 1);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (n < 16 && n % 4 == 3) { mb_mid(cl[0], af, bf); mb_mid(cl[1], af, bf); __builtin_amdgcn_sched_barrier(0); }
            }
        } else if constexpr (KIND == 17) {
            // 16 of the 16x16x32 FP16 instruction (half the result block, twice the contraction depth of the
            // 32x32x16 one): the same 8 * 32768 operations as kind 1
#pragma unroll
            for (int n = 0; n < 16; ++n) mb_mid(cm[n & 3], af, bf);
        } else if constexpr (KIND == 18) {
            // 16 of the 16x16x64 INT8 instruction: the same 8 * 65536 operations as kind 0
#pragma unroll
            for (int n = 0; n < 16; ++n) mb_mid_i8(cmi[n & 3], a8, b8);
        } else if constexpr (KIND == 14) {
#pragma unroll
            for (int n = 0; n < 8; ++n) mb_i8(ci[0], a8, b8);
        } else if constexpr (KIND == 10) {
#pragma unroll
            for (int n = 0; n < 16; ++n) mb_small(cl[n & 1], one2, n & 1 ? bl2 : bl);
        } else if constexpr (KIND >= 11 && KIND <= 13) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
#pragma unroll
                for (int n = 0; n < 4; ++n) mb_f16(cf[n], af, bf);
                if constexpr (KIND == 11) { mb_small(cl[0], one2, bl); mb_small(cl[1], one2, bl2); }
                else if constexpr (KIND == 12) mb_mid(cl[g & 1], af, bf);
                else mb_f16(cf[g & 3], af, bf);
            }
        } else if constexpr (KIND == 7) {
            // the K^ operand reads of the attention kernel: 32-key half h, contraction step ks -> row lane % 32,
            // 16-byte chunk 2 ks + lane / 32, swizzled by the row
            mb_v4i r[4];
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                r[n & 3] = *(const mb_v4i*)(tile + k_operand_at(lane, (n >> 2) & 1, n & 3) + (n >> 3) * 8192);
                asm volatile("" : : "v"(r[n & 3]));
            }
        } else if constexpr (KIND == 8) {
            // the V^T operand reads: two transposing 8-byte reads per operand
            mb_v4s r[4];
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                const int at = 16384 + v_operand_at(lane, (n >> 2) & 3, n & 3) + (n >> 4) * 8192;      // all inside the 48 KB
                r[n & 3] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at));
                asm volatile("" : : "v"(r[n & 3]));
                r[(n + 2) & 3] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at + 2048));
                asm volatile("" : : "v"(r[(n + 2) & 3]));
            }
        } else if constexpr (KIND == 9) {
            mb_v4i ring[4];
            auto fetch = [&](int n) {          // operand of matrix instruction n of the group
                if (n % 3 == 2) {
                    const int q = n / 3;                             // index among the 8 INT8 instructions
                    ring[n & 3] = *(const mb_v4i*)(tile + k_operand_at(lane, q >> 2, q & 3));
                } else {
                    const int m = n - n / 3;                         // index among the 16 FP16 instructions
                    const int at = 16384 + v_operand_at(lane, m >> 2, m & 3);
                    mb_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at));
                    mb_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at + 2048));
                    ring[n & 3] = __builtin_bit_cast(mb_v4i, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
            };
            if (it == 0) { fetch(0); fetch(1); fetch(2); }
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                if (n % 3 == 2) mb_i8(ci[n & 3], ring[n & 3], b8);
                else mb_f16(cf[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), bf);
                fetch((n + 3) % 24);
                __builtin_amdgcn_sched_barrier(0);
                if (n % 3 != 2) sp.tick(n);
                else { asm volatile("" : "+v"(mu), "+v"(mv)); mx = max(max(mx, mu), mv); asm volatile("" : "+v"(mx)); }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if constexpr (KIND == 15 || KIND == 16) {
            // The attention kernel's own order at D = 128: 16 FP16 instructions (V^T operands) with a row-sum
            // instruction after every fourth, then 8 INT8 ones (K^ operands); every operand read from LDS 3
            // ahead; the 16 three-way maxima of the row maximum behind the first 4.  Kind 15 puts the 16
            // softmax chunks behind instructions 4 .. 19, as the kernel must while the scores of one tile
            // live in one set of registers (the last 8 instructions overwrite them); kind 16 spreads them
            // over instructions 4 .. 23, which a second set of score registers would allow.
            mb_v4i ring[4];
            auto fetch = [&](int n) {
                if (n >= 16) {
                    ring[n & 3] = *(const mb_v4i*)(tile + k_operand_at(lane, (n - 16) >> 2, n & 3));
                } else {
                    const int at = 16384 + v_operand_at(lane, n >> 2, n & 3);
                    mb_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at));
                    mb_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(MB_LDS(mb_v4s, tile + at + 2048));
                    ring[n & 3] = __builtin_bit_cast(mb_v4i, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
            };
            if (it == 0) { fetch(0); fetch(1); fetch(2); }
            constexpr int LAST = KIND == 15 ? 20 : 24;          // chunks behind instructions 4 .. LAST - 1
#pragma unroll
            for (int n = 0; n < 24; ++n) {
                if (n >= 16) mb_i8(ci[n & 3], ring[n & 3], b8);
                else mb_f16(cf[n & 3], __builtin_bit_cast(mb_v8h, ring[n & 3]), bf);
                fetch((n + 3) % 24);
                __builtin_amdgcn_sched_barrier(0);
                if (n < 4) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { asm volatile("" : "+v"(mu), "+v"(mv)); mx = max(max(mx, mu), mv); asm volatile("" : "+v"(mx)); }
                } else if (n < LAST) {
                    const int first = (n - 4) * 16 / (LAST - 4), end = (n - 3) * 16 / (LAST - 4);
#pragma unroll
                    for (int c = first; c < end; ++c) sp.tick(c);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (n < 16 && n % 4 == 3) { mb_mid(cl[(n >> 2) & 1], af, bf); __builtin_amdgcn_sched_barrier(0); }
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
    asm volatile("s_nop 11" : "+v"(cl[0]), "+v"(cl[1]));
    asm volatile("s_nop 11" : "+v"(cm[0]), "+v"(cm[1]), "+v"(cm[2]), "+v"(cm[3]));
    asm volatile("s_nop 11" : "+v"(cmi[0]), "+v"(cmi[1]), "+v"(cmi[2]), "+v"(cmi[3]));
    asm volatile("s_nop 11" : "+v"(cm2[0]), "+v"(cm2[1]), "+v"(cm2[2]), "+v"(cm2[3]));
    asm volatile("s_nop 11" : "+v"(cmi2[0]), "+v"(cmi2[1]), "+v"(cmi2[2]), "+v"(cmi2[3]));
    asm volatile("s_nop 11" : "+v"(cm3[0]), "+v"(cm3[1]), "+v"(cm3[2]), "+v"(cm3[3]));
    asm volatile("s_nop 11" : "+v"(cm4[0]), "+v"(cm4[1]), "+v"(cm4[2]), "+v"(cm4[3]));
    asm volatile("s_nop 11" : "+v"(cmi3[0]), "+v"(cmi3[1]), "+v"(cmi3[2]), "+v"(cmi3[3]));
    asm volatile("s_nop 11" : "+v"(cmi4[0]), "+v"(cmi4[1]), "+v"(cmi4[2]), "+v"(cmi4[3]));
    float sum = cl[0][0] + cl[1][0] + cl[0][3] + cl[1][2] + cm[0][0] + cm[1][1] + cm[2][2] + cm[3][3] + cm2[0][0] + cm2[1][1] + cm2[2][2] + cm2[3][3]
                + cm3[0][0] + cm3[1][1] + cm3[2][2] + cm3[3][3] + cm4[0][0] + cm4[1][1] + cm4[2][2] + cm4[3][3];
    int isum = mx ^ cmi[0][0] ^ cmi[1][1] ^ cmi[2][2] ^ cmi[3][3] ^ cmi2[0][0] ^ cmi2[1][1] ^ cmi2[2][2] ^ cmi2[3][3]
               ^ cmi3[0][0] ^ cmi3[1][1] ^ cmi3[2][2] ^ cmi3[3][3] ^ cmi4[0][0] ^ cmi4[1][1] ^ cmi4[2][2] ^ cmi4[3][3];
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
        case 7: microbench_kernel<7><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 8: microbench_kernel<8><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 9: microbench_kernel<9><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 10: microbench_kernel<10><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 11: microbench_kernel<11><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 12: microbench_kernel<12><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 13: microbench_kernel<13><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 14: microbench_kernel<14><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 15: microbench_kernel<15><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 16: microbench_kernel<16><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 17: microbench_kernel<17><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 18: microbench_kernel<18><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 19: microbench_kernel<19><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        case 20: microbench_kernel<20><<<workgroups, threads, 0, st>>>(data, out, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sage
