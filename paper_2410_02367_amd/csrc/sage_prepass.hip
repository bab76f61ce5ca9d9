// Smooth-and-quantize pre-pass of SageAttention for gfx950 (HBM-bound kernels).
//
//   column sums of K over tokens      -> exact integer arithmetic (Section 4.2, mean(K))
//   K - mean(K), per-block absmax,    -> Section 4.2 (gamma) + Section 3.2 (per-block psi)
//   INT8 pack
//   Q * sm_scale, per-block absmax,   -> Section 4.6 (scale folded into Q) + Section 3.2
//   INT8 pack
//   optionally RoPE applied on the fly -> Section 4.6 (quantizer fused into the producer of Q, K)
//
// Every fp16 value is an integer multiple of 2^-24, so the column sum is accumulated as an
// integer count of 2^-24 units; the result does not depend on how tokens are split over
// threads and workgroups.  One fp64 division and one rounding to fp32 give the mean.
// The K side is two launches: partial column sums per chunk of tokens, then the quantizer, whose
// workgroups add the partial sums of their slab (no clearing pass, no atomics).
#include "sage_internal.h"
#include <hip/hip_fp16.h>

namespace sage {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));

// The 8 channels 8*c8 .. 8*c8+7 of one token row (fp16 [D]).  With ROPE the row passes through the
// rotary embedding first (Section 4.6: the quantizer is fused into the operator that produces Q
// and K): channel c < D/2 is paired with c + D/2,
//     y[c] = x[c] cos[c] - x[c+D/2] sin[c],    y[c+D/2] = x[c+D/2] cos[c] + x[c] sin[c],
// every product and the sum rounded to fp32, y rounded to fp16 -- the tensor an unfused RoPE kernel
// would have stored, so that the fused pre-pass returns exactly what the unfused one returns.
// cos_row / sin_row point at the D/2 fp32 table entries of the token's position.  The partner
// chunk is a second 16-byte load from the same cache line(s).
// The loads and the arithmetic are separate steps (fetch_row8 / finish_row8), so that a kernel can have
// the loads of several rows in flight before it rotates the first one.
template <bool ROPE> struct RowRaw;
template <> struct RowRaw<false> { h8 own; };
template <> struct RowRaw<true> { h8 own, partner; float4 c0, c1, s0, s1; };

template <int D, bool ROPE>
__device__ __forceinline__ RowRaw<ROPE> fetch_row8(const _Float16* __restrict__ row, int c8,
                                                   const float* __restrict__ cos_row, const float* __restrict__ sin_row) {
    RowRaw<ROPE> r;
    r.own = *(const h8*)(row + c8 * 8);
    if constexpr (ROPE) {
        constexpr int HALF = D / 2;
        const int c = c8 * 8;
        const bool upper = c >= HALF;
        const int cp = upper ? c - HALF : c + HALF, ct = upper ? c - HALF : c;
        r.partner = *(const h8*)(row + cp);
        r.c0 = *(const float4*)(cos_row + ct); r.c1 = *(const float4*)(cos_row + ct + 4);
        r.s0 = *(const float4*)(sin_row + ct); r.s1 = *(const float4*)(sin_row + ct + 4);
    }
    return r;
}
template <int D, bool ROPE>
__device__ __forceinline__ h8 finish_row8(const RowRaw<ROPE>& r, int c8) {
    if constexpr (!ROPE) {
        return r.own;
    } else {
        const bool upper = c8 * 8 >= D / 2;
        const float cs[8] = {r.c0.x, r.c0.y, r.c0.z, r.c0.w, r.c1.x, r.c1.y, r.c1.z, r.c1.w};
        const float sn[8] = {r.s0.x, r.s0.y, r.s0.z, r.s0.w, r.s1.x, r.s1.y, r.s1.z, r.s1.w};
        h8 y;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float oc = (float)r.own[e] * cs[e], ps = (float)r.partner[e] * sn[e];
            y[e] = (_Float16)(upper ? oc + ps : oc - ps);
        }
        return y;
    }
}
// rows in flight per thread where a kernel batches them: a fetched row is 4 registers, 24 with RoPE
template <bool ROPE> constexpr int rows_in_flight(int plain) { return ROPE ? (plain < 4 ? plain : 4) : plain; }

// Exact column sums, first level: the workgroup (chunk p, slab bh) of grid (P, BH) sums the rows
// p * chunk .. of its slab and leaves the D sums as 64-bit integers at part[(bh * P + p) * D ..];
// the quantizer kernels add the P partial sums of their slab themselves (integer addition: any order
// gives the same bits).  No atomics, nothing to clear beforehand, every word of the result written.
// A thread owns one 16-byte column group of every RG-th row and fetches BATCH rows at a time, all loads
// issued before the first is used (rows past the end are fetched from the last row and not added).
// (The kernels of this file are written as bodies that take their workgroup coordinates -- chunk or
// group index bx of gx, slab bh -- as arguments, so that two of them can share one launch: see
// "One launch for two jobs" below.)
template <int D, bool ROPE, int NT = 256>
__device__ __forceinline__ void k_colsum_body(const _Float16* __restrict__ k,
                                              long long* __restrict__ part_out, int N, int chunk,
                                              const float* __restrict__ cs, const float* __restrict__ sn,
                                              int bx, int P, int bh) {
    constexpr int VPR = D / 8;          // 16-byte vectors per token row
    constexpr int RG = NT / VPR;        // row groups per workgroup
    constexpr int BATCH = rows_in_flight<ROPE>(8);      // rows per thread in flight
    const int t = threadIdx.x, c8 = t % VPR, rg = t / VPR;
    const int row_begin = bx * chunk;
    const int row_end = row_begin + chunk < N ? row_begin + chunk : N;
    const _Float16* base = k + ((size_t)bh * N) * D;

    // A thread's partial sums are carried in fp64: every fp16 value is a multiple of 2^-24 below 2^16 in
    // magnitude, a thread adds at most 2^13 of them (chunk <= 2^17 rows, RG >= 16 row groups), so every
    // intermediate sum is a multiple of 2^-24 below 2^29 -- 53 bits, exact in fp64.  Three VALU
    // instructions per element (two conversions, one addition) instead of eight for an integer split,
    // which is what lets this kernel run at the memory rate.
    static_assert(RG >= 16, "at most 2^13 rows per thread in a chunk of 2^17");
    double acc_d[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc_d[e] = 0.0;
    // whole batches first (no row needs a check: every chunk but a slab's last is whole batches), then
    // at most one ragged batch whose rows past the end are fetched from the last row and not added
    const int whole = row_begin + (row_end - row_begin) / (BATCH * RG) * (BATCH * RG);
    for (int r0 = row_begin + rg; r0 < whole; r0 += BATCH * RG) {
        RowRaw<ROPE> xr[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int r = r0 + i * RG;
            xr[i] = fetch_row8<D, ROPE>(base + (size_t)r * D, c8, cs + (size_t)r * (D / 2), sn + (size_t)r * (D / 2));
        }
        // every load of the batch is issued before the first is used: without this fence the compiler's
        // scheduler sinks each load to its use -- one load in flight instead of eight, a third slower
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const h8 x = finish_row8<D, ROPE>(xr[i], c8);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc_d[e] += (double)(float)x[e];
        }
    }
    if (whole < row_end) {
        RowRaw<ROPE> xr[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int r = whole + rg + i * RG;
            const int rc = r < row_end ? r : row_end - 1;
            xr[i] = fetch_row8<D, ROPE>(base + (size_t)rc * D, c8, cs + (size_t)rc * (D / 2), sn + (size_t)rc * (D / 2));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const double live = whole + rg + i * RG < row_end ? 1.0 : 0.0;
            const h8 x = finish_row8<D, ROPE>(xr[i], c8);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc_d[e] += live * (double)(float)x[e];
        }
    }
    // exact conversion to a count of 2^-24 units: |v| < 2^53 is split into a 27-bit and a 26-bit part
    long long acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const double v = acc_d[e] * 16777216.0;
        const double hi = __builtin_trunc(v * 0x1p-26);
        const double lo = v - hi * 0x1p26;
        acc[e] = (long long)(int)hi * (1ll << 26) + (long long)(int)lo;
    }
    __shared__ long long part[RG][D];
#pragma unroll
    for (int e = 0; e < 8; ++e) part[rg][c8 * 8 + e] = acc[e];
    __syncthreads();
    if (t < D) {
        long long s = 0;
#pragma unroll 4
        for (int g = 0; g < RG; ++g) s += part[g][t];
        part_out[((size_t)bh * P + bx) * D + t] = s;
    }
}
template <int D, bool ROPE>
__global__ void __launch_bounds__(256) k_colsum_kernel(const _Float16* __restrict__ k,
                                                       long long* __restrict__ part_out, int N, int chunk,
                                                       const float* __restrict__ cs, const float* __restrict__ sn) {
    k_colsum_body<D, ROPE>(k, part_out, N, chunk, cs, sn, blockIdx.x, gridDim.x, blockIdx.y);
}

// mean[c] of a slab from its P partial column sums: exact integer total, one fp64 division, one
// rounding to fp32 (thread c < D of the workgroup; the others return 0).
template <int D>
__device__ __forceinline__ float slab_mean(const long long* __restrict__ parts, int bh, int P, int N, int c) {
    if (c >= D) return 0.0f;
    const long long* p = parts + (size_t)bh * P * D + c;
    long long s = 0;
#pragma unroll 4
    for (int i = 0; i < P; ++i) s += p[(size_t)i * D];
    const double avg = (double)s / (double)N;
    return (float)(avg * 0x1p-24);
}

template <int NT = 256>
__device__ __forceinline__ float wg_max(float v, float* red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = __builtin_fmaxf(v, __shfl_xor(v, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float m = red[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) m = __builtin_fmaxf(m, red[w]);
    return m;
}

// Per-block quantizer: a workgroup of NT threads takes quantization blocks g = blockIdx.x,
// blockIdx.x + gridDim.x, ... of its slab, one at a time; a block is `block` tokens x D channels,
// block * D = 8 * NT * LPT.  IS_K: x - mean (the mean formed once per workgroup from the partial
// column sums -- which is why a workgroup walks several blocks); else x * sm_scale.  All LPT loads
// of a block are issued before the first is used (rows past the end of the block are fetched from
// its last row and ignored).
template <int D, int LPT, bool IS_K, bool ROPE, int NT = 256>
__device__ __forceinline__ void quant_block_body(const _Float16* __restrict__ x,
                                                 int8_t* __restrict__ xq,
                                                 float* __restrict__ scale,
                                                 float* __restrict__ k_mean,
                                                 const long long* __restrict__ parts, int P,
                                                 int N, int block, float sm_scale,
                                                 const float* __restrict__ cs, const float* __restrict__ sn,
                                                 int bx, int gx, int bh) {
    constexpr int VPR = D / 8;
    constexpr int RSTEP = NT / VPR;
    const int t = threadIdx.x, c8 = t % VPR, rbase = t / VPR;
    const int nblk = (N + block - 1) / block;

    __shared__ float s_mean[D];
    __shared__ float s_red[2][NT / 64];
    // the LPT rows of block g that this thread owns (rows past the end of the block: its last row)
    auto fetch_block = [&](int g, RowRaw<ROPE> (&dst)[LPT]) {
        const int row0 = g * block;
        const int rows = (N - row0 < block) ? (N - row0) : block;
        const _Float16* xb = x + ((size_t)bh * N + row0) * D;
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int r = rbase + i * RSTEP;
            const int rc = r < rows ? r : rows - 1;
            dst[i] = fetch_row8<D, ROPE>(xb + (size_t)rc * D, c8, cs + (size_t)(row0 + rc) * (D / 2),
                                         sn + (size_t)(row0 + rc) * (D / 2));
        }
        __builtin_amdgcn_sched_barrier(0);       // all loads of the block issued here, none sunk to its use
    };
    static_assert(!ROPE || LPT <= 4, "a fetched row is 24 registers with RoPE");
    RowRaw<ROPE> ahead[LPT];       // the loads of the block after the current one (or of the first)
    h8 raw[LPT];                   // the current block's rows, rotated if ROPE
    int g = bx;                    // the launcher never starts more workgroups than there are blocks
    fetch_block(g, ahead);         // in flight while the mean is formed

    float mean[8];
    if (IS_K) {
        if (t < D) {
            const float m = slab_mean<D>(parts, bh, P, N, t);
            s_mean[t] = m;
            if (bx == 0 && k_mean != nullptr) k_mean[(size_t)bh * D + t] = m;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) mean[e] = s_mean[c8 * 8 + e];
    }
#pragma unroll
    for (int i = 0; i < LPT; ++i) raw[i] = finish_row8<D, ROPE>(ahead[i], c8);

    for (int turn = 0; g < nblk; g += gx, turn ^= 1) {
        const int row0 = g * block;
        const int rows = (N - row0 < block) ? (N - row0) : block;
        const size_t slab = ((size_t)bh * N + row0) * D + c8 * 8;
        // the next block of this workgroup is requested before this one is reduced and stored
        const bool more = g + gx < nblk;
        if (more) fetch_block(g + gx, ahead);
        float amax = 0.0f;
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {       // a clamped row repeats a row of the block: the maximum is unchanged
                float f = (float)raw[i][e];
                f = IS_K ? (f - mean[e]) : (f * sm_scale);
                amax = __builtin_fmaxf(amax, __builtin_fabsf(f));
            }
        }
        amax = wg_max<NT>(amax, s_red[turn]);       // alternating buffers: one barrier per block is enough
        const float delta = amax / 127.0f;
        const float rcp = amax > 0.0f ? 127.0f / amax : 0.0f;
        if (t == 0) scale[(size_t)bh * nblk + g] = delta;

#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int r = rbase + i * RSTEP;
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
        if (more) {
#pragma unroll
            for (int i = 0; i < LPT; ++i) raw[i] = finish_row8<D, ROPE>(ahead[i], c8);
        }
    }
}
template <int D, int LPT, bool IS_K, bool ROPE, int NT = 256>
__global__ void __launch_bounds__(NT) quant_block_kernel(const _Float16* __restrict__ x, int8_t* __restrict__ xq,
                                                          float* __restrict__ scale, float* __restrict__ k_mean,
                                                          const long long* __restrict__ parts, int P,
                                                          int N, int block, float sm_scale,
                                                          const float* __restrict__ cs, const float* __restrict__ sn) {
    quant_block_body<D, LPT, IS_K, ROPE, NT>(x, xq, scale, k_mean, parts, P, N, block, sm_scale, cs, sn,
                                             blockIdx.x, gridDim.x, blockIdx.y);
}

// Per-token quantizer (Section 3.2): one scale per token row.  D/8 adjacent lanes own a row
// (16 bytes each); the row's absmax is a butterfly over those lanes.  A workgroup takes groups of
// TOK_ROWS consecutive tokens (group blockIdx.x, blockIdx.x + gridDim.x, ...), TOK_LPT rows per
// thread, all loads of a group issued before the first use (rows past N fetched from row N - 1 and
// not stored).
constexpr int TOK_LPT = 8;
template <int D, bool IS_K, bool ROPE>
__device__ __forceinline__ void quant_token_body(const _Float16* __restrict__ x,
                                                 int8_t* __restrict__ xq,
                                                 float* __restrict__ scale,
                                                 float* __restrict__ k_mean,
                                                 const long long* __restrict__ parts, int P,
                                                 int N, float sm_scale,
                                                 const float* __restrict__ cs, const float* __restrict__ sn,
                                                 int bx, int gx, int bh) {
    constexpr int VPR = D / 8;
    constexpr int RSTEP = 256 / VPR;
    constexpr int ROWS = RSTEP * TOK_LPT;
    const int t = threadIdx.x, c8 = t % VPR, rbase = t / VPR;
    const int ngrp = (N + ROWS - 1) / ROWS;

    __shared__ float s_mean[D];
    float mean[8];
    if (IS_K) {
        if (t < D) {
            const float m = slab_mean<D>(parts, bh, P, N, t);
            s_mean[t] = m;
            if (bx == 0 && k_mean != nullptr) k_mean[(size_t)bh * D + t] = m;
        }
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) mean[e] = s_mean[c8 * 8 + e];
    }

    for (int grp = bx; grp < ngrp; grp += gx) {
        const int row0 = grp * ROWS;
        const _Float16* xs = x + (size_t)bh * N * D;
        constexpr int SUB = rows_in_flight<ROPE>(TOK_LPT);     // rows fetched together
#pragma unroll
        for (int i0 = 0; i0 < TOK_LPT; i0 += SUB) {
        RowRaw<ROPE> fetched[SUB];
#pragma unroll
        for (int i = 0; i < SUB; ++i) {
            const int r = row0 + rbase + (i0 + i) * RSTEP;
            const int rc = r < N ? r : N - 1;
            fetched[i] = fetch_row8<D, ROPE>(xs + (size_t)rc * D, c8, cs + (size_t)rc * (D / 2), sn + (size_t)rc * (D / 2));
        }
        __builtin_amdgcn_sched_barrier(0);       // all loads of the batch issued here, none sunk to its use
#pragma unroll
        for (int i = 0; i < SUB; ++i) {
            const int r = row0 + rbase + (i0 + i) * RSTEP;
            const h8 raw = finish_row8<D, ROPE>(fetched[i], c8);
            float f[8];
            float amax = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                f[e] = (float)raw[e];
                f[e] = IS_K ? (f[e] - mean[e]) : (f[e] * sm_scale);
                amax = __builtin_fmaxf(amax, __builtin_fabsf(f[e]));
            }
#pragma unroll
            for (int off = VPR / 2; off >= 1; off >>= 1) amax = __builtin_fmaxf(amax, __shfl_xor(amax, off, 64));
            const float delta = amax / 127.0f;
            const float rcp = amax > 0.0f ? 127.0f / amax : 0.0f;
            if (r < N) {
                if (c8 == 0) scale[(size_t)bh * N + r] = delta;
                unsigned w[2] = {0u, 0u};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float q = __builtin_rintf(f[e] * rcp);                 // round half to even
                    q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
                    w[e >> 2] |= ((unsigned)((int)q) & 0xffu) << (8 * (e & 3));
                }
                *(uint2*)(xq + ((size_t)bh * N + r) * D + c8 * 8) = make_uint2(w[0], w[1]);
            }
        }
        }
    }
}
template <int D, bool IS_K, bool ROPE>
__global__ void __launch_bounds__(256) quant_token_kernel(const _Float16* __restrict__ x, int8_t* __restrict__ xq,
                                                          float* __restrict__ scale, float* __restrict__ k_mean,
                                                          const long long* __restrict__ parts, int P,
                                                          int N, float sm_scale,
                                                          const float* __restrict__ cs, const float* __restrict__ sn) {
    quant_token_body<D, IS_K, ROPE>(x, xq, scale, k_mean, parts, P, N, sm_scale, cs, sn, blockIdx.x, gridDim.x, blockIdx.y);
}

// Short sequences (N <= SMALL_N): the whole K pre-pass of one (batch, head) slab in ONE workgroup
// and one launch.  The slab is read ONCE, all loads in flight together, and stays in registers
// (at most SMALL_N / RG rows of 16 bytes per thread): exact column sums, mean, per-block (or
// per-token) maxima and the quantization all work on those registers -- one memory round trip, two
// barriers.  The results are the same bits as the wide kernels' (the integer sum does not depend on
// how it is split).  Beyond a few blocks per slab one workgroup per slab loses against the wide
// launches (measured: faster at N = 197, slower at N = 1105), hence the low limit.
constexpr int SMALL_N = 512;
template <int D, bool ROPE>
__device__ __forceinline__ void k_small_body(const _Float16* __restrict__ k,
                                             int8_t* __restrict__ kq,
                                             float* __restrict__ scale,
                                             float* __restrict__ k_mean,
                                             int N, int block,
                                             const float* __restrict__ cs, const float* __restrict__ sn, int bh) {
    constexpr int VPR = D / 8;
    constexpr int RG = 256 / VPR;
    constexpr int HALF = D / 2;
    constexpr int MAXR = SMALL_N / RG;        // rows per thread: row rg + i * RG in register set i
    constexpr int MAXB = SMALL_N / 32;        // blocks per slab at the smallest block size
    const int t = threadIdx.x, c8 = t % VPR, rg = t / VPR;
    const _Float16* base = k + ((size_t)bh * N) * D;

    __shared__ long long part[RG][D];
    __shared__ float s_mean[D];
    __shared__ float s_red[MAXB][4];

    // register sets 0 .. nset - 1 hold rows (a wave-uniform count); a row past N inside the last set is
    // fetched from row N - 1 (no per-lane branch around a load) and left out of every sum and maximum
    const int nset = (N + RG - 1) / RG;
    h8 x[MAXR];
    constexpr int SUB = rows_in_flight<ROPE>(MAXR);       // without RoPE the whole slab is requested at once
#pragma unroll
    for (int i0 = 0; i0 < MAXR; i0 += SUB) {
        RowRaw<ROPE> fetched[SUB];
#pragma unroll
        for (int i = 0; i < SUB; ++i) {
            if (i0 + i < nset) {
                const int r = rg + (i0 + i) * RG, rc = r < N ? r : N - 1;
                fetched[i] = fetch_row8<D, ROPE>(base + (size_t)rc * D, c8, cs + (size_t)rc * HALF, sn + (size_t)rc * HALF);
            }
        }
        __builtin_amdgcn_sched_barrier(0);       // requested before anything is used
#pragma unroll
        for (int i = 0; i < SUB; ++i)
            if (i0 + i < nset) x[i0 + i] = finish_row8<D, ROPE>(fetched[i], c8);
    }
    // ---- exact column sums in fp64: multiples of 2^-24 below 2^16 in magnitude, at most 32 per thread --
    // every partial sum fits 53 bits; then an exact conversion to a count of 2^-24 units
    double acc_d[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc_d[e] = 0.0;
#pragma unroll
    for (int i = 0; i < MAXR; ++i) {
        if (i < nset) {
            const double live = rg + i * RG < N ? 1.0 : 0.0;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc_d[e] += live * (double)(float)x[i][e];
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const double v = acc_d[e] * 16777216.0;          // |v| < 2^46
        const double hi = __builtin_trunc(v * 0x1p-26);
        const double lo = v - hi * 0x1p26;
        part[rg][c8 * 8 + e] = (long long)(int)hi * (1ll << 26) + (long long)(int)lo;
    }
    __syncthreads();
    if (t < D) {
        long long sum = 0;
#pragma unroll 4
        for (int g = 0; g < RG; ++g) sum += part[g][t];
        const double avg = (double)sum / (double)N;
        const float m = (float)(avg * 0x1p-24);
        s_mean[t] = m;
        if (k_mean != nullptr) k_mean[(size_t)bh * D + t] = m;
    }
    __syncthreads();
    float mean[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) mean[e] = s_mean[c8 * 8 + e];

    int8_t* qbase = kq + ((size_t)bh * N) * D + c8 * 8;
    auto quantize_row = [&](const h8& raw, float rcp, int r) {
        unsigned w[2] = {0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float q = __builtin_rintf(((float)raw[e] - mean[e]) * rcp);     // round half to even
            q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
            w[e >> 2] |= ((unsigned)((int)q) & 0xffu) << (8 * (e & 3));
        }
        *(uint2*)(qbase + (size_t)r * D) = make_uint2(w[0], w[1]);
    };
    auto row_amax = [&](const h8& raw) {
        float a = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) a = __builtin_fmaxf(a, __builtin_fabsf((float)raw[e] - mean[e]));
        return a;
    };

    if (block == 1) {
        // per-token scales: the VPR lanes of a row reduce among themselves
#pragma unroll
        for (int i = 0; i < MAXR; ++i) {
            if (i < nset) {
                const int r = rg + i * RG;
                float amax = row_amax(x[i]);
#pragma unroll
                for (int off = VPR / 2; off >= 1; off >>= 1) amax = __builtin_fmaxf(amax, __shfl_xor(amax, off, 64));
                if (r < N) {
                    if (c8 == 0) scale[(size_t)bh * N + r] = amax / 127.0f;
                    quantize_row(x[i], amax > 0.0f ? 127.0f / amax : 0.0f, r);
                }
            }
        }
        return;
    }

    // per-block scales.  block = lpt * RG rows: register sets lpt * g .. lpt * g + lpt - 1 of every thread are
    // block g (lpt a power of two; the same for every thread).  Every thread folds its rows of a block, the
    // wavefront reduces by shuffles and leaves its maximum in LDS; after ONE barrier every block's maximum
    // is the largest of four words.  (A row past N holds zeros: |0 - mean| may exceed the block's true
    // maximum, so such rows are left out.)
    const int nblk = (N + block - 1) / block;
    const int lpt = block / RG;
    const int wave = t >> 6;
    float cur = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXR; ++i) {
        if (i < nset) {
            const float a = row_amax(x[i]);
            cur = rg + i * RG < N ? __builtin_fmaxf(cur, a) : cur;
        }
        if (((i + 1) & (lpt - 1)) == 0 && i / lpt < nblk) {          // last register set of block i / lpt (uniform)
            float m = cur;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) m = __builtin_fmaxf(m, __shfl_xor(m, off, 64));
            if ((t & 63) == 0) s_red[i / lpt][wave] = m;
            cur = 0.0f;
        }
    }
    __syncthreads();
    if (t < nblk) {
        const float amax = __builtin_fmaxf(__builtin_fmaxf(s_red[t][0], s_red[t][1]), __builtin_fmaxf(s_red[t][2], s_red[t][3]));
        scale[(size_t)bh * nblk + t] = amax / 127.0f;
    }
#pragma unroll
    for (int i = 0; i < MAXR; ++i) {
        if (i < nset) {
            const int r = rg + i * RG, g = i / lpt;
            const float amax = __builtin_fmaxf(__builtin_fmaxf(s_red[g][0], s_red[g][1]), __builtin_fmaxf(s_red[g][2], s_red[g][3]));
            if (r < N) quantize_row(x[i], amax > 0.0f ? 127.0f / amax : 0.0f, r);
        }
    }
}

template <int D, bool ROPE>
__global__ void __launch_bounds__(256) k_small_kernel(const _Float16* __restrict__ k, int8_t* __restrict__ kq,
                                                      float* __restrict__ scale, float* __restrict__ k_mean,
                                                      int N, int block,
                                                      const float* __restrict__ cs, const float* __restrict__ sn) {
    k_small_body<D, ROPE>(k, kq, scale, k_mean, N, block, cs, sn, blockIdx.x);
}

// Workgroups per slab of the quantizer kernels: enough to fill the chip a few times over, few
// enough that a workgroup of the K side walks several blocks per read of the partial sums.
static int quant_groups(int BH, int units) {
    const int want = (2048 + BH - 1) / BH;
    return units < want ? units : want;
}

template <int D, bool IS_K, bool ROPE>
static hipError_t launch_quant(const void* x, int8_t* xq, float* scale, float* mean, const long long* parts, int P,
                               int BH, int N, int block, float sm_scale, const float* cs, const float* sn,
                               hipStream_t st) {
    const _Float16* xp = (const _Float16*)x;
    if (block == 1) {
        constexpr int ROWS = (256 / (D / 8)) * TOK_LPT;
        const int ngrp = (N + ROWS - 1) / ROWS;
        quant_token_kernel<D, IS_K, ROPE><<<dim3(IS_K ? quant_groups(BH, ngrp) : ngrp, BH), 256, 0, st>>>(
            xp, xq, scale, mean, parts, P, N, sm_scale, cs, sn);
        return hipGetLastError();
    }
    const int nblk = (N + block - 1) / block;
    dim3 grid(quant_groups(BH, nblk), BH);
#define SAGE_QUANT(LPT) quant_block_kernel<D, LPT, IS_K, ROPE><<<grid, 256, 0, st>>>(xp, xq, scale, mean, parts, P, N, block, sm_scale, cs, sn)
    switch (block * D / 2048) {
        case 1: SAGE_QUANT(1); break;
        case 2: SAGE_QUANT(2); break;
        case 4: SAGE_QUANT(4); break;
        // the largest block (128 tokens x 128 channels) runs with 512 threads of 4 rows each: twice the
        // loads in flight per block and half the work per thread behind the block-wide maximum
        case 8: quant_block_kernel<D, 4, IS_K, ROPE, 512><<<grid, 512, 0, st>>>(xp, xq, scale, mean, parts, P, N, block, sm_scale, cs, sn); break;
        default: return hipErrorInvalidValue;
    }
#undef SAGE_QUANT
    return hipGetLastError();
}

template <int D, bool ROPE>
static hipError_t quant_q_d(const void* q, int8_t* qq, float* qscale, int BH, int N, float sm_scale, int block,
                            const float* cs, const float* sn, hipStream_t st) {
    return launch_quant<D, false, ROPE>(q, qq, qscale, nullptr, nullptr, 0, BH, N, block, sm_scale, cs, sn, st);
}

// cs, sn: RoPE tables [N, D/2] (both null: no rotation)
hipError_t launch_quant_q(const void* q, int8_t* qq, float* qscale, int BH, int N, int D,
                          float sm_scale, int block, const float* cs, const float* sn, hipStream_t st) {
    const bool rope = cs != nullptr;
    if (D == 64) return rope ? quant_q_d<64, true>(q, qq, qscale, BH, N, sm_scale, block, cs, sn, st)
                             : quant_q_d<64, false>(q, qq, qscale, BH, N, sm_scale, block, cs, sn, st);
    return rope ? quant_q_d<128, true>(q, qq, qscale, BH, N, sm_scale, block, cs, sn, st)
                : quant_q_d<128, false>(q, qq, qscale, BH, N, sm_scale, block, cs, sn, st);
}

// How the tokens of a slab are cut for the first level of the column sums: about 512 workgroups in
// all (two per compute unit keep enough loads in flight), at most 64 partial sums per slab (every
// quantizer workgroup adds them up again), chunks of whole 256-row batches and at least 512 rows.
ColsumPlan plan_colsum(int BH, int N) {
    if (N <= SMALL_N) return {0, 0};                    // single-launch kernel, no partial sums
    const int want = (512 + BH - 1) / BH;
    long chunk = (N + want - 1) / want;
    chunk = 256 * ((chunk + 255) / 256);
    if (chunk < 512) chunk = 512;
    int P = (int)((N + chunk - 1) / chunk);
    if (P > 64) {
        chunk = 256 * (((N + 63) / 64 + 255) / 256);
        P = (int)((N + chunk - 1) / chunk);
    }
    return {P, (int)chunk};
}

template <int D, bool ROPE>
static hipError_t smooth_quant_k_d(const void* k, int8_t* kq, float* kscale, float* kmean, long long* parts,
                                   int BH, int N, int block, const float* cs, const float* sn, hipStream_t st) {
    const ColsumPlan cp = plan_colsum(BH, N);
    k_colsum_kernel<D, ROPE><<<dim3(cp.parts, BH), 256, 0, st>>>((const _Float16*)k, parts, N, cp.chunk, cs, sn);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_quant<D, true, ROPE>(k, kq, kscale, kmean, parts, cp.parts, BH, N, block, 1.0f, cs, sn, st);
}

hipError_t launch_smooth_quant_k(const void* k, int8_t* kq, float* kscale, float* kmean,
                                 long long* parts, int BH, int N, int D, int block,
                                 const float* cs, const float* sn, hipStream_t st) {
    const bool rope = cs != nullptr;
    if (N <= SMALL_N) {
        const _Float16* kp = (const _Float16*)k;
        if (D == 64) {
            if (rope) k_small_kernel<64, true><<<BH, 256, 0, st>>>(kp, kq, kscale, kmean, N, block, cs, sn);
            else k_small_kernel<64, false><<<BH, 256, 0, st>>>(kp, kq, kscale, kmean, N, block, cs, sn);
        } else {
            if (rope) k_small_kernel<128, true><<<BH, 256, 0, st>>>(kp, kq, kscale, kmean, N, block, cs, sn);
            else k_small_kernel<128, false><<<BH, 256, 0, st>>>(kp, kq, kscale, kmean, N, block, cs, sn);
        }
        return hipGetLastError();
    }
    if (D == 64) return rope ? smooth_quant_k_d<64, true>(k, kq, kscale, kmean, parts, BH, N, block, cs, sn, st)
                             : smooth_quant_k_d<64, false>(k, kq, kscale, kmean, parts, BH, N, block, cs, sn, st);
    return rope ? smooth_quant_k_d<128, true>(k, kq, kscale, kmean, parts, BH, N, block, cs, sn, st)
                : smooth_quant_k_d<128, false>(k, kq, kscale, kmean, parts, BH, N, block, cs, sn, st);
}

// ---- One launch for two jobs (sage_quant_qk) -----------------------------------------------------
// The quantization of Q (Section 4.6 + 3.2) depends on nothing the K side computes, and the K side
// needs a grid-wide result (the mean, Section 4.2) between its two halves.  So the first launch of the
// pair does the K side's first half AND all of Q: workgroups 0 .. n_k - 1 of a slab's row of the grid
// run the K job, the others the Q job; the second launch is the K quantizer as it is.  For short key
// sequences the K job is the whole K pre-pass of the slab (k_small_body) and there is no second launch.
// Same bodies, same arithmetic, same bits as the separate calls; one launch (a few microseconds, which
// is what short sequences are made of) less.
template <int D, int LPT, int NT, bool SMALL_K>
__global__ void __launch_bounds__(NT) qk_first_block_kernel(const _Float16* __restrict__ k, long long* __restrict__ parts,
                                                             int8_t* __restrict__ kq, float* __restrict__ kscale,
                                                             float* __restrict__ kmean, int Nkv, int chunk, int block_k, int n_k,
                                                             const _Float16* __restrict__ q, int8_t* __restrict__ qq,
                                                             float* __restrict__ qscale, int Nq, int block_q, float sm_scale) {
    const int bx = blockIdx.x, bh = blockIdx.y;
    if (bx < n_k) {
        if constexpr (SMALL_K) k_small_body<D, false>(k, kq, kscale, kmean, Nkv, block_k, nullptr, nullptr, bh);
        else k_colsum_body<D, false, NT>(k, parts, Nkv, chunk, nullptr, nullptr, bx, n_k, bh);
    } else {
        quant_block_body<D, LPT, false, false, NT>(q, qq, qscale, nullptr, nullptr, 0, Nq, block_q, sm_scale, nullptr, nullptr,
                                                   bx - n_k, (int)gridDim.x - n_k, bh);
    }
}
template <int D, bool SMALL_K>
__global__ void __launch_bounds__(256) qk_first_token_kernel(const _Float16* __restrict__ k, long long* __restrict__ parts,
                                                             int8_t* __restrict__ kq, float* __restrict__ kscale,
                                                             float* __restrict__ kmean, int Nkv, int chunk, int block_k, int n_k,
                                                             const _Float16* __restrict__ q, int8_t* __restrict__ qq,
                                                             float* __restrict__ qscale, int Nq, float sm_scale) {
    const int bx = blockIdx.x, bh = blockIdx.y;
    if (bx < n_k) {
        if constexpr (SMALL_K) k_small_body<D, false>(k, kq, kscale, kmean, Nkv, block_k, nullptr, nullptr, bh);
        else k_colsum_body<D, false, 256>(k, parts, Nkv, chunk, nullptr, nullptr, bx, n_k, bh);
    } else {
        quant_token_body<D, false, false>(q, qq, qscale, nullptr, nullptr, 0, Nq, sm_scale, nullptr, nullptr,
                                          bx - n_k, (int)gridDim.x - n_k, bh);
    }
}

template <int D, bool SMALL_K>
static hipError_t quant_qk_first(const void* q, const void* k, int8_t* qq, float* qscale, int8_t* kq, float* kscale,
                                 float* kmean, long long* parts, int BH, int Nq, int Nkv, float sm_scale,
                                 int block_q, int block_k, const ColsumPlan& cp, hipStream_t st) {
    const _Float16* qp = (const _Float16*)q;
    const _Float16* kp = (const _Float16*)k;
    const int n_k = SMALL_K ? 1 : cp.parts;
    if (block_q == 1) {
        constexpr int ROWS = (256 / (D / 8)) * TOK_LPT;
        const int ngrp = (Nq + ROWS - 1) / ROWS;
        qk_first_token_kernel<D, SMALL_K><<<dim3(n_k + ngrp, BH), 256, 0, st>>>(kp, parts, kq, kscale, kmean, Nkv, cp.chunk,
                                                                               block_k, n_k, qp, qq, qscale, Nq, sm_scale);
        return hipGetLastError();
    }
    const int nblk = (Nq + block_q - 1) / block_q;
    const dim3 grid(n_k + quant_groups(BH, nblk), BH);
#define SAGE_QK(LPT, NT) qk_first_block_kernel<D, LPT, NT, SMALL_K><<<grid, NT, 0, st>>>(kp, parts, kq, kscale, kmean, Nkv, cp.chunk, block_k, n_k, qp, qq, qscale, Nq, block_q, sm_scale)
    switch (block_q * D / 2048) {
        case 1: SAGE_QK(1, 256); break;
        case 2: SAGE_QK(2, 256); break;
        case 4: SAGE_QK(4, 256); break;
        case 8:
            // (the single-workgroup K job is written for 256 threads: 8 rows per thread on the Q side there)
            if constexpr (SMALL_K) SAGE_QK(8, 256);
            else SAGE_QK(4, 512);
            break;
        default: return hipErrorInvalidValue;
    }
#undef SAGE_QK
    return hipGetLastError();
}

template <int D>
static hipError_t quant_qk_d(const void* q, const void* k, int8_t* qq, float* qscale, int8_t* kq, float* kscale,
                             float* kmean, long long* parts, int BH, int Nq, int Nkv, float sm_scale,
                             int block_q, int block_k, hipStream_t st) {
    const ColsumPlan cp = plan_colsum(BH, Nkv);
    if (Nkv <= SMALL_N)
        return quant_qk_first<D, true>(q, k, qq, qscale, kq, kscale, kmean, parts, BH, Nq, Nkv, sm_scale, block_q, block_k, cp, st);
    hipError_t e = quant_qk_first<D, false>(q, k, qq, qscale, kq, kscale, kmean, parts, BH, Nq, Nkv, sm_scale, block_q, block_k, cp, st);
    if (e != hipSuccess) return e;
    return launch_quant<D, true, false>(k, kq, kscale, kmean, parts, cp.parts, BH, Nkv, block_k, 1.0f, nullptr, nullptr, st);
}

hipError_t launch_quant_qk(const void* q, const void* k, int8_t* qq, float* qscale, int8_t* kq, float* kscale,
                           float* kmean, long long* parts, int BH, int Nq, int Nkv, int D, float sm_scale,
                           int block_q, int block_k, hipStream_t st) {
    if (D == 64) return quant_qk_d<64>(q, k, qq, qscale, kq, kscale, kmean, parts, BH, Nq, Nkv, sm_scale, block_q, block_k, st);
    return quant_qk_d<128>(q, k, qq, qscale, kq, kscale, kmean, parts, BH, Nq, Nkv, sm_scale, block_q, block_k, st);
}

}  // namespace sage
