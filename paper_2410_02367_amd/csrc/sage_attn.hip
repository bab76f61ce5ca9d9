// Fused SageAttention forward kernel for gfx950 (Algorithm 1, inner loops).
//
// One workgroup = 4 wavefronts = 128 query rows (32 per wavefront); key/value tiles of 64 tokens
// are double-buffered in LDS.  Scores are computed TRANSPOSED, S^T = K^ Q^^T, with the 32x32x32
// INT8 matrix instruction: each lane then owns one query column and 16 keys per 32-key sub-tile, so
//   - row max / row sum need one cross-lane step (lane <-> lane+32),
//   - the exponentiated scores are already in the register layout the FP16 32x32x16 instruction
//     wants for its B operand (P~^T), and O^T = V^T P~^T accumulates with the rescale factor
//     being a per-lane scalar.
// V^T operands come from the row-major V tile in LDS through the transposing LDS read.
//
// Register layout facts used below (established on hardware by a probe):
//   32x32 result:  lane l, register r  ->  row 8*(r/4) + 4*(l/32) + r%4, column l%32
//   INT8 operand:  lane l holds row/column l%32, contraction indices 16*(l/32) .. +15
//   FP16 operand:  lane l holds row/column l%32, contraction indices 8*(l/32) .. +7
//   ds_read_tr16_b64: inside each group of 16 lanes, destination lane i, slot j receives element
//                  i%4 of the 8-byte chunk addressed by source lane 4*j + i/4.
//
// Softmax arithmetic (VALU is as scarce as MFMA here, so every per-element operation counts):
//   - the int32 accumulators start at 0x4B400000; reinterpreted as fp32 the result is exactly
//     12582912 + S^ (|S^| <= 127*127*128 < 2^22), so no int->float conversion is issued and the
//     dequantization, the log2(e) factor and the subtraction of the running maximum are one FMA;
//   - the row maximum is taken on the raw accumulators with integer max;
//   - P~ is packed to FP16 by truncation and the row sum l is accumulated from those packed
//     values (dot-product instruction against (1,1)), so numerator and denominator see the same
//     P~ and the truncation bias cancels in O = (P~ V) / l.
#include "sage_internal.h"
#include <type_traits>

namespace sage {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef __fp16 v2hh __attribute__((ext_vector_type(2)));
typedef short v4s __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int QTILE = 128;   // query rows per workgroup
constexpr int KTILE = 64;    // keys per LDS tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr int MAGIC_I = 0x4B400000;        // bit pattern of 12582912.0f = 1.5 * 2^23
constexpr float MAGIC_F = 12582912.0f;

// LDS tiles are unpadded; 16-byte chunks are XOR-swizzled inside each row so that the operand
// reads of 16 consecutive rows touch every bank once.
#ifdef SAGE_DBG_NOSWZ
template <int D> __device__ __forceinline__ int k_swz(int row) { return 0; }
template <int D> __device__ __forceinline__ int v_swz(int row) { return 0; }
#else
template <int D> __device__ __forceinline__ int k_swz(int row) { return D == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
template <int D> __device__ __forceinline__ int v_swz(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }
#endif

__device__ __forceinline__ int swap32i(int v) {
    // value held by the lane 32 away
    auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (threadIdx.x & 32) ? r[0] : r[1];
}
__device__ __forceinline__ float swap32(float v) {
    return __builtin_bit_cast(float, swap32i(__builtin_bit_cast(int, v)));
}
// by-value reinterpretation (never bit_cast a vector element in place)
__device__ __forceinline__ float as_f32(int v) { return __builtin_bit_cast(float, v); }
__device__ __forceinline__ int imax3(int a, int b, int c) { return max(max(a, b), c); }

#ifdef SAGE_DBG_TIMING
__device__ unsigned long long g_timing[16384 * 8];
#define TSTAMP(k) do { unsigned long long now_ = __builtin_amdgcn_s_memtime(); tacc[k] += now_ - tlast; tlast = now_; } while (0)
#else
#define TSTAMP(k) do {} while (0)
#endif

template <int D, bool CAUSAL, bool DUMP>
__global__ void __launch_bounds__(256, 2)
sage_attn_kernel(const int8_t* __restrict__ qi, const float* __restrict__ qsc,
                 const int8_t* __restrict__ ki, const float* __restrict__ ksc,
                 const _Float16* __restrict__ vg, _Float16* __restrict__ og,
                 int32_t* __restrict__ sdump,
                 int N, int shift_q, int shift_k, int tiles_q, int per_xcd, long total_tiles) {
    constexpr int KROW = D;             // bytes per K^ row in LDS
    constexpr int VROW = 2 * D;         // bytes per V row in LDS
    constexpr int KB = KTILE * KROW;    // bytes per K^ tile
    constexpr int VB = KTILE * VROW;    // bytes per V tile
    constexpr int KS = D / 32;          // INT8 MFMA steps along the head dimension
    constexpr int DT = D / 32;          // 32-wide output tiles along the head dimension
    constexpr int KL = KB / 16 / 256;   // 16-byte K^ vectors per thread per tile
    constexpr int VL = VB / 16 / 256;   // 16-byte V vectors per thread per tile
    constexpr int KCH = KROW / 16, VCH = VROW / 16;   // chunks per row
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * KB + 2 * VB];

    // Workgroup -> (slab, query tile).  Consecutive workgroup ids land on the 8 XCDs in turn; give
    // each XCD a contiguous range of the (slab-major, heaviest-query-tile-first) order so that the
    // workgroups resident on one XCD share K^/V in its L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const long gidx = (long)xcd * per_xcd + slot;
    if (slot >= per_xcd || gidx >= total_tiles) return;
    const int bh = (int)(gidx / tiles_q);
    const int qt = tiles_q - 1 - (int)(gidx % tiles_q);

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);     // wave-uniform: keeps tile control flow scalar
    const int ql = lane & 31, g = lane >> 5;
    const int qrow0 = qt * QTILE + wave * 32;
    const int q_row = qrow0 + ql;
    const size_t slab = (size_t)bh * N;
    const int nbq = (N + (1 << shift_q) - 1) >> shift_q, nbk = (N + (1 << shift_k) - 1) >> shift_k;

    // Q^ operands (B matrix of S^T = K^ Q^^T) stay in registers for the whole kernel.
    v4i qreg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        qreg[ks] = (v4i){0, 0, 0, 0};
        if (q_row < N) qreg[ks] = *(const v4i*)(qi + (slab + q_row) * D + ks * 32 + g * 16);
    }
    float dq = 0.0f;
    if (!DUMP) {
        const int qrow_c = qrow0 < N ? qrow0 : N - 1;
        dq = qsc[(size_t)bh * nbq + (qrow_c >> shift_q)] * LOG2E;
    }

    const float* __restrict__ ksc_bh = ksc + (size_t)bh * nbk;
    const int kv_tiles_all = (N + KTILE - 1) / KTILE;
    int kv_tiles = kv_tiles_all;
    if (CAUSAL) {
        int last = (qt * QTILE + QTILE - 1) / KTILE + 1;
        kv_tiles = last < kv_tiles_all ? last : kv_tiles_all;
    }

    // ---- global -> register -> LDS staging.  Thread t moves the 16-byte vectors t, t+256, ...
    // of the (linear, unpadded) LDS tile; the global chunk it fetches is the swizzled one.  Rows
    // past N are clamped to the last row: their scores are masked, so the values never matter.
    v4i kpre[KL], vpre[VL];
    int k_goff[KL], v_goff[VL];          // byte offsets inside a full tile (row * pitch + swizzled chunk)
#pragma unroll
    for (int i = 0; i < KL; ++i) {
        int vidx = t + 256 * i, row = vidx / KCH, c = (vidx % KCH) ^ k_swz<D>(row);
        k_goff[i] = row * D + c * 16;
    }
#pragma unroll
    for (int i = 0; i < VL; ++i) {
        int vidx = t + 256 * i, row = vidx / VCH, c = (vidx % VCH) ^ v_swz<D>(row);
        v_goff[i] = row * 2 * D + c * 16;
    }
    const unsigned char* k_slab = (const unsigned char*)(ki + slab * D);
    const unsigned char* v_slab = (const unsigned char*)(vg + slab * D);
    auto fetch = [&](int j) {
        const int kv0 = j * KTILE;
        const unsigned char* kt = k_slab + (size_t)kv0 * D;
        const unsigned char* vt = v_slab + (size_t)kv0 * 2 * D;
        if (kv0 + KTILE <= N) {
#pragma unroll
            for (int i = 0; i < KL; ++i) kpre[i] = *(const v4i*)(kt + k_goff[i]);
            if (DUMP) return;                 // the score dump never touches V
#pragma unroll
            for (int i = 0; i < VL; ++i) vpre[i] = *(const v4i*)(vt + v_goff[i]);
        } else {
            const int lim = N - 1 - kv0;      // last valid row of the tail tile
#pragma unroll
            for (int i = 0; i < KL; ++i) {
                int row = k_goff[i] / D, rc = row < lim ? row : lim;
                kpre[i] = *(const v4i*)(kt + k_goff[i] + (rc - row) * D);
            }
            if (DUMP) return;
#pragma unroll
            for (int i = 0; i < VL; ++i) {
                int row = v_goff[i] / (2 * D), rc = row < lim ? row : lim;
                vpre[i] = *(const v4i*)(vt + v_goff[i] + (rc - row) * 2 * D);
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < KL; ++i) *(v4i*)(lds + buf * KB + (t + 256 * i) * 16) = kpre[i];
        if (DUMP) return;
#pragma unroll
        for (int i = 0; i < VL; ++i) *(v4i*)(lds + 2 * KB + buf * VB + (t + 256 * i) * 16) = vpre[i];
    };

    // ---- per-lane LDS read offsets
    // K^ operand: row ql (+32 per sub-tile), chunk 2*ks+g, swizzled
    int k_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_off[ks] = ql * KROW + (((2 * ks + g) ^ k_swz<D>(ql)) << 4);
    // V^T operand through the transposing read: source lane li of a 16-lane group addresses key
    // (li/4) and the 4-channel chunk (li%4) of the group's 16 channels
    const int grp = lane >> 4, li = lane & 15;
    const int v_row = 4 * (grp >> 1) + (li >> 2);
    int v_off[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
        int chunk = (4 * dt + 2 * (grp & 1) + ((li & 3) >> 1)) ^ v_swz<D>(v_row);
        v_off[dt] = v_row * VROW + chunk * 16 + (li & 1) * 8;
    }

    v16f acc_o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] = 0.0f;
    float m_run = -__builtin_inff(), l_run = 0.0f;

    v16i magic;
#pragma unroll
    for (int r = 0; r < 16; ++r) magic[r] = MAGIC_I;
    asm volatile("" : "+v"(magic));      // keep it resident: re-materializing costs 16 moves per sub-tile

    fetch(0);
    stage(0);
    if (kv_tiles > 1) fetch(1);
#ifdef SAGE_DBG_TIMING
    unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    unsigned long long tlast = __builtin_amdgcn_s_memtime();
    const unsigned long long tstart = tlast;
#endif
    for (int j = 0; j < kv_tiles; ++j) {
        TSTAMP(0);
        const int kv0 = j * KTILE;
        const int buf = j & 1;
        __syncthreads();      // tile j is visible; everyone has finished with the other buffer
        TSTAMP(1);
        if (j + 1 < kv_tiles) stage(buf ^ 1);
        if (j + 2 < kv_tiles) fetch(j + 2);     // in flight while this tile is computed
        TSTAMP(2);

        if (CAUSAL && !DUMP && kv0 > qrow0 + 31) continue;     // tile is above this wave's rows

        const unsigned char* kb = lds + buf * KB;
        const unsigned char* vb = lds + 2 * KB + buf * VB;

        // ---- S^T = K^ Q^^T (INT8, int32 accumulate): two 32-key sub-tiles
        v16i acc_s[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                v4i a = *(const v4i*)(kb + s * 32 * KROW + k_off[ks]);
                acc_s[s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qreg[ks], ks == 0 ? magic : acc_s[s], 0, 0, 0);
            }
        }

        TSTAMP(3);
        if (DUMP) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (q_row < N && key < N) sdump[(slab + q_row) * (size_t)N + key] = acc_s[s][r] - MAGIC_I;
                }
            continue;
        }

        // ---- dequantize + online softmax in the base-2 domain
        const float sc = dq * ksc_bh[kv0 >> shift_k];
        const bool need_mask = (kv0 + KTILE > N) || (CAUSAL && kv0 + KTILE - 1 > qrow0);
        v4i pk[2][2];
        float alpha;
        // MASK = true only on diagonal and tail tiles: hidden keys (beyond N, or after the query
        // when causal) are excluded from the maximum and get P~ = 0.
        auto softmax = [&](auto mask_tag) {
            constexpr bool MASK = decltype(mask_tag)::value;
            unsigned hidden[2] = {0u, 0u};
            int mi;
            if (MASK) {
                mi = 0;     // below every live accumulator (those are > 0x4B000000)
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                        bool hide = (key >= N) || (CAUSAL && key > q_row);
                        if (hide) hidden[s] |= 1u << r;
                        mi = max(mi, hide ? 0 : acc_s[s][r]);
                    }
            } else {
                mi = acc_s[0][0];
#pragma unroll
                for (int r = 1; r < 16; r += 2) mi = imax3(mi, acc_s[0][r], acc_s[0][(r + 1) & 15]);
#pragma unroll
                for (int r = 0; r < 16; r += 2) mi = imax3(mi, acc_s[1][r], acc_s[1][r + 1]);
            }
            mi = max(mi, swap32i(mi));
            const float m_cand = (MASK && mi == 0) ? -__builtin_inff() : (as_f32(mi) - MAGIC_F) * sc;
            const float m_new = __builtin_fmaxf(m_run, m_cand);
            alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            const float bias = -__builtin_fmaf(MAGIC_F, sc, m_new);      // exp2 argument = acc*sc + bias

            float rowsum = 0.0f;
            const v2hh ones = {(__fp16)1.0f, (__fp16)1.0f};
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float x0 = __builtin_fmaf(as_f32(acc_s[s][r]), sc, bias);
                    float x1 = __builtin_fmaf(as_f32(acc_s[s][r + 1]), sc, bias);
                    if (MASK) {
                        x0 = ((hidden[s] >> r) & 1u) ? -__builtin_inff() : x0;
                        x1 = ((hidden[s] >> (r + 1)) & 1u) ? -__builtin_inff() : x1;
                    }
                    v2hh h = __builtin_amdgcn_cvt_pkrtz(__builtin_amdgcn_exp2f(x0), __builtin_amdgcn_exp2f(x1));
                    rowsum = __builtin_amdgcn_fdot2(h, ones, rowsum, false);
                    pk[s][r >> 3][(r >> 1) & 3] = __builtin_bit_cast(int, h);
                }
            l_run = __builtin_fmaf(l_run, alpha, rowsum);
        };
        if (need_mask) softmax(std::true_type{}); else softmax(std::false_type{});
        TSTAMP(4);

        // ---- O^T = diag-rescale + V^T P~^T (FP16 inputs, fp32 accumulate)
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0ull) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[dt][r] *= alpha;
        }
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const unsigned char* p0 = vb + (32 * s + 16 * u) * VROW + v_off[dt];
                    v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, p0));
                    v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, p0 + 8 * VROW));
                    v8h a = __builtin_bit_cast(v8h, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                    acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, __builtin_bit_cast(v8h, pk[s][u]), acc_o[dt], 0, 0, 0);
                }
        TSTAMP(0);
    }
#ifdef SAGE_DBG_TIMING
    if (lane == 0 && gidx < 16384 / 4) {
        unsigned long long* d = g_timing + (gidx * 4 + wave) * 8;
        for (int k = 0; k < 5; ++k) d[k] = tacc[k];
        d[5] = __builtin_amdgcn_s_memtime() - tstart; d[6] = kv_tiles; d[7] = tstart;
    }
#endif
    if (DUMP) return;

    // ---- O = diag(l)^-1 O, fp16 store
    const float l_tot = l_run + swap32(l_run);
    const float inv = 1.0f / l_tot;
    if (q_row < N) {
        _Float16* orow = og + (slab + q_row) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                v4h w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (_Float16)(acc_o[dt][4 * rq + e] * inv);
                *(v4h*)(orow + dt * 32 + 8 * rq + 4 * g) = w;
            }
    }
}

template <int D>
static hipError_t launch_d(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                           const void* v, void* o, int32_t* sdump, int BH, int N, int causal,
                           int block_q, int block_k, hipStream_t st) {
    const int tiles_q = (N + QTILE - 1) / QTILE;
    const long total = (long)BH * tiles_q;
    const int per_xcd = (int)((total + 7) / 8);
    dim3 grid((unsigned)(per_xcd * 8));
    const int shift_q = __builtin_ctz((unsigned)block_q), shift_k = __builtin_ctz((unsigned)block_k);
    const _Float16* vp = (const _Float16*)v;
    _Float16* op = (_Float16*)o;
    if (sdump)
        sage_attn_kernel<D, false, true><<<grid, 256, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, shift_q, shift_k, tiles_q, per_xcd, total);
    else if (causal)
        sage_attn_kernel<D, true, false><<<grid, 256, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, shift_q, shift_k, tiles_q, per_xcd, total);
    else
        sage_attn_kernel<D, false, false><<<grid, 256, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, shift_q, shift_k, tiles_q, per_xcd, total);
    return hipGetLastError();
}

hipError_t launch_attn(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                       const void* v, void* o, int32_t* sdump, int BH, int N, int D, int causal,
                       int block_q, int block_k, hipStream_t st) {
    if (D == 64) return launch_d<64>(qq, qscale, kq, kscale, v, o, sdump, BH, N, causal, block_q, block_k, st);
    return launch_d<128>(qq, qscale, kq, kscale, v, o, sdump, BH, N, causal, block_q, block_k, st);
}

#ifdef SAGE_DBG_TIMING
extern "C" int sage_dbg_read_timing(void* host, size_t bytes) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_timing), bytes);
}
#endif

}  // namespace sage
