// Fused SageAttention forward kernel for gfx950 (Algorithm 1, inner loops).
//
// One workgroup = 4 wavefronts = 128 query rows (32 per wavefront); key/value tiles of 64 tokens
// are staged through LDS.  Scores are computed TRANSPOSED, S^T = K^ Q^^T, with the 32x32x32 INT8
// matrix instruction: each lane then owns one query column and 16 keys per 32-key sub-tile, so
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
#include "sage_internal.h"

namespace sage {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

constexpr int QTILE = 128;   // query rows per workgroup
constexpr int KTILE = 64;    // keys per LDS tile
constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float swap32(float v) {
    // value held by the lane 32 away
    auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(int, v), __builtin_bit_cast(int, v), false, false);
    return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}

template <int D, bool CAUSAL, bool DUMP>
__global__ void __launch_bounds__(256, 2)
sage_attn_kernel(const int8_t* __restrict__ qi, const float* __restrict__ qsc,
                 const int8_t* __restrict__ ki, const float* __restrict__ ksc,
                 const _Float16* __restrict__ vg, _Float16* __restrict__ og,
                 int32_t* __restrict__ sdump,
                 int N, int block_q, int block_k, int tiles_q, int per_xcd, long total_tiles) {
    constexpr int KP = D + 16;          // K^ row pitch in LDS (bytes): 16-byte skew per row
    constexpr int VP = 2 * D + 64;      // V row pitch in LDS (bytes): 4 rows tile the 64 banks
    constexpr int KS = D / 32;          // INT8 MFMA steps along the head dimension
    constexpr int DT = D / 32;          // 32-wide output tiles along the head dimension
    constexpr int KL = KTILE * D / 16 / 256;      // 16-byte K^ vectors per thread per tile
    constexpr int VL = KTILE * D / 8 / 256;       // 16-byte V vectors per thread per tile
    __shared__ __attribute__((aligned(16))) unsigned char lds_k[KTILE * KP];
    __shared__ __attribute__((aligned(16))) unsigned char lds_v[KTILE * VP];

    // Workgroup -> (slab, query tile).  Consecutive workgroup ids land on the 8 XCDs in turn; give
    // each XCD a contiguous range of the (slab-major, heaviest-query-tile-first) order so that the
    // workgroups resident on one XCD share K^/V in its L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const long gidx = (long)xcd * per_xcd + slot;
    if (slot >= per_xcd || gidx >= total_tiles) return;
    const int bh = (int)(gidx / tiles_q);
    const int qt = tiles_q - 1 - (int)(gidx % tiles_q);

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int ql = lane & 31, g = lane >> 5;
    const int qrow0 = qt * QTILE + wave * 32;
    const int q_row = qrow0 + ql;
    const size_t slab = (size_t)bh * N;
    const int nbq = (N + block_q - 1) / block_q, nbk = (N + block_k - 1) / block_k;

    // Q^ operands (B matrix of S^T = K^ Q^^T) stay in registers for the whole kernel.
    v4i qreg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        qreg[ks] = (v4i){0, 0, 0, 0};
        if (q_row < N) qreg[ks] = *(const v4i*)(qi + (slab + q_row) * D + ks * 32 + g * 16);
    }
    const int qrow_c = qrow0 < N ? qrow0 : N - 1;
    const float dq = qsc[(size_t)bh * nbq + qrow_c / block_q];

    const int kv_tiles_all = (N + KTILE - 1) / KTILE;
    int kv_tiles = kv_tiles_all;
    if (CAUSAL) {
        int last = (qt * QTILE + QTILE - 1) / KTILE + 1;
        kv_tiles = last < kv_tiles_all ? last : kv_tiles_all;
    }

    // global -> register staging of one K^/V tile
    v4i kpre[KL], vpre[VL];
    auto fetch = [&](int j) {
        const int kv0 = j * KTILE;
#pragma unroll
        for (int i = 0; i < KL; ++i) {
            int vidx = t + 256 * i, row = vidx / (D / 16), c = vidx % (D / 16);
            kpre[i] = (v4i){0, 0, 0, 0};
            if (kv0 + row < N) kpre[i] = *(const v4i*)(ki + (slab + kv0 + row) * D + c * 16);
        }
        if (DUMP) return;                 // the score dump never touches V
#pragma unroll
        for (int i = 0; i < VL; ++i) {
            int vidx = t + 256 * i, row = vidx / (D / 8), c = vidx % (D / 8);
            vpre[i] = (v4i){0, 0, 0, 0};
            if (kv0 + row < N) vpre[i] = *(const v4i*)(vg + (slab + kv0 + row) * D + c * 8);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < KL; ++i) {
            int vidx = t + 256 * i, row = vidx / (D / 16), c = vidx % (D / 16);
            *(v4i*)(lds_k + row * KP + c * 16) = kpre[i];
        }
        if (DUMP) return;
#pragma unroll
        for (int i = 0; i < VL; ++i) {
            int vidx = t + 256 * i, row = vidx / (D / 8), c = vidx % (D / 8);
            *(v4i*)(lds_v + row * VP + c * 16) = vpre[i];
        }
    };

    // per-lane base of the transposing V reads: source lane i of a 16-lane group addresses
    // key (i/4) and the 4-channel chunk (i%4) of the group's 16 channels
    const int grp = lane >> 4, li = lane & 15;
    const unsigned char* v_lane = lds_v + (4 * (grp >> 1) + (li >> 2)) * VP + (16 * (grp & 1) + 4 * (li & 3)) * 2;
    const unsigned char* k_lane = lds_k + ql * KP + g * 16;

    v16f acc_o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[dt][r] = 0.0f;
    float m_run = -__builtin_inff(), l_run = 0.0f;

    fetch(0);
    for (int j = 0; j < kv_tiles; ++j) {
        const int kv0 = j * KTILE;
        __syncthreads();                 // everyone is done reading the previous tile
        stage();
        __syncthreads();
        if (j + 1 < kv_tiles) fetch(j + 1);     // in flight while this tile is computed

        if (CAUSAL && !DUMP && kv0 > qrow0 + 31) continue;     // tile is above this wave's rows

        // ---- S^T = K^ Q^^T (INT8, int32 accumulate): two 32-key sub-tiles
        v16i acc_s[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_s[s][r] = 0;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                v4i a = *(const v4i*)(k_lane + s * 32 * KP + ks * 32);
                acc_s[s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qreg[ks], acc_s[s], 0, 0, 0);
            }
        }

        if (DUMP) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (q_row < N && key < N) sdump[(slab + q_row) * (size_t)N + key] = acc_s[s][r];
                }
            continue;
        }

        // ---- dequantize + online softmax (base-2 domain: scores are multiplied by log2 e)
        const float sc = dq * ksc[(size_t)bh * nbk + kv0 / block_k] * LOG2E;
        const bool need_mask = (kv0 + KTILE > N) || (CAUSAL && kv0 + KTILE - 1 > qrow0);
        float f[2][16];
        float mx = -__builtin_inff();
        unsigned masked[2] = {0u, 0u};
        if (need_mask) {
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                    bool hide = (key >= N) || (CAUSAL && key > q_row);
                    if (hide) masked[s] |= 1u << r;
                }
        }
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                f[s][r] = (float)acc_s[s][r];
                float cand = ((masked[s] >> r) & 1u) ? -__builtin_inff() : f[s][r];
                mx = __builtin_fmaxf(mx, cand);
            }
        mx = __builtin_fmaxf(mx, swap32(mx));
        const float m_cand = (mx == -__builtin_inff()) ? mx : mx * sc;
        const float m_new = __builtin_fmaxf(m_run, m_cand);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;

        float rowsum = 0.0f;
        v8h pk[2][2];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float x = __builtin_fmaf(f[s][r], sc, -m_new);
                if ((masked[s] >> r) & 1u) x = -__builtin_inff();
                float p = __builtin_amdgcn_exp2f(x);
                rowsum += p;
                pk[s][r >> 3][r & 7] = (_Float16)p;
            }
        l_run = l_run * alpha + rowsum;

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
                    const unsigned char* p0 = v_lane + (32 * s + 16 * u) * VP + dt * 64;
                    v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, p0));
                    v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, p0 + 8 * VP));
                    v8h a = __builtin_bit_cast(v8h, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                    acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, pk[s][u], acc_o[dt], 0, 0, 0);
                }
    }
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
    const _Float16* vp = (const _Float16*)v;
    _Float16* op = (_Float16*)o;
    if (sdump)
        sage_attn_kernel<D, false, true><<<grid, 256, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, block_q, block_k, tiles_q, per_xcd, total);
    else if (causal)
        sage_attn_kernel<D, true, false><<<grid, 256, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, block_q, block_k, tiles_q, per_xcd, total);
    else
        sage_attn_kernel<D, false, false><<<grid, 256, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, block_q, block_k, tiles_q, per_xcd, total);
    return hipGetLastError();
}

hipError_t launch_attn(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                       const void* v, void* o, int32_t* sdump, int BH, int N, int D, int causal,
                       int block_q, int block_k, hipStream_t st) {
    if (D == 64) return launch_d<64>(qq, qscale, kq, kscale, v, o, sdump, BH, N, causal, block_q, block_k, st);
    return launch_d<128>(qq, qscale, kq, kscale, v, o, sdump, BH, N, causal, block_q, block_k, st);
}

}  // namespace sage
