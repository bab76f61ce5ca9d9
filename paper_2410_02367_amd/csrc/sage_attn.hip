// Fused SageAttention forward kernel for gfx950 (Algorithm 1, inner loops).
//
// Work decomposition
//   One workgroup = 4 wavefronts (one per SIMD, so each may use the full 512-register budget)
//   = 256 query rows, 64 per wavefront as two 32-row sub-tiles.  Key/value tiles of 64 tokens are
//   double-buffered in LDS and shared by the 4 wavefronts; every K^ / V^T operand read from LDS
//   feeds two matrix instructions (one per query sub-tile).
//   Scores are computed TRANSPOSED, S^T = K^ Q^^T, with the 32x32x32 INT8 matrix instruction: each
//   lane then owns one query column and 16 keys per 32-key sub-tile, so
//     - row max / row sum need one cross-lane step (lane <-> lane+32),
//     - the exponentiated scores are already in the register layout the FP16 32x32x16 instruction
//       wants for its B operand (P~^T), and O^T = V^T P~^T accumulates with the rescale factor
//       being a per-lane scalar.
//   V^T operands come from the row-major V tile in LDS through the transposing LDS read.
//
// Schedule (software pipeline inside every wavefront)
//   On this chip the softmax arithmetic (VALU + transcendental) of a tile costs about as many
//   issue cycles as its matrix instructions.  A wavefront that alternates a matrix phase and a
//   softmax phase leaves one pipe idle at any time (and two such wavefronts on a SIMD fall into
//   lock-step instead of complementing each other).  So every wavefront runs three tiles at once:
//   while the softmax of tile j is computed (VALU), the matrix pipe is fed with P~V of tile j-1
//   and K^Q^^T of tile j+1.  A step is a flat sequence of LDS operands, each feeding one matrix
//   instruction per query sub-tile; after every matrix instruction comes one "chunk" of softmax
//   VALU work (2 scores: 2 FMA, 2 exp2, 1 pack, 1 row-sum), fenced so the order survives:
//        slot A  PV_{j-1}[ 0:16]                      slot D  PV_{j-1}[48:64] | softmax_j[32:48]
//        slot B  PV_{j-1}[16:32] | softmax_j[ 0:16]   slot E  QK_{j+1}[ 0:32] | softmax_j[48:64]
//        slot C  PV_{j-1}[32:48] | softmax_j[16:32]   slot F  QK_{j+1}[32:64]
//   S and P~ live in single register buffers: a 16-key group of P~_{j-1} is consumed by its
//   matrix instructions one slot before the softmax overwrites it, and each half of S_{j+1} is
//   produced after the softmax has consumed that half of S_j.
//   The running maximum is only raised when a row's tile maximum exceeds it by more than 2^8
//   (P~ <= 256 fits FP16 comfortably); the O rescale is then a rare, wave-uniform branch.
//
// Register layout facts used below (established on hardware by a probe):
//   32x32 result:  lane l, register r  ->  row 8*(r/4) + 4*(l/32) + r%4, column l%32
//   INT8 operand:  lane l holds row/column l%32, contraction indices 16*(l/32) .. +15
//   FP16 operand:  lane l holds row/column l%32, contraction indices 8*(l/32) .. +7
//   ds_read_tr16_b64: inside each group of 16 lanes, destination lane i, slot j receives element
//                  i%4 of the 8-byte chunk addressed by source lane 4*j + i/4.
//
// Softmax arithmetic (every per-element VALU operation counts):
//   - the int32 accumulators start at 0x4B400000; reinterpreted as fp32 the result is exactly
//     12582912 + S^ (|S^| <= 127*127*128 < 2^22), so no int->float conversion is issued and the
//     dequantization, the log2(e) factor and the subtraction of the running maximum are one FMA;
//   - the row maximum is taken on the raw accumulators with integer max;
//   - P~ is packed to FP16 with the packed round-to-nearest-even convert; the row sum l is one more
//     matrix instruction per 16 keys (a ones operand against P~^T), so l is exactly the sum of the
//     FP16 P~ that multiplies V, and costs no VALU issue slots.  (Dot-product instructions such as
//     v_dot2c run on the matrix pipe as well, but block it for VALU work -- measured.)
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

#ifndef SAGE_NWAVES
#define SAGE_NWAVES 4
#endif
#ifndef SAGE_QS
#define SAGE_QS 2
#endif
#ifndef SAGE_PHASED
#define SAGE_PHASED 0
#endif
#ifndef SAGE_PRIO
#define SAGE_PRIO 0
#endif
// The magic accumulator seed must stay resident.  With one wavefront per SIMD (512 registers) it is
// pinned in the accumulator half of the file; with two per SIMD the kernel must not touch AGPRs at
// all, or the compiler splits the 256-register budget 128/128.
#if SAGE_NWAVES * SAGE_QS * 32 / 64 <= 4 && SAGE_QS >= 2
#define SAGE_PIN_MAGIC(m) asm volatile("" : "+a"(m))
#else
#define SAGE_PIN_MAGIC(m) asm volatile("" : "+v"(m))
#endif
#ifndef SAGE_LAUNCH_BOUNDS
#define SAGE_LAUNCH_BOUNDS __launch_bounds__(SAGE_NWAVES * 64, 1)
#endif
constexpr int NWAVES = SAGE_NWAVES;    // wavefronts per workgroup
constexpr int QS = SAGE_QS;            // 32-row query sub-tiles per wavefront
constexpr int NTHREADS = NWAVES * 64;
constexpr int WROWS = 32 * QS;         // query rows per wavefront
constexpr int QTILE = NWAVES * WROWS;  // query rows per workgroup
constexpr int KTILE = 64;            // keys per LDS tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr int MAGIC_I = 0x4B400000;        // bit pattern of 12582912.0f = 1.5 * 2^23
constexpr float MAGIC_F = 12582912.0f;
constexpr float MAX_SLACK = 8.0f;          // log2 of the largest P~ tolerated before the maximum is raised

// LDS tiles are unpadded; 16-byte chunks are XOR-swizzled inside each row so that the operand
// reads of 16 consecutive rows touch every bank once.
template <int D> __device__ __forceinline__ int k_swz(int row) { return D == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
template <int D> __device__ __forceinline__ int v_swz(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }

__device__ __forceinline__ int swap32i(int v) {
    // value held by the lane 32 away
    auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (threadIdx.x & 32) ? r[0] : r[1];
}
// by-value reinterpretation (never bit_cast a vector element in place)
__device__ __forceinline__ float as_f32(int v) { return __builtin_bit_cast(float, v); }
__device__ __forceinline__ int as_i32(float v) { return __builtin_bit_cast(int, v); }
__device__ __forceinline__ int imax3(int a, int b, int c) { return max(max(a, b), c); }

#ifdef SAGE_DBG_TIMING
__device__ unsigned long long g_timing[16384 * 8];
#define TSTAMP(k) do { unsigned long long now_ = __builtin_amdgcn_s_memtime(); tacc[k] += now_ - tlast; tlast = now_; } while (0)
#else
#define TSTAMP(k) do {} while (0)
#endif

template <int D, bool CAUSAL, bool DUMP>
__global__ void SAGE_LAUNCH_BOUNDS
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
    constexpr int KVEC = KB / 16, VVEC = VB / 16;               // 16-byte vectors per tile
    constexpr int KL = (KVEC + NTHREADS - 1) / NTHREADS, VL = (VVEC + NTHREADS - 1) / NTHREADS;    // per thread
    // when a tile has fewer vectors than the workgroup has threads, only the first threads move data
    constexpr bool K_PART = KVEC % NTHREADS != 0, V_PART = VVEC % NTHREADS != 0;
    static_assert(!K_PART || KL == 1, "partial staging only for single-vector tiles");
    static_assert(!V_PART || VL == 1, "partial staging only for single-vector tiles");
    const bool k_mine = !K_PART || threadIdx.x < KVEC, v_mine = !V_PART || threadIdx.x < VVEC;
    constexpr int KCH = KROW / 16, VCH = VROW / 16;             // chunks per row
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
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);     // wave-uniform: keeps control flow scalar
    const int ql = lane & 31, g = lane >> 5;
#if SAGE_PRIO
    if (wave >= NWAVES / 2) __builtin_amdgcn_s_setprio(0); else __builtin_amdgcn_s_setprio(3);
#endif
    const int qrow0 = qt * QTILE + wave * WROWS;     // first row of the wavefront; sub-tile qs starts 32*qs later
    const size_t slab = (size_t)bh * N;
    const int nbq = (N + (1 << shift_q) - 1) >> shift_q, nbk = (N + (1 << shift_k) - 1) >> shift_k;

    // Q^ operands (B matrix of S^T = K^ Q^^T) stay in registers for the whole kernel.
    v4i qreg[QS][KS];
    float dq[QS];
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
        const int q_row = qrow0 + 32 * qs + ql;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qreg[qs][ks] = (v4i){0, 0, 0, 0};
            if (q_row < N) qreg[qs][ks] = *(const v4i*)(qi + (slab + q_row) * D + ks * 32 + g * 16);
        }
        dq[qs] = 0.0f;
        if (!DUMP) {
            const int r0 = qrow0 + 32 * qs, rc = r0 < N ? r0 : N - 1;
            dq[qs] = qsc[(size_t)bh * nbq + (rc >> shift_q)] * LOG2E;
        }
    }
    const float* __restrict__ ksc_bh = ksc + (size_t)bh * nbk;

    // kv tiles visited by the workgroup (T) and by this wavefront (Tw <= T: tiles above the
    // wavefront's last row are skipped when causal)
    const int kv_tiles_all = (N + KTILE - 1) / KTILE;
    int T = kv_tiles_all, Tw = kv_tiles_all;
    if (CAUSAL && !DUMP) {
        int last = (qt * QTILE + QTILE - 1) / KTILE + 1;
        T = last < kv_tiles_all ? last : kv_tiles_all;
        last = (qrow0 + WROWS - 1) / KTILE + 1;
        Tw = last < T ? last : T;
    }

    // ---- global -> register -> LDS staging.  Thread t moves the 16-byte vectors t, t+256, ...
    // of the (linear, unpadded) LDS tile; the global chunk it fetches is the swizzled one.  Rows
    // past N are clamped to the last row: their scores are masked, so the values never matter.
    v4i kpre[KL], vpre[VL];
    int k_goff[KL], v_goff[VL];          // byte offsets inside a full tile (row * pitch + swizzled chunk)
#pragma unroll
    for (int i = 0; i < KL; ++i) {
        int vidx = t + NTHREADS * i, row = vidx / KCH, c = (vidx % KCH) ^ k_swz<D>(row);
        k_goff[i] = row * D + c * 16;
    }
#pragma unroll
    for (int i = 0; i < VL; ++i) {
        int vidx = t + NTHREADS * i, row = vidx / VCH, c = (vidx % VCH) ^ v_swz<D>(row);
        v_goff[i] = row * 2 * D + c * 16;
    }
    const unsigned char* k_slab = (const unsigned char*)(ki + slab * D);
    const unsigned char* v_slab = (const unsigned char*)(vg + slab * D);
    auto fetch_k = [&](int j) {
        const int kv0 = j * KTILE, lim = N - 1 - kv0;
        const unsigned char* kt = k_slab + (size_t)kv0 * D;
#pragma unroll
        for (int i = 0; i < KL; ++i) {
            int row = k_goff[i] / D, rc = row < lim ? row : lim;
            if (k_mine) kpre[i] = *(const v4i*)(kt + k_goff[i] + (rc - row) * D);
        }
    };
    auto fetch_v = [&](int j) {
        if (DUMP) return;                 // the score dump never touches V
        const int kv0 = j * KTILE, lim = N - 1 - kv0;
        const unsigned char* vt = v_slab + (size_t)kv0 * 2 * D;
#pragma unroll
        for (int i = 0; i < VL; ++i) {
            int row = v_goff[i] / (2 * D), rc = row < lim ? row : lim;
            if (v_mine) vpre[i] = *(const v4i*)(vt + v_goff[i] + (rc - row) * 2 * D);
        }
    };
    auto stage_k = [&](int buf) {
#pragma unroll
        for (int i = 0; i < KL; ++i)
            if (k_mine) *(v4i*)(lds + buf * KB + (t + NTHREADS * i) * 16) = kpre[i];
    };
    auto stage_v = [&](int buf) {
        if (DUMP) return;
#pragma unroll
        for (int i = 0; i < VL; ++i)
            if (v_mine) *(v4i*)(lds + 2 * KB + buf * VB + (t + NTHREADS * i) * 16) = vpre[i];
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

    v16f acc_o[QS][DT];
    v16i acc_s[QS][2];
    v4i pk[QS][2][2];
    v16f acc_l[QS];          // row sums l, accumulated on the matrix pipe (every register of a lane holds its query's l)
    float m_run[QS];
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[qs][dt][r] = 0.0f;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) pk[qs][a][b] = (v4i){0, 0, 0, 0};
        m_run[qs] = -__builtin_inff();
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_l[qs][r] = 0.0f;
    }
    v8h ones8;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones8[e] = (_Float16)1.0f;

    v16i magic;
#pragma unroll
    for (int r = 0; r < 16; ++r) magic[r] = MAGIC_I;
    SAGE_PIN_MAGIC(magic);      // keep it resident (accumulator file): re-materializing costs 16 moves per sub-tile

    // ---- pieces of per-tile work
    // half of S^T = K^ Q^^T (INT8, int32 accumulate): 32-key sub-tile s of the K^ tile in buffer kbuf
    auto qk_half = [&](int kbuf, int s) {
        const unsigned char* kb = lds + kbuf * KB + s * 32 * KROW;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v4i a = *(const v4i*)(kb + k_off[ks]);
#pragma unroll
            for (int qs = 0; qs < QS; ++qs)
                acc_s[qs][s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, qreg[qs][ks], ks == 0 ? magic : acc_s[qs][s], 0, 0, 0);
        }
    };
    // O^T += V^T P~^T for the 16 keys of group (s, u) of the V tile in buffer vbuf
    auto pv_group = [&](int vbuf, int s, int u) {
        const unsigned char* vb = lds + 2 * KB + vbuf * VB + (32 * s + 16 * u) * VROW;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb + v_off[dt]));
            v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb + v_off[dt] + 8 * VROW));
            v8h a = __builtin_bit_cast(v8h, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int qs = 0; qs < QS; ++qs)
                acc_o[qs][dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, __builtin_bit_cast(v8h, pk[qs][s][u]), acc_o[qs][dt], 0, 0, 0);
        }
    };

    // Running-maximum bookkeeping for the tile whose scores sit in acc_s (tile j), done BETWEEN
    // pipeline steps so that the step itself stays one straight-line block:
    //   - on diagonal / tail tiles, hidden keys (beyond N, or after the query when causal) get the
    //     bit pattern of -inf, which the integer maximum ignores and which exponentiates to 0;
    //   - the running maximum is raised only if some row's tile maximum exceeds it by MAX_SLACK;
    //     then O, l and the not-yet-accumulated P~ of tile j-1 are rescaled (rare).
    float sc[QS], bias[QS];
    float dk_next = DUMP ? 0.0f : ksc_bh[0];
    auto prepare = [&](int j) {
        const int kv0 = j * KTILE;
        const float dk = dk_next;                      // loaded one step ahead
        {
            const int jn = j + 1 < kv_tiles_all ? j + 1 : j;
            dk_next = ksc_bh[(jn * KTILE) >> shift_k];
        }
        const bool need_mask = (kv0 + KTILE > N) || (CAUSAL && kv0 + KTILE - 1 > qrow0);
        float m_cand[QS];
        bool want = false;
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            // a zero scale (all-zero quantization block) would turn -inf * scale into NaN
            sc[qs] = __builtin_fmaxf(dq[qs] * dk, 1e-30f);
            if (need_mask) {
                const int q_row = qrow0 + 32 * qs + ql;
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                        bool hide = (key >= N) || (CAUSAL && key > q_row);
                        acc_s[qs][s][r] = hide ? (int)0xFF800000 : acc_s[qs][s][r];
                    }
            }
            int mi = acc_s[qs][0][0];
#pragma unroll
            for (int r = 1; r < 16; r += 2) mi = imax3(mi, acc_s[qs][0][r], acc_s[qs][0][(r + 1) & 15]);
#pragma unroll
            for (int r = 0; r < 16; r += 2) mi = imax3(mi, acc_s[qs][1][r], acc_s[qs][1][r + 1]);
            mi = max(mi, swap32i(mi));
            m_cand[qs] = (mi < 0) ? -__builtin_inff() : (as_f32(mi) - MAGIC_F) * sc[qs];
            want = want || (m_cand[qs] > m_run[qs] + MAX_SLACK);
        }
        if (__builtin_amdgcn_ballot_w64(want) != 0ull) {
#pragma unroll
            for (int qs = 0; qs < QS; ++qs) {
                const float m_new = __builtin_fmaxf(m_run[qs], m_cand[qs]);
                const float alpha = __builtin_amdgcn_exp2f(m_run[qs] - m_new);
                m_run[qs] = m_new;
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_l[qs][r] *= alpha;
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                const h2 a2 = {(_Float16)alpha, (_Float16)alpha};
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            int w = pk[qs][s][u][e];
                            pk[qs][s][u][e] = __builtin_bit_cast(int, __builtin_bit_cast(h2, w) * a2);
                        }
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc_o[qs][dt][r] *= alpha;
            }
        }
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) bias[qs] = -__builtin_fmaf(MAGIC_F, sc[qs], m_run[qs]);   // exp2 argument = acc*sc + bias
    };

    // One pipeline step, a single straight-line block: softmax of tile j (scores in acc_s, scale
    // and bias from prepare(j)), P~V of tile j-1, K^Q^^T of tile j+1.  For j = 0 the P~ registers
    // are zero and the V buffer that is read is zero-filled, so that P~V adds nothing.
    //
    // Flat operand sequence o = 0 .. 4*DT + 2*KS - 1: four P~V groups (DT operands each), then
    // the two K^Q^^T halves (KS operands each).  Operand o+1 is read from LDS before the matrix
    // instructions of operand o are issued.
    constexpr int NOPS = 4 * DT + 2 * KS;
    constexpr int PD = 2;        // LDS operands are read PD operands ahead of their matrix instructions
    v4i opnd[PD + 1];            // operand ring (V^T operands are reinterpreted)
    auto load_operand = [&](int o, int vbuf, int kbuf) {
        if (o < 4 * DT) {
            const int grp_su = o / DT, dt = o % DT;         // group (s,u) = (grp_su / 2, grp_su % 2)
            const unsigned char* vb = lds + 2 * KB + vbuf * VB + 16 * grp_su * VROW + v_off[dt];
            v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb));
            v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb + 8 * VROW));
            opnd[o % (PD + 1)] = __builtin_bit_cast(v4i, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            const int half = (o - 4 * DT) / KS, ks = (o - 4 * DT) % KS;
            opnd[o % (PD + 1)] = *(const v4i*)(lds + kbuf * KB + half * 32 * KROW + k_off[ks]);
        }
    };
    auto issue_mfma = [&](int o, int qs) {
        if (o < 4 * DT) {
            const int grp_su = o / DT, dt = o % DT;
            acc_o[qs][dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, opnd[o % (PD + 1)]),
                                                                    __builtin_bit_cast(v8h, pk[qs][grp_su >> 1][grp_su & 1]),
                                                                    acc_o[qs][dt], 0, 0, 0);
        } else {
            const int half = (o - 4 * DT) / KS, ks = (o - 4 * DT) % KS;
            acc_s[qs][half] = __builtin_amdgcn_mfma_i32_32x32x32_i8(opnd[o % (PD + 1)], qreg[qs][ks],
                                                                    ks == 0 ? magic : acc_s[qs][half], 0, 0, 0);
        }
    };
    // The softmax of a tile is cut into chunks of two scores of one query sub-tile; chunk ch
    // belongs to 16-key group ch / (4*QS).  A chunk passes three stages in three consecutive
    // pipeline ticks (scale+bias FMA, exp2, pack + row sum) so that dependent instructions of
    // one chunk are never adjacent in the single in-order instruction stream.
    constexpr int CHUNKS = 4 * QS;                     // chunks per 16-key group
    constexpr int NCH = 4 * CHUNKS;                    // chunks per tile
    float xs[3][2];
    auto chunk_fma = [&](int ch) {
        const int grp_su = ch / CHUNKS, cc = ch % CHUNKS, qs = cc / 4, pair = cc % 4;
        const int s_ = grp_su >> 1, r = 8 * (grp_su & 1) + 2 * pair;
        xs[ch % 3][0] = __builtin_fmaf(as_f32(acc_s[qs][s_][r]), sc[qs], bias[qs]);
        xs[ch % 3][1] = __builtin_fmaf(as_f32(acc_s[qs][s_][r + 1]), sc[qs], bias[qs]);
    };
    auto chunk_exp = [&](int ch) {
        xs[ch % 3][0] = __builtin_amdgcn_exp2f(xs[ch % 3][0]);
        xs[ch % 3][1] = __builtin_amdgcn_exp2f(xs[ch % 3][1]);
    };
    auto chunk_pack = [&](int ch) {
        // P~ is rounded to FP16 with round-to-nearest-even (one packed convert), as Algorithm 1 has it.
        typedef float f2 __attribute__((ext_vector_type(2)));
        typedef _Float16 h2 __attribute__((ext_vector_type(2)));
        const int grp_su = ch / CHUNKS, cc = ch % CHUNKS, qs = cc / 4, pair = cc % 4;
        const f2 pp = {xs[ch % 3][0], xs[ch % 3][1]};
        pk[qs][grp_su >> 1][grp_su & 1][pair] = __builtin_bit_cast(int, __builtin_convertvector(pp, h2));
    };
    auto step = [&](int j) {
        const int vbuf = (j - 1) & 1, kbuf = (j + 1) & 1;
        constexpr int MF_PER_SLOT = DT * QS;               // matrix instructions per slot (DT == KS)
        static_assert(CHUNKS % MF_PER_SLOT == 0, "whole chunks per matrix instruction");
        constexpr int CPM = CHUNKS / MF_PER_SLOT;          // pipeline ticks per matrix instruction
        constexpr int LEAD = MF_PER_SLOT - (2 + CPM - 1) / CPM;   // first tick: so that chunk 0 is packed right after slot A
#if SAGE_PHASED
        // matrix phase / VALU phase / matrix phase: overlap is left to the OTHER wavefront of the SIMD
        load_operand(0, vbuf, kbuf);
#pragma unroll
        for (int o = 0; o < 4 * DT; ++o) {
            if (o + 1 < 4 * DT) load_operand(o + 1, vbuf, kbuf);
#pragma unroll
            for (int qs = 0; qs < QS; ++qs) issue_mfma(o, qs);
        }
#pragma unroll
        for (int grp_su = 0; grp_su < 4; ++grp_su)
#pragma unroll
            for (int qs = 0; qs < QS; ++qs)
                acc_l[qs] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ones8, __builtin_bit_cast(v8h, pk[qs][grp_su >> 1][grp_su & 1]), acc_l[qs], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        load_operand(4 * DT, vbuf, kbuf);
#pragma unroll
        for (int n = 0; n < NCH + 2; ++n) {
            if (n - 2 >= 0 && n - 2 < NCH) chunk_pack(n - 2);
            if (n - 1 >= 0 && n - 1 < NCH) chunk_exp(n - 1);
            if (n >= 0 && n < NCH) chunk_fma(n);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int o = 4 * DT; o < NOPS; ++o) {
            if (o + 1 < NOPS) load_operand(o + 1, vbuf, kbuf);
#pragma unroll
            for (int qs = 0; qs < QS; ++qs) issue_mfma(o, qs);
        }
        __builtin_amdgcn_sched_barrier(0);
#else
#pragma unroll
        for (int o = 0; o < PD; ++o) load_operand(o, vbuf, kbuf);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int o = 0; o < NOPS; ++o) {
#ifndef SAGE_ABL_NOLDS
            if (o + PD < NOPS) load_operand(o + PD, vbuf, kbuf);
#endif
#pragma unroll
            for (int qs = 0; qs < QS; ++qs) {
#ifndef SAGE_ABL_NOMFMA
                issue_mfma(o, qs);
#endif
                const int mm = o * QS + qs;                // index of the matrix instruction in the step
#pragma unroll
                for (int c = 0; c < CPM; ++c) {
                    const int n = (mm - LEAD) * CPM + c;   // pipeline tick
#ifndef SAGE_ABL_NOVALU
                    if (n - 2 >= 0 && n - 2 < NCH) chunk_pack(n - 2);
                    if (n - 1 >= 0 && n - 1 < NCH) chunk_exp(n - 1);
                    if (n >= 0 && n < NCH) chunk_fma(n);
#endif
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (o < 4 * DT && o % DT == DT - 1) {
                // row sums of the 16-key group just consumed: l += 1^T P~^T on the matrix pipe
#pragma unroll
                for (int qs = 0; qs < QS; ++qs) {
                    const int grp_su = o / DT;
                    acc_l[qs] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ones8, __builtin_bit_cast(v8h, pk[qs][grp_su >> 1][grp_su & 1]),
                                                                        acc_l[qs], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#endif
    };

    auto dump_tile = [&](int j) {
        const int kv0 = j * KTILE;
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            const int q_row = qrow0 + 32 * qs + ql;
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (q_row < N && key < N) sdump[(slab + q_row) * (size_t)N + key] = acc_s[qs][s][r] - MAGIC_I;
                }
        }
    };

    // ---- prologue: K^(0), K^(1) into LDS; V(0), K^(2) into the staging registers; S_0
    if (!DUMP) {
#pragma unroll
        for (int i = 0; i < VL; ++i)
            if (v_mine) *(v4i*)(lds + 2 * KB + VB + (t + NTHREADS * i) * 16) = (v4i){0, 0, 0, 0};
    }
    fetch_k(0); stage_k(0);
    if (T > 1) { fetch_k(1); stage_k(1); }
    fetch_v(0);
    if (T > 2) fetch_k(2);
    __syncthreads();
    qk_half(0, 0);
    qk_half(0, 1);

    // ---- main loop.  At the top of iteration j the buffers of V(j-2) and K^(j) are free (their
    // last readers ran in iteration j-1): V(j) and K^(j+2) are written there from the staging
    // registers and the next pair is fetched.  Iteration j reads V(j-1) and K^(j+1).
    // Every wavefront passes T+1 barriers; the loops below are kept free of per-iteration branches
    // around the accumulators (straight-line bodies keep them in place in the register file).
    auto turn = [&](int j) {
#ifndef SAGE_ABL_NOBARRIER
        __syncthreads();
#endif
#ifndef SAGE_ABL_NOSTAGE
        if (j < T) stage_v(j & 1);
        if (j + 2 < T) stage_k(j & 1);
        if (j + 1 < T) fetch_v(j + 1);
        if (j + 3 < T) fetch_k(j + 3);
#endif
    };
    int j = 0;
    if (DUMP) {
        for (; j < T; ++j) {
            turn(j);
            dump_tile(j);
            qk_half((j + 1) & 1, 0);
            qk_half((j + 1) & 1, 1);
        }
        return;
    }
#ifdef SAGE_DBG_TIMING
    unsigned long long tacc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    unsigned long long tlast = __builtin_amdgcn_s_memtime();
    const unsigned long long tstart = tlast;
#endif
    for (; j < Tw; ++j) {
        TSTAMP(0);
#ifdef SAGE_ABL_CHEAPPREP
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) { sc[qs] = dq[qs] * 1e-5f; m_run[qs] = 20.0f; bias[qs] = -__builtin_fmaf(MAGIC_F, sc[qs], m_run[qs]); }
#else
        prepare(j);
#endif
        TSTAMP(1);
        turn(j);
        TSTAMP(2);
        step(j);
        TSTAMP(3);
    }
#ifdef SAGE_DBG_TIMING
    if (lane == 0 && gidx < 16384 / 8) {
        unsigned long long* d = g_timing + (gidx * 4 + wave) * 8;
        for (int k = 0; k < 5; ++k) d[k] = tacc[k];
        d[5] = __builtin_amdgcn_s_memtime() - tstart; d[6] = Tw; d[7] = tstart;
    }
#endif
    // the P~V of the wavefront's last tile ...
    turn(j);
    {
        const int vbuf = (j - 1) & 1;
        pv_group(vbuf, 0, 0); pv_group(vbuf, 0, 1); pv_group(vbuf, 1, 0); pv_group(vbuf, 1, 1);
#pragma unroll
        for (int grp_su = 0; grp_su < 4; ++grp_su)
#pragma unroll
            for (int qs = 0; qs < QS; ++qs)
                acc_l[qs] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ones8, __builtin_bit_cast(v8h, pk[qs][grp_su >> 1][grp_su & 1]), acc_l[qs], 0, 0, 0);
    }
    // ... and the wavefront keeps feeding the workgroup's tile pipeline until all are done.
    for (++j; j <= T; ++j) turn(j);

    // ---- O = diag(l)^-1 O, fp16 store
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
        const int q_row = qrow0 + 32 * qs + ql;
        const float inv = 1.0f / acc_l[qs][0];
        if (q_row < N) {
            _Float16* orow = og + (slab + q_row) * D;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    v4h w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = (_Float16)(acc_o[qs][dt][4 * rq + e] * inv);
                    *(v4h*)(orow + dt * 32 + 8 * rq + 4 * g) = w;
                }
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
        sage_attn_kernel<D, false, true><<<grid, NTHREADS, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, shift_q, shift_k, tiles_q, per_xcd, total);
    else if (causal)
        sage_attn_kernel<D, true, false><<<grid, NTHREADS, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, shift_q, shift_k, tiles_q, per_xcd, total);
    else
        sage_attn_kernel<D, false, false><<<grid, NTHREADS, 0, st>>>(qq, qscale, kq, kscale, vp, op, sdump, N, shift_q, shift_k, tiles_q, per_xcd, total);
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
