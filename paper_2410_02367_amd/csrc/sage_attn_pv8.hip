// SageAttention forward kernel with an INT8 second product for gfx950 (Section 4.3: P~ quantized
// per block with the static scale 1/127, V per channel; the SAGEAttn-vB / -vT kernels of Section 4.5).
//
// Same decomposition as the FP16-P~V kernel, in its plain form: a workgroup of 4 wavefronts owns 128
// query rows (32 per wavefront), K^ and V^^T tiles of 64 keys are double-buffered in LDS, scores are
// computed transposed (S^T = K^ Q^^T) so that a lane owns one query, and O^T = V^^T P^^T.  Both
// products use the 32x32x32 INT8 matrix instruction.  What is specific to this variant:
//
//   - Key order.  A lane's 16 result registers of a 32-key score block are the rows
//     8*(r/4) + 4*(lane/32) + r%4 of the instruction, but as the B operand of the second product
//     a lane must hold 16 CONSECUTIVE contraction indices.  The rows of K^ are therefore fed in a
//     permuted order (row 8g + 4h + b of the instruction is key 16h + 4g + b of the block): register
//     r of lane half h then is key 16h + r, the 16 codes of a lane pack into the B operand as they
//     are, and the matching A operand is 16 consecutive tokens of one channel -- one 16-byte read of
//     the channel-major V^^T tile.  The permutation is applied where the K^ tile is written to LDS.
//   - Exact running maximum.  The codes round(127 exp(S - m)) depend on m, so m is the exact
//     running maximum of the dequantized scores as in the recursion of Section 3.1 (no lazy update, no
//     grid rounding), and the largest code of a row is 127.
//   - Integer accumulation between maximum changes.  An int32 accumulator cannot be rescaled, so it
//     is flushed into an fp32 accumulator (O = (O + A) * alpha, A = 0; carried with the rescaling
//     factored out, so that a flush is a conversion and an FMA per element) whenever a row of the wavefront
//     raises its maximum (and every 1024 tiles, long before 64 * 127 * 127 * tiles reaches 2^31);
//     between two flushes alpha = 1 and the tiles' products add exactly in the matrix instruction.
//     The per-channel scale delta_V and the static 1/127 are constant over the row's whole loop and
//     are applied once, in the epilogue; l is carried as the sum of 127 P~ (fp32, unrounded P~),
//     which cancels the 1/127.
//   - 127 P~ = exp2(S' - (m' - log2 127)) comes out of the exponential directly; the packed
//     float-to-byte conversion rounds it to the nearest integer, ties to even, and packs four codes
//     into a register with one instruction per code.
//
// This variant is written with compiler builtins and compiler scheduling; it trades the second
// product's instruction count (half) for more VALU work per score (conversion, rounding, packing,
// flushes).  Measured on MI355X against the FP16-second-product kernel: 0-5 % faster at 16K keys,
// 8-15 % from 32K up (flushes are rare there), 3-6 % slower below 8K; it is bound by VALU issue
// (about 264 VALU instructions against 16 matrix instructions per 32 x 64 step).
#include "sage_internal.h"
#include <type_traits>

namespace sage {

typedef int p4i __attribute__((ext_vector_type(4)));
typedef int p16i __attribute__((ext_vector_type(16)));
typedef float p16f __attribute__((ext_vector_type(16)));
typedef _Float16 p4h __attribute__((ext_vector_type(4)));

namespace {
constexpr float PV8_LOG2E = 1.4426950408889634f;
constexpr float PV8_LOG2_127 = 6.988684686772166f;
constexpr float PV8_HIDDEN = -3.0e38f;            // stands for a masked score: finite, so that 0 * it is not NaN
constexpr int PV8_FLUSH_TILES = 1024;

__device__ __forceinline__ float lane32_partner(float v) { return __shfl_xor(v, 32, 64); }
// Raw-buffer descriptor of `bytes` bytes at `base` (wave-uniform, pinned to scalar registers): loads
// through it are range-checked by the hardware, lanes past the end read zero.
__device__ __forceinline__ p4i pv8_descriptor(const void* base, unsigned bytes) {
    const unsigned long long a = (unsigned long long)base;
    return (p4i){__builtin_amdgcn_readfirstlane((int)(unsigned)a),
                 __builtin_amdgcn_readfirstlane((int)((unsigned)(a >> 32) & 0xffffu)),
                 __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
}
// 16 bytes per lane from global memory straight into LDS (no staging registers): lane l lands at
// LDS byte lds_addr + 16 * l (lds_addr wave-uniform).  Asynchronous: the issuing wavefront waits
// with s_waitcnt vmcnt(0) before the barrier that publishes the tile.
__device__ __forceinline__ void pv8_load_to_lds16(const p4i& rsrc, unsigned goff, unsigned lds_addr) {
    const unsigned uniform_addr = (unsigned)__builtin_amdgcn_readfirstlane((int)lds_addr);      // pins it to a scalar register
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
                 : : "v"(goff), "s"(rsrc), "s"(uniform_addr) : "memory");
}
__device__ __forceinline__ int k_unperm(int p) {
    // key of a tile held by LDS row p: row 32kb + 8g + 4h + b holds key 32kb + 16h + 4g + b
    return (p & 32) | ((p & 4) << 2) | ((p & 24) >> 1) | (p & 3);
}
template <int D> __device__ __forceinline__ int k_swz8(int row) { return D == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); }
__device__ __forceinline__ int vt_swz(int ch) { return (ch >> 2) & 3; }
}  // namespace

template <int D, bool CAUSAL, bool KTOK, bool SPLIT>
__global__ void __launch_bounds__(256, 2)
sage_attn_pv8_kernel(const int8_t* __restrict__ qi, const float* __restrict__ qsc,
                     const int8_t* __restrict__ ki, const float* __restrict__ ksc,
                     const int8_t* __restrict__ vt, const float* __restrict__ vsc,
                     _Float16* __restrict__ og, float* __restrict__ lse,
                     int Nq, int Nkv, int Np, int shift_q, int shift_k, int tiles_q, int per_xcd, long total_tiles,
                     int BH, int n_splits, int chunk, int tm_group) {
    constexpr int NT = 256, QTILE = 128, KT = 64;
    constexpr int KS = D / 32, DT = D / 32;
    constexpr int KB = KT * D, VB = D * KT;            // bytes per K^ tile / V^^T tile
    constexpr int KCH = D / 16;                        // 16-byte chunks per K^ row
    constexpr int KL = KB / 16 / NT, VL = VB / 16 / NT;
    static_assert(KL >= 1 && VL >= 1, "tile loads cover whole workgroups");
    constexpr int KSL = KTOK ? KT * 4 : 0;             // per-key scales of a tile (per-token variant)
    // Q^ operands (B matrix of S^T = K^ Q^^T): QREG of the KS contraction steps stay in registers for
    // the whole kernel, the others are read from an LDS copy of the workgroup's Q^ rows tile after
    // tile (16 bytes per lane and step).  Registers are faster (no second LDS operand per matrix
    // instruction); the LDS copy is what keeps the pipeline below inside the register budget: 168
    // registers at D = 64 (three wavefronts per SIMD), 256 without spills at D = 128 with a causal mask.
    constexpr int QREG = D == 64 ? 0 : (CAUSAL ? 2 : KS);
    constexpr int QB = QREG < KS ? QTILE * D : 0;
    constexpr int QOFF = 3 * (KB + VB) + 3 * KSL;
    __shared__ __attribute__((aligned(16))) unsigned char lds[QOFF + QB];

    // workgroup -> (slab, query tile): contiguous ranges per XCD, heaviest query tiles first
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const long gidx = (long)xcd * per_xcd + slot;
    if (slot >= per_xcd || gidx >= total_tiles) return;
    int unit = (int)(gidx / tiles_q);                // (slab, key chunk), chunk fastest
    int qt = tiles_q - 1 - (int)(gidx % tiles_q);
    // causal launches: groups of tm_group slabs walked tile-major, heaviest query tiles first (see sage_attn.hip)
    if (tm_group > 0) {
        const int gi = slot / (tm_group * tiles_q), r = slot % (tm_group * tiles_q);
        unit = xcd * (per_xcd / tiles_q) + gi * tm_group + r % tm_group;
        qt = tiles_q - 1 - r / tm_group;
    }
    const int bh = SPLIT ? unit / n_splits : unit, split = SPLIT ? unit - bh * n_splits : 0;

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int ql = lane & 31, h = lane >> 5;
    const int qrow0 = qt * QTILE + wave * 32;
    const int q_row = qrow0 + ql;
    // Nq query rows against Nkv keys per slab; with a causal mask the queries are the last Nq tokens.
    // With n_splits > 1 the workgroup sees only the keys k0 .. k0 + N - 1 of its slab (chunk is a
    // multiple of 128 keys; the last chunk takes the remainder), runs the whole recursion on them --
    // own running maximum, hence own codes of P~ -- and leaves a partial result: its normalized O and,
    // per row, lse = m + log2(sum of 127 P~), from which the partial results of a row are merged.
    // N is the chunk's key count from here on.  SPLIT is a template parameter so that the unsplit
    // kernels keep their register allocation (as a run-time case it cost them 5-8 %).
    const int k0 = SPLIT ? split * chunk : 0;
    const int N = SPLIT ? (split == n_splits - 1 ? Nkv - k0 : chunk) : Nkv;
    const size_t slab = (size_t)bh * Nkv + k0, slab_q = (size_t)bh * Nq;
    const size_t slab_o = SPLIT ? ((size_t)split * BH + bh) * Nq : slab_q;
    const int coff = Nkv - Nq - k0;
    const int nbq = (Nq + (1 << shift_q) - 1) >> shift_q, nbk = (Nkv + (1 << shift_k) - 1) >> shift_k;

    p4i qreg[QREG > 0 ? QREG : 1];
#pragma unroll
    for (int ks = 0; ks < QREG; ++ks) {
        qreg[ks] = (p4i){0, 0, 0, 0};
        if (q_row < Nq) qreg[ks] = *(const p4i*)(qi + (slab_q + q_row) * D + ks * 32 + h * 16);
    }
    const float dq = qsc[(size_t)bh * nbq + ((q_row < Nq ? q_row : Nq - 1) >> shift_q)] * PV8_LOG2E;
    const float* __restrict__ ksc_bh = ksc + (size_t)bh * nbk + (k0 >> shift_k);

    const int kv_tiles_all = (N + KT - 1) / KT;
    int T = kv_tiles_all, Tw = kv_tiles_all;
    if (CAUSAL) {
        int last = (qt * QTILE + QTILE - 1 + coff) / KT + 1;
        T = last < kv_tiles_all ? last : kv_tiles_all;
        last = (qrow0 + 31 + coff) / KT + 1;
        Tw = last < T ? last : T;
    }

    // ---- tile loads: global -> LDS directly.  Instruction i of the workgroup fills the 16-byte
    // vectors NT*i + t of the (linear) LDS tile, one per lane; the global chunk a lane fetches is the
    // one that belongs there (row permutation and chunk swizzle inverted).  K^ rows past N lie beyond
    // the slab's descriptor and read as zero; V^^T rows are padded to whole tiles.
    // (instruction i of a tensor is instruction 0 plus a constant: NT / KCH further K^ rows -- a
    // multiple of 32, which neither the permutation nor the swizzle sees -- or 64 further channels)
    static_assert((NT / KCH) % 32 == 0, "K^ rows of consecutive load instructions differ by whole 32-key blocks");
    const unsigned k_goff0 = (unsigned)(k_unperm(t / KCH) * D + (((t % KCH) ^ k_swz8<D>(t / KCH)) * 16));
    const unsigned v_goff0 = (unsigned)((t >> 2) * Np + (((t & 3) ^ vt_swz(t >> 2)) * 16));
    const p4i k_desc = pv8_descriptor(ki + slab * D, (unsigned)N * D);
    const p4i v_desc = pv8_descriptor(vt + (size_t)bh * D * Np + k0, (unsigned)D * Np - (unsigned)k0);
    const p4i ks_desc = pv8_descriptor(ksc_bh, (unsigned)N * 4u);      // per-token variant: N scales; past the end reads 0
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    if (QREG < KS) {
        // same row pitch and chunk swizzle as a K^ tile (no key permutation); rows past Nq read as zero
        const p4i q_desc = pv8_descriptor(qi + slab_q * D, (unsigned)Nq * D);
#pragma unroll
        for (int i = 0; i < QB / 16 / NT; ++i) {
            const int vidx = t + NT * i, p = vidx / KCH, slot = vidx % KCH;
            pv8_load_to_lds16(q_desc, (unsigned)((qt * QTILE + p) * D + ((slot ^ k_swz8<D>(p)) * 16)),
                              lds_base + QOFF + wave * 1024 + i * (NT * 16));
        }
    }
    auto fetch = [&](int j, int buf) {
        if (KTOK && wave == 0 && lane < KT / 4)          // the tile's 64 key scales, 16 bytes per lane
            pv8_load_to_lds16(ks_desc, (unsigned)lane * 16u + (unsigned)j * (KT * 4), lds_base + 3 * (KB + VB) + buf * KSL);
        const unsigned kb_addr = lds_base + buf * (KB + VB) + wave * 1024;
#pragma unroll
        for (int i = 0; i < KL; ++i)
            pv8_load_to_lds16(k_desc, k_goff0 + (unsigned)(i * (NT / KCH) * D) + (unsigned)j * (KT * D), kb_addr + i * (NT * 16));
#pragma unroll
        for (int i = 0; i < VL; ++i)
            pv8_load_to_lds16(v_desc, v_goff0 + (unsigned)(i * (NT / 4)) * (unsigned)Np + (unsigned)j * KT, kb_addr + KB + i * (NT * 16));
    };

    // ---- operand read offsets (per lane, inside a buffer).  The swizzle of a row depends on the
    // row's low bits only, so the second 32-key block of K^ and the further 32-channel blocks of
    // V^^T are the first ones plus a constant: KS + 2 registers, the rest immediates.
    int k_rd0[KS], v_rd0[2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_rd0[ks] = ql * D + (((2 * ks + h) ^ k_swz8<D>(ql)) * 16);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) v_rd0[kb] = KB + ql * KT + (((2 * kb + h) ^ vt_swz(ql)) * 16);
    auto k_rd = [&](int kb, int ks) { return k_rd0[ks] + kb * (32 * D); };
    auto v_rd = [&](int cb, int kb) { return v_rd0[kb] + cb * (32 * KT); };

    p16i acc[DT];          // int32 product since the last flush
    p16f of[DT];           // fp32 accumulator in units of delta_V / 127; relative to the running maximum it counts g = 1 / ginv times
#pragma unroll
    for (int cb = 0; cb < DT; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc[cb][r] = 0; of[cb][r] = 0.0f; }
    float m_run = -__builtin_inff(), l127 = 0.0f, ginv = 1.0f;
    int since = 0;
    bool fresh = false;

    // Software pipeline over the key tiles.  The second 32-key half of a tile is finished one
    // iteration late, so that every group of matrix instructions but one has independent VALU work
    // next to it in the instruction stream:
    //     K^Q^^T of tile j (8 matrix instructions)            | codes of tile j-1, second half
    //     V^^T P^^T of tile j-1, second half (4)              | int -> float conversion of tile j's scores
    //     maximum, flush if a row's maximum rose (rare), codes of tile j, first half
    //     V^^T P^^T of tile j, first half (4)
    // State carried to the next iteration: the second half's 16 dequantizable scores per lane, the
    // tile's scale and softmax offset, and the LDS address of its V^^T tile (three tile buffers: that
    // tile is still read while tile j+1 is being loaded).
    p4i pk[2];             // codes: B operands of the second product
    float yp[16];          // second-half scores of the previous tile (per-token variant: already times delta_K)
    float sc_p = 1.0f, mb_p = 0.0f;
    bool pending = false;  // a second half is waiting
    const unsigned char* pend_tb = lds;
#pragma unroll
    for (int r = 0; r < 16; ++r) yp[r] = 0.0f;

    // second product, one 32-key half: O^T blocks += V^^T operand (LDS) x codes
    auto pv_half = [&](const unsigned char* tb, int kb, const p4i& codes, bool from_zero) {
        const p16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        if (from_zero) {          // wave-uniform
#pragma unroll
            for (int cb = 0; cb < DT; ++cb) {
                const p4i a = *(const p4i*)(tb + v_rd(cb, kb));
                acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, codes, zero, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int cb = 0; cb < DT; ++cb) {
                const p4i a = *(const p4i*)(tb + v_rd(cb, kb));
                acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, codes, acc[cb], 0, 0, 0);
            }
        }
    };
    // codes of 16 scores: 127 P~ (0 for hidden keys) out of the exponential; the packed conversion
    // rounds to the nearest integer, ties to even (checked on hardware), and inserts byte b
    auto codes16 = [&](const float* y16, float sc, float mb, p4i& out) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            unsigned word = 0u;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const float v = __builtin_amdgcn_exp2f(__builtin_fmaf(y16[4 * w + b], sc, -mb));
                l127 += v;
                word = __builtin_amdgcn_cvt_pk_u8_f32(v, (unsigned)b, word);
            }
            out[w] = (int)word;
        }
    };
    auto finish_previous = [&]() {          // a wavefront's last tile, or the drain after the loop
        codes16(yp, sc_p, mb_p, pk[1]);
        pv_half(pend_tb, 1, pk[1], false);
        pending = false;
    };

    // one tile; HAS_PREV (a compile-time constant) says whether a second half is waiting, so that the
    // deferred work sits in the same basic block as the matrix instructions it is to run beside
    auto tile = [&](int j, auto has_prev) {
        constexpr bool HAS_PREV = decltype(has_prev)::value;
        const int buf = j % 3;
        const unsigned char* tb = lds + buf * (KB + VB);
        // S^T block kb: keys 64j + 32kb + 16h + r in register r
        p16i s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kb][r] = 0;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const p4i a = *(const p4i*)(tb + k_rd(kb, ks));
                p4i b;
                if (ks < QREG) b = qreg[ks];
                else b = *(const p4i*)(lds + QOFF + wave * (32 * D) + k_rd0[ks]);      // this wavefront's Q^ rows
                s[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, s[kb], 0, 0, 0);
            }
        }
        if (HAS_PREV) {
            codes16(yp, sc_p, mb_p, pk[1]);
            pv_half(pend_tb, 1, pk[1], false);
        }
        // mask: keys past N, and keys after the lane's query when causal (edge tiles only)
        const bool edge = (j * KT + KT > N) || (CAUSAL && j * KT + KT - 1 > qrow0 + coff);
        // Per-block key scale: y = (float)S^ and sc = delta_Q log2(e) delta_K[tile]; per-token key
        // scales: y = (float)S^ * delta_K[key] and sc = delta_Q log2(e).  Either way the maximum is
        // taken on y and scaled once (sc > 0), and the softmax argument is one FMA, y * sc - m'.
        // Hidden scores become a huge negative number whose exponential is 0 (sc >= 1e-30 keeps the
        // product far below any maximum).
        const float sc = __builtin_fmaxf(KTOK ? dq : dq * ksc_bh[(j * KT) >> shift_k], 1e-30f);
        float y[2][16];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                y[kb][r] = (float)s[kb][r];
                if (KTOK) {
                    const float* kl = (const float*)(lds + 3 * (KB + VB) + buf * KSL);
                    y[kb][r] *= kl[32 * kb + 16 * h + r];
                }
            }
            // per-token variant: one half's 16 key scales in registers at a time
            if (KTOK && kb == 0) __builtin_amdgcn_sched_barrier(0);
        }
        if (edge) {          // wave-uniform: interior tiles skip the mask arithmetic
            asm volatile("" ::: "memory");      // keeps this a branch (not 64 compare-and-select pairs on every tile)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kidx = j * KT + 32 * kb + 16 * h + r;
                    if (kidx >= N || (CAUSAL && kidx > q_row + coff)) y[kb][r] = PV8_HIDDEN;
                }
        }
        float tmax = PV8_HIDDEN;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = __builtin_fmaxf(tmax, y[kb][r]);
        tmax *= sc;
        tmax = __builtin_fmaxf(tmax, lane32_partner(tmax));
        const float m_new = __builtin_fmaxf(m_run, tmax);
        ++since;
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0ull || since >= PV8_FLUSH_TILES) {
            // O relative to the running maximum is g * of + A with a per-lane factor g that takes
            // the rescaling: (g of + A) alpha = (g alpha) (of + A / g), so a flush is one conversion and
            // one FMA per element, of += A * (1 / g), and then g *= alpha.  1 / g = 2^(rise of the
            // maximum since the row began) is carried instead of g; the first tile (m_run = -inf,
            // of = A = 0) leaves it at 1.
#pragma unroll
            for (int cb = 0; cb < DT; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) of[cb][r] = __builtin_fmaf((float)acc[cb][r], ginv, of[cb][r]);
            const bool first = m_run == -__builtin_inff();
            l127 *= __builtin_amdgcn_exp2f(m_run - m_new);          // 0 on the first tile; l127 is 0 there
            // (a rise of more than 60 is taken as 60: what was accumulated before is then below 2^-60
            // of the new terms either way, and 1 / g stays finite: <= 2^60 * 2^60)
            ginv = first ? 1.0f : ginv * __builtin_amdgcn_exp2f(__builtin_fminf(m_new - m_run, 60.0f));
            if (__builtin_amdgcn_ballot_w64(ginv > 0x1p60f) != 0ull) {      // rare: fold g into of before 1 / g overflows
                const float g = ginv > 0x1p60f ? 1.0f / ginv : 1.0f;
#pragma unroll
                for (int cb = 0; cb < DT; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) of[cb][r] *= g;
                ginv = ginv > 0x1p60f ? 1.0f : ginv;
            }
            m_run = m_new;
            since = 0;
            fresh = true;          // the next product starts from zero inside the matrix instruction
        }
        const float mb = m_run - PV8_LOG2_127;
        codes16(y[0], sc, mb, pk[0]);
        // first half of the product; the first product after a flush starts from zero inside the
        // matrix instruction
        pv_half(tb, 0, pk[0], fresh);
        fresh = false;
#pragma unroll
        for (int r = 0; r < 16; ++r) yp[r] = y[1][r];
        sc_p = sc; mb_p = mb;
        pend_tb = tb;
        pending = true;
    };

    fetch(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // tile 0 has no predecessor (every wavefront computes it: Tw >= 1)
    if (1 < T) fetch(1, 1);
    tile(0, std::false_type{});
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wavefront's part of tile 1 has landed
    __syncthreads();
    for (int j = 1; j < T; ++j) {
        if (j + 1 < T) fetch(j + 1, (j + 1) % 3);
        if (j < Tw) tile(j, std::true_type{});
        else if (pending) finish_previous();
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wavefront's part of tile j + 1 has landed
        __syncthreads();
    }
    if (pending) finish_previous();

    // ---- epilogue: O = (O_fp32 + A) * delta_V[c] / sum(127 P~)
    const float lt = l127 + lane32_partner(l127);
    const float inv = 1.0f / lt, g_run = 1.0f / ginv;
    int q_out = q_row;
    if (SPLIT) asm volatile("" : "+v"(q_out));       // the output addresses are formed here, not carried through the loop
    if (q_out < Nq) {
        if (SPLIT && h == 0) lse[slab_o + q_out] = m_run + __builtin_amdgcn_logf(lt);
        _Float16* orow = og + (slab_o + q_out) * D;
        const float* dv = vsc + (size_t)bh * D;
#pragma unroll
        for (int cb = 0; cb < DT; ++cb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ch = 32 * cb + 8 * g + 4 * h;
                const float4 d4 = *(const float4*)(dv + ch);
                const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
                p4h o4;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const float tot = __builtin_fmaf(of[cb][4 * g + b], g_run, (float)acc[cb][4 * g + b]);
                    o4[b] = (_Float16)(tot * (dd[b] * inv));
                }
                *(p4h*)(orow + ch) = o4;
            }
    }
}

template <int D>
static hipError_t launch_pv8_d(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                               const int8_t* vt, const float* vscale, void* o, int BH, int Nq, int N, int causal,
                               int shift_q, int shift_k, bool ktok, const SplitPlan& sp, hipStream_t st) {
    const int tiles_q = (Nq + 127) / 128, Np = 64 * ((N + 63) / 64);
    const long total = (long)BH * sp.n_splits * tiles_q;
    const int per_xcd = (int)((total + 7) / 8);
    const dim3 grid((unsigned)(per_xcd * 8)), block(256);
    const int tm_group = causal ? tile_major_group(total, tiles_q, (long)(sp.n_splits > 1 ? sp.chunk : N) * 2 * D) : 0;
#define SAGE_PV8_S(C, K, S) sage_attn_pv8_kernel<D, C, K, S><<<grid, block, 0, st>>>( \
        qq, qscale, kq, kscale, vt, vscale, (_Float16*)o, sp.lse, Nq, N, Np, shift_q, shift_k, tiles_q, per_xcd, total, \
        BH, sp.n_splits, sp.chunk, tm_group)
#define SAGE_PV8(C, K) do { if (sp.n_splits > 1) SAGE_PV8_S(C, K, true); else SAGE_PV8_S(C, K, false); } while (0)
    if (causal) { if (ktok) SAGE_PV8(true, true); else SAGE_PV8(true, false); }
    else        { if (ktok) SAGE_PV8(false, true); else SAGE_PV8(false, false); }
#undef SAGE_PV8
#undef SAGE_PV8_S
    return hipGetLastError();
}

static hipError_t launch_pv8_plan(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                                  const int8_t* vt, const float* vscale, void* o, int BH, int Nq, int N, int D, int causal,
                                  int block_q, int block_k, const SplitPlan& sp, hipStream_t st) {
    int shift_q = 0, shift_k = 0;
    while ((1 << shift_q) < block_q) ++shift_q;
    while ((1 << shift_k) < block_k) ++shift_k;
    const bool ktok = block_k == 1;
    if (D == 64) return launch_pv8_d<64>(qq, qscale, kq, kscale, vt, vscale, o, BH, Nq, N, causal, shift_q, shift_k, ktok, sp, st);
    return launch_pv8_d<128>(qq, qscale, kq, kscale, vt, vscale, o, BH, Nq, N, causal, shift_q, shift_k, ktok, sp, st);
}

hipError_t launch_attn_pv8(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                           const int8_t* vt, const float* vscale, void* o, int BH, int Nq, int N, int D, int causal,
                           int block_q, int block_k, hipStream_t st) {
    const SplitPlan whole = {1, 0, nullptr};
    return launch_pv8_plan(qq, qscale, kq, kscale, vt, vscale, o, BH, Nq, N, D, causal, block_q, block_k, whole, st);
}

// The keys cut into chunks, as in launch_attn_split(): same plan, same workspace layout, same merge
// (the common factor 127 of the chunks' denominators cancels in the weights).
hipError_t launch_attn_pv8_split(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                                 const int8_t* vt, const float* vscale, void* o, void* workspace, int BH, int Nq, int N,
                                 int D, int causal, int block_q, int block_k, int requested, hipStream_t st) {
    SplitPlan sp = plan_split(BH, Nq, N, causal, requested);
    if (sp.n_splits == 1) return launch_attn_pv8(qq, qscale, kq, kscale, vt, vscale, o, BH, Nq, N, D, causal, block_q, block_k, st);
    const long rows = (long)BH * Nq;
    sp.lse = (float*)((char*)workspace + (size_t)sp.n_splits * rows * D * sizeof(_Float16));
    hipError_t e = launch_pv8_plan(qq, qscale, kq, kscale, vt, vscale, workspace, BH, Nq, N, D, causal, block_q, block_k, sp, st);
    if (e != hipSuccess) return e;
    return launch_merge_splits(workspace, sp.lse, o, rows, D, sp.n_splits, st);
}

}  // namespace sage
