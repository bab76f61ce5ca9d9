// Fused SageAttention forward kernel for gfx950 (Algorithm 1, inner loops).
//
// Work decomposition
//   One workgroup = 8 wavefronts (two per SIMD, 256 registers each) = 256 query rows, 32 per
//   wavefront; for D = 64, for short sequences and for small problems 4 wavefronts = 128 rows,
//   two or three workgroups per CU.
//   Key/value tiles of 64 tokens are double-buffered in LDS and shared by all wavefronts of the
//   workgroup; they are brought in by asynchronous, range-checked buffer loads that write LDS
//   directly and bypass the register file.
//   Scores are computed TRANSPOSED, S^T = K^ Q^^T, with the 32x32x32 INT8 matrix instruction: each
//   lane then owns one query column and 16 keys per 32-key sub-tile, so
//     - the row maximum needs one cross-lane step (lane <-> lane+32), the row sum none (see l_mfma),
//     - the exponentiated scores are already in the register layout the FP16 32x32x16 instruction
//       wants for its B operand (P~^T), and O^T = V^T P~^T accumulates with the rescale factor
//       being a per-lane scalar.
//   V^T operands come from the row-major V tile in LDS through the transposing LDS read.
//
// Schedule (software pipeline inside every wavefront)
//   A wavefront issues its instructions in order, and VALU work hides behind a matrix instruction
//   only in the stream that issued it: a probe with one wavefront of a SIMD issuing matrix
//   instructions and the other the softmax takes the sum of both times.  Every wavefront therefore
//   runs three tiles at once: the softmax of
//   tile j (VALU) is spread between the matrix instructions of P~V of tile j-1 and K^Q^^T of tile
//   j+1.  A step is a flat sequence of LDS operands, each feeding one matrix instruction per query
//   sub-tile, with VALU work after every matrix instruction, fenced so the order survives:
//        slot A  PV_{j-1}[ 0:16] | row maximum of S_j   slot D  PV_{j-1}[48:64] | softmax_j[32:48]
//        slot B  PV_{j-1}[16:32] | softmax_j[ 0:16]     slot E  QK_{j+1}[ 0:32] | softmax_j[48:64]
//        slot C  PV_{j-1}[32:48] | softmax_j[16:32]     slot F  QK_{j+1}[32:64]
//   (a softmax "chunk" = 2 scores: 2 FMA, 2 exp2, 1 pack).  S and P~ live in single register
//   buffers: a 16-key group of P~_{j-1} is consumed by its matrix instructions before the softmax
//   overwrites it, and each half of S_{j+1} is produced after the softmax has consumed that half
//   of S_j.
//   The running maximum is only raised when a row's tile maximum exceeds it by more than 2^8
//   (P~ <= 256 fits FP16 comfortably); the rescale of O is then a rare branch between slots A and B.
//   Inside a softmax slot the order is: matrix instruction, the LDS reads of the operand three
//   instructions ahead, the chunk's VALU work.  At D = 128 two steps share one loop body, so that the
//   buffer parity is a constant and every LDS address is a register plus an immediate.
//
// Register files
//   The matrix instructions are written as inline assembly so that the register file of every
//   operand is chosen by hand: O^T (QS*DT*16 registers), the row sums, the resident Q^ operands
//   and the row-sum selector operand are pinned in the accumulator file (AGPRs) -- only matrix instructions
//   touch them in the steady state, so there are no AGPR<->VGPR moves at all -- while scores, P~,
//   LDS operands and staging data are ordinary variables in VGPRs.
//   The O^T / row-sum statements name their accumulator as an INPUT and update that register
//   behind the compiler's back: to the compiler the accumulators are loop-invariant values, which
//   it keeps in one place; refresh() ("+a") tells it the truth before C++ code reads them (rare
//   rescale, epilogue).  This only works while the compiler never copies such a value to a second
//   register inside the loops, so the build inspects the generated assembly for that.
//   The compiler does not know these are matrix instructions, so the waits it would insert are
//   placed by hand:
//     - 12 wait states between a matrix instruction that writes a register and a VALU or memory
//       instruction that reads or writes it (score_fence(), refresh());
//     - 2 wait states between a VALU write of a register and a matrix instruction reading it --
//       guaranteed by construction: P~ is packed at least one slot before it is consumed.
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
//     that FMA rounds once only if its bias -(12582912 * sc + m) is exact, which holds because sc
//     carries 22 significant bits and m is kept on the grid of 12582912 * sc (see begin_tile(),
//     finish_max(), raise_maximum());
//   - the row maximum is taken on the raw accumulators with integer max;
//   - P~ is packed to FP16 with the packed round-to-nearest-even convert; the row sum l comes from
//     one 16x16x32 FP16 matrix instruction per 16 keys whose A operand selects, for every query, the
//     contraction blocks that hold its keys (see l_mfma): l is exactly the sum of the FP16 P~ that
//     multiplies V, and costs no VALU issue slot.  (Dot-product instructions such as v_dot2c run on the
//     matrix pipe as well, but block it for VALU work -- measured.)
#include "sage_internal.h"
#include <type_traits>
#include <utility>

namespace sage {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef short v4s __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// Shape of a workgroup: NW wavefronts (a template parameter of the kernel, 8 or 4) of WROWS rows.
//   8 wavefronts, one workgroup per CU  -- two wavefronts per SIMD share one set of LDS tiles;
//   4 wavefronts, two or three workgroups per CU -- chosen by the launcher for D = 64, for short
//                                          sequences and whenever the larger tile would leave CUs
//                                          without work (see launch_d()).
// QS = 2 (64 rows per wavefront, every LDS operand feeding two matrix instructions, one wavefront
// per SIMD) is what the QS loops in the kernel are for; an earlier version measured it 2-3 % slower
// than QS = 1, and the build and the tests cover QS = 1 only.
#ifndef SAGE_QS
#define SAGE_QS 1
#endif
// SAGE_SA: P~V groups issued ahead of the softmax, beside the row maximum (see "Schedule of a step"
// in the kernel).  2 gives the maximum more matrix instructions to hide behind and packs the softmax
// chunks denser afterwards; it measured equal at D = 128 and 1 % slower at D = 64.
#ifndef SAGE_SA
#define SAGE_SA 1
#endif
constexpr int QS = SAGE_QS;            // 32-row query sub-tiles per wavefront
constexpr int WROWS = 32 * QS;         // query rows per wavefront
constexpr int KTILE = 64;              // keys per LDS tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr int MAGIC_I = 0x4B400000;        // bit pattern of 12582912.0f = 1.5 * 2^23
constexpr float MAGIC_F = 12582912.0f;
constexpr float MAX_SLACK = 8.0f;          // log2 of the largest P~ tolerated before the maximum is raised

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}).
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F& f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }
#define IDX(x) (std::remove_reference_t<decltype(x)>::value)

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

// Which softmax pipeline ticks run behind matrix instruction i of a step's second part: the first
// MB instructions share the NCH chunk entries as evenly as they divide, the two after them take
// the two ticks that drain the three-stage chunk pipeline.
template <int NCH, int MB>
struct TickPlan {
    static constexpr int first(int i) { return i < MB ? i * NCH / MB : NCH + (i - MB); }
    static constexpr int end(int i) { return i < MB ? (i + 1) * NCH / MB : (i - MB < 2 ? NCH + (i - MB) + 1 : NCH + (i - MB)); }
    static constexpr int slot_of(int n) { int i = 0; while (end(i) <= n) ++i; return i; }
};

// ---- matrix instructions, register files chosen by hand
// S^T block: scores in VGPRs (the softmax reads them with VALU instructions); the destination and
// the accumulator input of one instruction must sit in the same register file, so the seed is a
// VGPR tuple as well.  The Q^ operand is pinned in AGPRs.
__device__ __forceinline__ void qk_mfma_first(v16i& acc, const v4i& a, const v4i& q, const v16i& seed) {
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %3" : "=&v"(acc) : "v"(a), "a"(q), "v"(seed));
}
__device__ __forceinline__ void qk_mfma_next(v16i& acc, const v4i& a, const v4i& q) {
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(q));
}
// O^T block acc += V^T operand (VGPRs, from LDS) x P~^T operand (VGPRs).  acc is declared as an
// input and modified in place (see "Register files" above).
__device__ __forceinline__ void pv_mfma(const v16f& acc, const v8h& a, const v8h& b) {
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : : "a"(acc), "v"(a), "v"(b));
}
// Row sums on the matrix pipe: ONE 16x16x32 FP16 instruction per 16-key group.  Its B operand is the
// group's P~^T operand as it stands (lane l: query l % 32, the 8 keys of half l / 32).  Read in the
// 16x16x32 layout the same registers are "column l % 16, contraction block l / 16": blocks 0 and 2 hold
// the two key halves of query l % 16, blocks 1 and 3 those of query 16 + l % 16.  The A operand `sel`
// has ones in the blocks of the row's parity and zeros in the others (row i: blocks with the parity of
// i), so result row i of column c is the complete 16-key sum of query c (i even) or 16 + c (i odd); a
// lane's result registers 0 and 1 (rows 4 (l / 16) + 0, + 1 of column l % 16) are the row sums of the
// queries l % 16 and 16 + l % 16, and the one that is the lane's own query is selected in the epilogue.
// No VALU slot, no cross-lane step, 18 clocks of the matrix pipe in the stream of 32-clock
// instructions (measured; two of the 4x4x4 instructions, which did this before, took 27).  acc += sums;
// same in-place convention as pv_mfma.
__device__ __forceinline__ void l_mfma(const v4f& acc, const v4i& sel, const v4i& b) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : : "a"(acc), "a"(sel), "v"(b));
}
// One 16-byte-per-lane load from global memory straight into LDS: lane l lands at LDS byte address
// lds_addr + 16*l (lds_addr wave-uniform).  Written as assembly because the compiler, which cannot
// tell which LDS bytes such a load writes, makes every later LDS read wait for it (vmcnt(0)) and
// so turns the asynchronous load into a synchronous one.  Completion is tracked by hand: the
// issuing wavefront waits with s_waitcnt vmcnt before the barrier that publishes the tile.
//
// The load is a raw-buffer load: the descriptor (four scalar registers) carries the base address
// and the byte size of the (batch, head) slab, the per-lane offset is checked against that size by
// the hardware and a lane beyond it reads zero instead of memory.  The ragged last tile therefore
// needs no clamping code at all (its rows are masked or multiplied by P~ = 0 anyway).
__device__ __forceinline__ v4i slab_descriptor(const void* base, unsigned bytes) {
    const unsigned long long p = (unsigned long long)base;
    // dword 0-1: 48-bit base, stride 0 (raw buffer); dword 2: size in bytes; dword 3: 32-bit data format
    // (readfirstlane: the values are wave-uniform, this pins them to scalar registers)
    return (v4i){__builtin_amdgcn_readfirstlane((int)(unsigned)p),
                 __builtin_amdgcn_readfirstlane((int)((unsigned)(p >> 32) & 0xffffu)),
                 __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
}
// The descriptor of a slab moved forward to one of its tiles: base + tile bytes, size - tile bytes
// (scalar arithmetic).  The per-lane offset inside the tile then goes into the load as it is, and
// the range check still ends at the end of the slab.  (Adding the tile offset to the per-lane
// offset instead costs a VALU instruction per load; the scalar-offset field of the instruction
// would not do: it is not part of the range check.)
__device__ __forceinline__ v4i tile_descriptor(const v4i& slab, unsigned tile) {
    const unsigned lo = (unsigned)slab[0] + tile;
    const unsigned hi = (unsigned)slab[1] + (lo < tile ? 1u : 0u);
    return (v4i){(int)lo, (int)hi, (int)((unsigned)slab[2] - tile), slab[3]};
}
__device__ __forceinline__ void load_to_lds16(const v4i& rsrc, unsigned goff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
                 : : "v"(goff), "s"(rsrc), "s"(lds_addr) : "memory");
}
// Tells the compiler that an accumulator changed, 12 wait states after the last matrix instruction
// that wrote it (all of these statements are volatile, so their order is kept).
__device__ __forceinline__ void refresh(v16f& acc) { asm volatile("s_nop 11" : "+a"(acc)); }
__device__ __forceinline__ void refresh(v4f& acc) { asm volatile("s_nop 11" : "+a"(acc)); }
// Makes a value opaque and resident in the accumulator file.
template <class T> __device__ __forceinline__ void pin_a(T& x) { asm volatile("" : "+a"(x)); }

// KTOK: one scale per key token (Section 3.2's per-token quantizer, the SAGEAttn-T kernel of
// Section 4.5) instead of one per block of keys.  A lane's 32 scores of a tile then belong to 32
// different scales, so the dequantization cannot be folded into the softmax FMA: wavefront 0
// stages, per tile, a_k = delta_K[k] and b_k = -12582912 * a_k in LDS, every wavefront turns its
// raw scores into t = S^ * delta_K[k] = fma(seeded score, a_k, b_k) while it takes the row maximum
// (now a floating-point maximum), and the softmax FMA becomes t * (delta_Q log2 e) - m.  One
// scale per QUERY token costs nothing in either variant: a lane owns one query.
//
// CLOCKS (measurement build of the same kernel): every wavefront also leaves the shader-clock and
// constant-rate (100 MHz) counter ticks it ran for, how often it raised a running maximum and how
// many key tiles it visited -- from which the clock the chip held and the clocks per tile follow.
template <int D, int NW, bool CAUSAL, bool DUMP, bool KTOK, bool CLOCKS = false>
// Workgroups of 4 wavefronts per CU that the register budget is cut for: 3 at D = 64 (168 registers
// per lane; measured 4 % faster than 2; the per-token variant needs more), else 2.
__global__ void __launch_bounds__(NW * 64, NW == 4 && SAGE_QS == 1 ? 2 : 1)
sage_attn_kernel(const int8_t* __restrict__ qi, const float* __restrict__ qsc,
                 const int8_t* __restrict__ ki, const float* __restrict__ ksc,
                 const _Float16* __restrict__ vg, _Float16* __restrict__ og,
                 int32_t* __restrict__ sdump, float* __restrict__ lse, unsigned long long* __restrict__ clocks,
                 int Nq, int Nkv, int shift_q, int shift_k, int tiles_q, int per_xcd, long total_tiles,
                 int BH, int n_splits, int chunk, int tm_group) {
    constexpr int NWAVES = NW, NTHREADS = NW * 64;
    constexpr int QTILE = NW * WROWS;   // query rows per workgroup
    constexpr int KROW = D;             // bytes per K^ row in LDS
    constexpr int VROW = 2 * D;         // bytes per V row in LDS
    constexpr int KB = KTILE * KROW;    // bytes per K^ tile
    constexpr int VB = KTILE * VROW;    // bytes per V tile
    constexpr int KS = D / 32;          // INT8 MFMA steps along the head dimension
    constexpr int DT = D / 32;          // 32-wide output tiles along the head dimension
    constexpr int KVEC = KB / 16, VVEC = VB / 16;               // 16-byte vectors per tile
    static_assert(KVEC % 64 == 0 && VVEC % 64 == 0, "whole vectors per wavefront instruction");
    // load instructions per wavefront and tile (the last may cover only the first wavefronts)
    constexpr int KL = (KVEC + NTHREADS - 1) / NTHREADS, VL = (VVEC + NTHREADS - 1) / NTHREADS;
    constexpr int KCH = KROW / 16, VCH = VROW / 16;             // chunks per row
    static_assert(!(KTOK && DUMP), "the score dump has no scales");
    constexpr int KSL = KTOK ? 2 * 2 * KTILE * 4 : 0;           // per-key (a, b) factors, two tiles
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * KB + 2 * VB + KSL];

    // Workgroup -> (slab, query tile).  Consecutive workgroup ids land on the 8 XCDs in turn; give
    // each XCD a contiguous range of the (slab-major, heaviest-query-tile-first) order so that the
    // workgroups resident on one XCD share K^/V in its L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const long gidx = (long)xcd * per_xcd + slot;
    if (slot >= per_xcd || gidx >= total_tiles) return;
    int unit = (int)(gidx / tiles_q);                // (slab, key chunk), chunk fastest
    int qt = tiles_q - 1 - (int)(gidx % tiles_q);
    // With a causal mask the query tiles of a slab differ in weight by up to tiles_q : 1, and slab-major the
    // last slab's light tiles fill in behind the other slabs' heavy ones: the tail of the launch is as long
    // as a heavy tile.  tm_group > 0 (chosen by the launcher, see tile_major_group()): the XCD's range, a
    // whole number of slabs, is walked in groups of tm_group slabs, tile-major inside a group -- the heaviest
    // query tile of each of the group's slabs first, the lightest ones last.
    if (tm_group > 0) {
        const int gi = slot / (tm_group * tiles_q), r = slot % (tm_group * tiles_q);
        unit = xcd * (per_xcd / tiles_q) + gi * tm_group + r % tm_group;
        qt = tiles_q - 1 - r / tm_group;
    }
    const int bh = unit / n_splits, split = unit - bh * n_splits;

    unsigned long long clock_t0 = 0, clock_r0 = 0;
    int n_raised = 0;
    if constexpr (CLOCKS) { clock_t0 = __builtin_readcyclecounter(); clock_r0 = wall_clock64(); }
    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);     // wave-uniform: keeps control flow scalar
    const int ql = lane & 31, g = lane >> 5;
    const int qrow0 = qt * QTILE + wave * WROWS;     // first row of the wavefront; sub-tile qs starts 32*qs later
    // Nq query rows against N keys per slab (the paper's setting is Nq = N).  With a causal mask the
    // queries are the LAST Nq tokens: query row t sits at position t + coff among the keys.
    // With n_splits > 1 the workgroup sees only the keys k0 .. k0 + N - 1 of its slab (chunk is a
    // multiple of the key tile and of the K block; the last chunk takes the remainder) and leaves a
    // partial result: its own normalized O and, per row, log2 of its softmax denominator in absolute
    // terms (lse), from which the partial results of a row are merged.  N is the chunk's key count
    // from here on; one chunk is the whole slab.
    const int k0 = split * chunk;
    const int N = split == n_splits - 1 ? Nkv - k0 : chunk;
    const size_t slab = (size_t)bh * Nkv + k0, slab_q = (size_t)bh * Nq;
    const size_t slab_o = ((size_t)split * BH + bh) * Nq;
    const int coff = Nkv - Nq - k0;
    const int nbq = (Nq + (1 << shift_q) - 1) >> shift_q, nbk = (Nkv + (1 << shift_k) - 1) >> shift_k;

    // Q^ operands (B matrix of S^T = K^ Q^^T) stay in accumulator registers for the whole kernel.
    v4i qreg[QS][KS];
    float dq[QS];
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
        const int q_row = qrow0 + 32 * qs + ql;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qreg[qs][ks] = (v4i){0, 0, 0, 0};
            if (q_row < Nq) qreg[qs][ks] = *(const v4i*)(qi + (slab_q + q_row) * D + ks * 32 + g * 16);
            pin_a(qreg[qs][ks]);
        }
        dq[qs] = 0.0f;
        if (!DUMP) {
            const int rc = q_row < Nq ? q_row : Nq - 1;           // the lane's own query: any block_q down to 1
            dq[qs] = qsc[(size_t)bh * nbq + (rc >> shift_q)] * LOG2E;
        }
    }
    v16f acc_o[QS][DT];      // O^T accumulators
    // Row sums l, accumulated on the matrix pipe (see l_mfma): registers 0 and 1 hold the sums of the
    // queries lane % 16 and 16 + lane % 16 over all keys so far.
    v4f acc_l[QS];
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[qs][dt][r] = 0.0f;
            pin_a(acc_o[qs][dt]);
        }
        acc_l[qs] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
        pin_a(acc_l[qs]);
    }
    // selector operand of the row-sum instruction: FP16 ones in the contraction blocks of the row's parity
    const int sel_word = (((lane >> 4) ^ lane) & 1) ? 0 : 0x3C003C00;
    v4i sel = {sel_word, sel_word, sel_word, sel_word};
    pin_a(sel);
    const float* __restrict__ ksc_bh = ksc + (size_t)bh * nbk + (k0 >> shift_k);

    // kv tiles visited by the workgroup (T) and by this wavefront (Tw <= T: tiles above the
    // wavefront's last row are skipped when causal)
    const int kv_tiles_all = (N + KTILE - 1) / KTILE;
    int T = kv_tiles_all, Tw = kv_tiles_all;
    if (CAUSAL && !DUMP) {
        int last = (qt * QTILE + QTILE - 1 + coff) / KTILE + 1;
        T = last < kv_tiles_all ? last : kv_tiles_all;
        last = (qrow0 + WROWS - 1 + coff) / KTILE + 1;
        Tw = last < T ? last : T;
    }

    // ---- global -> LDS tile loads without staging registers (the load unit writes LDS directly).
    // Instruction i of wavefront w fills the 16-byte vectors (NTHREADS*i + 64*w) .. +63 of the
    // (linear, unpadded) LDS tile, one per lane; the global chunk a lane fetches is the swizzled
    // one.  Rows past N lie beyond the slab's descriptor and are not fetched: their scores are masked
    // and their P~ is zero, so the values never matter (as long as the V rows are finite: see the
    // prologue).  The loads are asynchronous: a wavefront waits for its own (vmcnt) before the
    // barrier that publishes the tile.
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
    const v4i k_rsrc = slab_descriptor(ki + slab * D, (unsigned)N * D);
    const v4i v_rsrc = slab_descriptor(vg + slab * D, (unsigned)N * 2 * D);
    const unsigned lds_base = (unsigned)(size_t)LDS_PTR(unsigned char, lds);     // LDS byte address of the tile area
    auto load_k = [&](int j, int buf) {
        const v4i rsrc = tile_descriptor(k_rsrc, (unsigned)j * (KTILE * D));
#pragma unroll
        for (int i = 0; i < KL; ++i) {
            if (NTHREADS * (i + 1) > KVEC && NTHREADS * i + wave * 64 >= KVEC) continue;   // piece beyond the tile for this wavefront
            load_to_lds16(rsrc, k_goff[i], lds_base + buf * KB + (NTHREADS * i + wave * 64) * 16);
        }
    };
    auto load_v = [&](int j, int buf) {
        if (DUMP) return;                 // the score dump never touches V
        const v4i rsrc = tile_descriptor(v_rsrc, (unsigned)j * (KTILE * 2 * D));
#pragma unroll
        for (int i = 0; i < VL; ++i) {
            if (NTHREADS * (i + 1) > VVEC && NTHREADS * i + wave * 64 >= VVEC) continue;
            load_to_lds16(rsrc, v_goff[i], lds_base + 2 * KB + buf * VB + (NTHREADS * i + wave * 64) * 16);
        }
    };
    // own tile loads landed (vmcnt(0)), then the workgroup barrier
    auto tiles_ready_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0); expcnt and lgkmcnt fields at their maximum = no wait
        __syncthreads();
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

    v16i acc_s[QS][2];       // S^T of the current tile, two 32-key halves per sub-tile (raw int32 + seed)
    v4i pk[QS][2][2];        // P~^T as FP16 pairs: [sub-tile][32-key half][16-key group]
    float m_run[QS], sc[QS], bias[QS], m_cand[QS];
    bool off_grid[QS];       // the running maximum is not on the grid on which this tile's bias is exact
    int pmax[QS][DT];        // partial integer row maxima of the current tile
    float pmaxf[QS][DT];     // ... floating-point ones when every key has its own scale
    // P~V groups (of DT matrix instructions) that a step issues before the softmax starts, i.e.
    // while the row maximum is being taken
    constexpr int SA = SAGE_SA;
    constexpr int NA = SA * DT;
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) pk[qs][a][b] = (v4i){0, 0, 0, 0};
        m_run[qs] = -__builtin_inff();
        sc[qs] = 0.0f; bias[qs] = 0.0f; m_cand[qs] = 0.0f; off_grid[qs] = false;
    }
    v16i magic;
#pragma unroll
    for (int r = 0; r < 16; ++r) magic[r] = MAGIC_I;
    asm volatile("" : "+v"(magic));      // keep it resident: re-materializing costs 16 moves per sub-tile
    float dk_next = (DUMP || KTOK) ? 0.0f : ksc_bh[0];
    // KTOK: wavefront 0 carries the scale of key (tile j, lane) from the load in slot j-1 to the
    // LDS write before barrier j.
    float dk_tok = 0.0f;
    float* const ksl = (float*)(lds + 2 * KB + 2 * VB);          // [tile parity][a | b][key]
    auto request_key_scales = [&](int j) {
        if constexpr (KTOK) {
            if (wave == 0) {
                const int key = j * KTILE + lane;
                dk_tok = ksc_bh[key < N ? key : N - 1];
            }
        }
    };
    auto publish_key_scales = [&](int par) {
        if constexpr (KTOK) {
            if (wave == 0) {
                // a zero scale (all-zero token) would turn -inf * scale into NaN for hidden keys
                // 22 significant bits, so that 12582912 * a = 3 * 2^22 * a is exact and the fma
                // below returns S^ * a rounded once
                const float a = as_f32(as_i32(__builtin_fmaxf(dk_tok, 1e-30f)) & ~3);
                ksl[par * 2 * KTILE + lane] = a;
                ksl[par * 2 * KTILE + KTILE + lane] = -MAGIC_F * a;
            }
        }
    };

    // 12 wait states between the matrix instructions that wrote the scores and the first VALU or
    // memory instruction that touches them; the operands tie every later use to the fence.
    auto score_fence = [&]() {
        static_assert(QS == 1 || QS == 2, "the fence lists the score registers explicitly");
        if constexpr (QS == 2) asm volatile("s_nop 11" : "+v"(acc_s[0][0]), "+v"(acc_s[0][1]), "+v"(acc_s[QS - 1][0]), "+v"(acc_s[QS - 1][1]));
        else asm volatile("s_nop 11" : "+v"(acc_s[0][0]), "+v"(acc_s[0][1]));
    };
    // The same tie without the pause, for the main loop: there the barrier and the tile requests of
    // turn() already stand between the matrix instructions and the first use (the build's assembly
    // check counts the wait states).
    auto score_tie = [&]() {
        if constexpr (QS == 2) asm volatile("" : "+v"(acc_s[0][0]), "+v"(acc_s[0][1]), "+v"(acc_s[QS - 1][0]), "+v"(acc_s[QS - 1][1]));
        else asm volatile("" : "+v"(acc_s[0][0]), "+v"(acc_s[0][1]));
    };

    // ---- pieces of per-tile work
    // half of S^T = K^ Q^^T (INT8, int32 accumulate): 32-key sub-tile s of the K^ tile in buffer kbuf
    auto qk_half = [&](int kbuf, auto S) {
        constexpr int s = IDX(S);
        const unsigned char* kb = lds + kbuf * KB + s * 32 * KROW;
        static_for<KS>([&](auto KSI) {
            constexpr int ks = IDX(KSI);
            const v4i a = *(const v4i*)(kb + k_off[ks]);
            static_for<QS>([&](auto QSI) {
                constexpr int qs = IDX(QSI);
                if constexpr (ks == 0) qk_mfma_first(acc_s[qs][s], a, qreg[qs][ks], magic);
                else qk_mfma_next(acc_s[qs][s], a, qreg[qs][ks]);
            });
        });
    };
    // O^T += V^T P~^T for the 16 keys of group (s, u) of the V tile in buffer vbuf, and their row sums
    auto pv_group = [&](int vbuf, auto S, auto U) {
        constexpr int s = IDX(S), u = IDX(U);
        const unsigned char* vb = lds + 2 * KB + vbuf * VB + (32 * s + 16 * u) * VROW;
        static_for<DT>([&](auto DTI) {
            constexpr int dt = IDX(DTI);
            v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb + v_off[dt]));
            v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb + v_off[dt] + 8 * VROW));
            const v8h a = __builtin_bit_cast(v8h, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            static_for<QS>([&](auto QSI) {
                constexpr int qs = IDX(QSI);
                pv_mfma(acc_o[qs][dt], a, __builtin_bit_cast(v8h, pk[qs][s][u]));
            });
        });
        static_for<QS>([&](auto QSI) {
            constexpr int qs = IDX(QSI);
            l_mfma(acc_l[qs], sel, pk[qs][s][u]);
        });
    };

    // ---- running-maximum bookkeeping for the tile whose scores sit in acc_s (tile j)
    // begin_tile: scale of the tile; on diagonal / tail tiles, hidden keys (beyond N, or after the
    // query when causal) get the bit pattern of -inf, which is below every real score as an
    // integer and exponentiates to 0.
    auto begin_tile = [&](int j) {
        const int kv0 = j * KTILE;
        score_tie();
        float dk = 1.0f;
        if constexpr (!KTOK) {
            dk = dk_next;                              // loaded one step ahead
            const int jn = j + 1 < kv_tiles_all ? j + 1 : j;
            dk_next = ksc_bh[(jn * KTILE) >> shift_k];
        }
        const bool need_mask = (kv0 + KTILE > N) || (CAUSAL && kv0 + KTILE - 1 > qrow0 + coff);
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            // a zero scale (all-zero quantization block) would turn -inf * scale into NaN
            sc[qs] = __builtin_fmaxf(dq[qs] * dk, 1e-30f);
            if constexpr (!KTOK) {
                // The exp2 argument is fma(seeded score, sc, bias) with bias = -(12582912 * sc + m):
                // it equals S^ * sc - m rounded ONCE only if that bias is exact.  The product is
                // exact once sc is cut to 22 significant bits (a relative change of 2^-22 in the
                // scale); the sum is exact when m is a multiple of the product's ulp, which
                // the check below detects and raise_maximum() establishes.
                sc[qs] = as_f32(as_i32(sc[qs]) & ~3);
            }
            // Everything the steady state needs from the running maximum is prepared here, ahead
            // of the matrix instructions of step_a, so that between the two parts of a step only
            // one compare and one branch stand (a chain of dependent VALU instructions there stalls
            // the in-order stream and, with it, the matrix pipe: measured 15 % of the kernel):
            //   bias      for the softmax FMA, valid as long as the maximum is not raised -- the same
            //             FMA applied to the own tile maximum tells whether it must be (must_raise());
            //   off_grid  whether the running maximum is off the grid on which this tile's bias is
            //             exact (then it is re-rounded in the rare path as well).
            if constexpr (KTOK) {
                bias[qs] = -m_run[qs];
                off_grid[qs] = false;
            } else {
                // 12582912 * sc is exact (22 bits), so both FMAs round their sum only: the first gives
                // the bias, the second what the bias really subtracts besides the seed
                const float sum = __builtin_fmaf(MAGIC_F, sc[qs], m_run[qs]);
                bias[qs] = -sum;
                off_grid[qs] = __builtin_fmaf(-MAGIC_F, sc[qs], sum) != m_run[qs];
            }
            if (need_mask) {
                const int q_row = qrow0 + 32 * qs + ql;
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                        bool hide = (key >= N) || (CAUSAL && key > q_row + coff);
                        acc_s[qs][s][r] = hide ? (int)0xFF800000 : acc_s[qs][s][r];
                    }
            }
        }
    };
    // partial_max(qs, p): integer maximum over part p (of DT) of sub-tile qs's 32 scores per lane;
    // issued between the matrix instructions of the step's first slot.
    auto partial_max = [&](auto QSI, auto P, int par) {
        constexpr int qs = IDX(QSI), p = IDX(P);
        constexpr int CNT = 32 / NA, FIRST = p * CNT;              // flat index = 16*s + r
        static_assert(CNT % 4 == 0, "whole groups of four registers per part");
        if constexpr (KTOK) {
            // registers 4*q4 .. +3 of sub-tile s are keys 32*s + 8*q4 + 4*g .. +3: one 16-byte
            // read each of a and b; the scores are replaced by t = S^ * delta_K[key]
            const float* kf = ksl + par * 2 * KTILE + 4 * g;
            float mf = p == 0 ? -__builtin_inff() : pmaxf[qs][0];       // the maximum is carried from part to part
#pragma unroll
            for (int f = FIRST; f < FIRST + CNT; f += 4) {
                const int s_ = f >> 4, r = f & 15;
                const v4f a = *(const v4f*)(kf + 32 * s_ + 2 * r), b = *(const v4f*)(kf + KTILE + 32 * s_ + 2 * r);
                float tv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    tv[e] = __builtin_fmaf(as_f32(acc_s[qs][s_][r + e]), a[e], b[e]);
                    acc_s[qs][s_][r + e] = as_i32(tv[e]);
                }
                mf = __builtin_fmaxf(__builtin_fmaxf(mf, tv[0]), tv[1]);
                mf = __builtin_fmaxf(__builtin_fmaxf(mf, tv[2]), tv[3]);
            }
            pmaxf[qs][0] = mf;
            return;
        }
        // the maximum is carried from part to part: CNT new values and the carry are CNT/2
        // three-way maxima (the first part, without a carry, ends on a two-way one)
        auto val = [&](int f) { return acc_s[qs][f >> 4][f & 15]; };
        if constexpr (p == 0) {
            int mi = val(FIRST);
#pragma unroll
            for (int f = FIRST + 1; f + 1 < FIRST + CNT; f += 2) mi = imax3(mi, val(f), val(f + 1));
            pmax[qs][0] = max(mi, val(FIRST + CNT - 1));
        } else {
            int mi = pmax[qs][0];
#pragma unroll
            for (int f = FIRST; f < FIRST + CNT; f += 2) mi = imax3(mi, val(f), val(f + 1));
            pmax[qs][0] = mi;
        }
    };
    // must_raise: does some row of the wavefront need a higher running maximum?  A lane looks at
    // the maximum over its own 32 keys only; the query's other 32 keys are with the lane 32 away,
    // which takes part in the same vote.
    auto must_raise = [&]() -> bool {
        bool want = false;
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            // the exp2 argument of the own maximum; on the first tile the bias is +inf and so is this
            const float top = __builtin_fmaf(KTOK ? pmaxf[qs][0] : as_f32(pmax[qs][0]), sc[qs], bias[qs]);
            want = want || off_grid[qs] || (top > MAX_SLACK);
        }
        return __builtin_amdgcn_ballot_w64(want) != 0ull;
    };
    // finish_max (rare path only): the row maximum of the tile in the exp2 domain.
    auto finish_max = [&]() {
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            // after the swap one result holds the own value and the other the partner's, in
            // either half of the wavefront
            if constexpr (KTOK) {
                const int mb = as_i32(pmaxf[qs][0]);
                auto r = __builtin_amdgcn_permlane32_swap(mb, mb, false, false);
                m_cand[qs] = __builtin_fmaxf(as_f32(r[0]), as_f32(r[1])) * sc[qs];     // -inf stays -inf: sc > 0
            } else {
                auto r = __builtin_amdgcn_permlane32_swap(pmax[qs][0], pmax[qs][0], false, false);
                const int mi = max((int)r[0], (int)r[1]);      // signed: the hidden pattern is negative
                // a row whose keys are all hidden holds the pattern of -inf, and stays -inf here
                m_cand[qs] = (as_f32(mi) - MAGIC_F) * sc[qs];
            }
        }
    };
    // The rare path: new running maximum; O^T, l and the P~ still waiting for its matrix
    // instructions are rescaled.
    auto raise_maximum = [&]() {
        finish_max();
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            refresh(acc_l[qs]);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) refresh(acc_o[qs][dt]);
        }
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            float m_new = __builtin_fmaxf(m_run[qs], m_cand[qs]);
            if constexpr (!KTOK)        // onto the grid on which the bias is exact
                m_new = __builtin_fmaf(-MAGIC_F, sc[qs], __builtin_fmaf(MAGIC_F, sc[qs], m_new));
            const float alpha = __builtin_amdgcn_exp2f(m_run[qs] - m_new);
            m_run[qs] = m_new;
            acc_l[qs] *= alpha;        // the register of the lane's own query is the one that counts
            pin_a(acc_l[qs]);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[qs][dt][r] *= alpha;
                pin_a(acc_o[qs][dt]);
            }
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
        }
    };
    auto set_bias = [&]() {
#pragma unroll
        for (int qs = 0; qs < QS; ++qs)       // exp2 argument = acc*sc + bias
            bias[qs] = KTOK ? -m_run[qs] : -__builtin_fmaf(MAGIC_F, sc[qs], m_run[qs]);
    };

    // ---- one pipeline step: softmax of tile j (scores in acc_s), P~V of tile j-1, K^Q^^T of tile
    // j+1.  For j = 0 the P~ registers are zero and the V buffer that is read is zero-filled, so
    // that P~V adds nothing.
    //
    // Flat operand sequence o = 0 .. 4*DT + 2*KS - 1: four P~V groups (DT operands each), then
    // the two K^Q^^T halves (KS operands each).  Operand o+PD is read from LDS before the matrix
    // instructions of operand o are issued.  The step comes in two parts:
    //   step_a  the first P~V group, with the row maximum of tile j computed between its matrix
    //           instructions (nothing of tile j's softmax can start before the maximum is known);
    //   step_b  everything else, with the softmax chunks between the matrix instructions.
    // Between the two the (rare) raise of the running maximum takes place.
    constexpr int NOPS = 4 * DT + 2 * KS;
    // LDS operands are read PD operands ahead of their matrix instructions.  The depth does not show
    // in the timing, but at D = 64 the four registers of a ring slot decide whether a third
    // wavefront fits on a SIMD (168 registers): worth 4-5 %, hence the shallower rings there.
    constexpr int PD = D == 64 ? (KTOK ? 1 : 2) : 3;
    v4i opnd[PD + 1];            // operand ring (V^T operands are reinterpreted)
    auto load_operand = [&](auto O, int vbuf, int kbuf) {
        constexpr int o = IDX(O);
        if constexpr (o < 4 * DT) {
            constexpr int grp_su = o / DT, dt = o % DT;         // group (s,u) = (grp_su / 2, grp_su % 2)
            const unsigned char* vb = lds + 2 * KB + vbuf * VB + 16 * grp_su * VROW + v_off[dt];
            v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb));
            v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(v4s, vb + 8 * VROW));
            opnd[o % (PD + 1)] = __builtin_bit_cast(v4i, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            constexpr int half = (o - 4 * DT) / KS, ks = (o - 4 * DT) % KS;
            opnd[o % (PD + 1)] = *(const v4i*)(lds + kbuf * KB + half * 32 * KROW + k_off[ks]);
        }
    };
    auto issue_mfma = [&](auto O, auto QSI) {
        constexpr int o = IDX(O), qs = IDX(QSI);
        if constexpr (o < 4 * DT) {
            constexpr int grp_su = o / DT, dt = o % DT;
            pv_mfma(acc_o[qs][dt], __builtin_bit_cast(v8h, opnd[o % (PD + 1)]), __builtin_bit_cast(v8h, pk[qs][grp_su >> 1][grp_su & 1]));
        } else {
            constexpr int half = (o - 4 * DT) / KS, ks = (o - 4 * DT) % KS;
            if constexpr (ks == 0) qk_mfma_first(acc_s[qs][half], opnd[o % (PD + 1)], qreg[qs][ks], magic);
            else qk_mfma_next(acc_s[qs][half], opnd[o % (PD + 1)], qreg[qs][ks]);
        }
    };
    auto row_sums = [&](auto G) {
        // row sums of a 16-key group just consumed: l += 1^T P~^T on the matrix pipe
        constexpr int grp_su = IDX(G);
        static_for<QS>([&](auto QSI) {
            constexpr int qs = IDX(QSI);
            l_mfma(acc_l[qs], sel, pk[qs][grp_su >> 1][grp_su & 1]);
        });
        __builtin_amdgcn_sched_barrier(0);
    };
    // The softmax of a tile is cut into chunks of two scores of one query sub-tile; chunk ch
    // belongs to 16-key group ch / (4*QS).  A chunk passes three stages in three consecutive
    // pipeline ticks (scale+bias FMA, exp2, pack) so that dependent instructions of one chunk are
    // never adjacent in the single in-order instruction stream.
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
        int packed = __builtin_bit_cast(int, __builtin_convertvector(pp, h2));
        // Pinned to this place in the instruction stream: otherwise the compiler is free to sink the
        // whole softmax of the step down to its first use in the next step (it does, once two steps
        // share a loop body), out of the shadow of this step's matrix instructions.
        if constexpr (D == 128) asm volatile("" : "+v"(packed));     // (only the unrolled loop needs it)
        pk[qs][grp_su >> 1][grp_su & 1][pair] = packed;
    };
    // Schedule of a step (QS = 1 in the formulas):
    //   step_a  the first SA P~V groups (NA matrix instructions); the row maximum of tile j is
    //           taken between them -- nothing of tile j's softmax can start before it is known;
    //   step_b  the other P~V groups and the first half of K^Q^^T (MB matrix instructions) carry
    //           the NCH softmax chunks, as evenly as they divide; the second half of K^Q^^T
    //           follows (it overwrites the half of S that the last chunks read) and takes the two
    //           ticks that drain the chunk pipeline.
    // Chunk c enters at tick c (fma), is exponentiated at tick c+1 and packed at tick c+2.
    static_assert(QS == 1 || SA == 1, "the generalized schedule is written for one query sub-tile");
    constexpr int MB = ((4 - SA) * DT + KS) * QS;
    constexpr int NB = (NOPS - NA) * QS;                // matrix instructions of step_b
    using Plan = TickPlan<NCH, MB>;
    static_assert(KS * QS >= 2, "two drain ticks need two matrix instructions after the last fma");
    // a P~ group is packed only after its P~V of tile j-1 has been issued ...
    static_assert(SA >= 2 || Plan::slot_of(CHUNKS * 1 + 2) >= (2 - SA) * DT * QS - 1, "group 1 packed after its matrix instructions");
    static_assert(SA >= 3 || Plan::slot_of(CHUNKS * 2 + 2) >= (3 - SA) * DT * QS - 1, "group 2 packed after its matrix instructions");
    static_assert(SA >= 4 || Plan::slot_of(CHUNKS * 3 + 2) >= (4 - SA) * DT * QS - 1, "group 3 packed after its matrix instructions");
    // ... and each half of S_j is consumed before the K^Q^^T of that half is issued
    static_assert(Plan::slot_of(NCH / 2 - 1) < (4 - SA) * DT * QS, "first half of S consumed before it is overwritten");
    static_assert(Plan::slot_of(NCH - 1) < MB, "second half of S consumed before it is overwritten");
    // par = j & 1, passed separately so that the unrolled main loop can give it as a constant: every
    // LDS address of the step is then a per-lane register plus an immediate.
    auto step_a = [&](int par) {
        const int vbuf = par ^ 1, kbuf = par ^ 1;       // V(j-1) and K^(j+1) sit in the other buffer
        static_for<PD>([&](auto O) { load_operand(O, vbuf, kbuf); });
        __builtin_amdgcn_sched_barrier(0);
        static_for<NA>([&](auto O) {
            constexpr int o = IDX(O);
            load_operand(std::integral_constant<int, o + PD>{}, vbuf, kbuf);
            static_for<QS>([&](auto QSI) {
                issue_mfma(O, QSI);
                partial_max(QSI, O, par);
                __builtin_amdgcn_sched_barrier(0);
            });
            if constexpr (o % DT == DT - 1) row_sums(std::integral_constant<int, o / DT>{});
        });
    };
    auto step_b = [&](int par) {
        const int vbuf = par ^ 1, kbuf = par ^ 1;
        static_for<NOPS - NA>([&](auto OO) {
            constexpr int o = IDX(OO) + NA;
            static_for<QS>([&](auto QSI) {
                constexpr int qs = IDX(QSI);
                issue_mfma(std::integral_constant<int, o>{}, QSI);
                if constexpr (qs == 0 && o + PD < NOPS) {
                    // the next operand read goes out in the shadow of the matrix instruction
                    load_operand(std::integral_constant<int, o + PD>{}, vbuf, kbuf);
                    __builtin_amdgcn_sched_barrier(0);
                }
                constexpr int i = (o - NA) * QS + qs;       // index of the matrix instruction in step_b
#pragma unroll
                for (int n = Plan::first(i); n < Plan::end(i); ++n) {
                    if (n - 2 >= 0 && n - 2 < NCH) chunk_pack(n - 2);
                    if (n - 1 >= 0 && n - 1 < NCH) chunk_exp(n - 1);
                    if (n >= 0 && n < NCH) chunk_fma(n);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            if constexpr (o < 4 * DT && o % DT == DT - 1) row_sums(std::integral_constant<int, o / DT>{});
        });
    };

    auto dump_tile = [&](int j) {
        const int kv0 = j * KTILE;
        score_fence();
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
            const int q_row = qrow0 + 32 * qs + ql;
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int key = kv0 + 32 * s + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (q_row < Nq && key < N) sdump[(slab_q + q_row) * (size_t)N + key] = acc_s[qs][s][r] - MAGIC_I;
                }
        }
    };

    // ---- prologue: K^(0), K^(1) into LDS; S_0.  Both V buffers start zero-filled: step 0 reads
    // buffer 1 before any tile has arrived (its P~ is zero, but 0 * NaN would not be), and rows of a
    // ragged last tile that lie beyond the slab must hold finite values whatever the load leaves there.
    if (!DUMP) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < VL; ++i)
                if (NTHREADS * i + wave * 64 < VVEC) *(v4i*)(lds + 2 * KB + b * VB + (t + NTHREADS * i) * 16) = (v4i){0, 0, 0, 0};
    }
    load_k(0, 0);
    if (T > 1) load_k(1, 1);
    request_key_scales(0);
    tiles_ready_barrier();
    qk_half(0, std::integral_constant<int, 0>{});
    qk_half(0, std::integral_constant<int, 1>{});

    // ---- main loop.  Time slot j lies between barriers j and j+1.  At barrier j the tiles
    // requested in slot j-1 have landed and the buffers of V(j-2) and K^(j) are free (their last
    // readers ran in slot j-1): V(j) and K^(j+2) are requested into them and have the whole slot
    // to arrive.  Slot j reads V(j-1) and K^(j+1).  Every wavefront passes T+1 barriers after the
    // prologue's.
    auto turn = [&](int j, int par) {
        __builtin_amdgcn_s_waitcnt(0x0F70);     // own loads landed: vmcnt(0), no wait on the other counters
        if (j < T) publish_key_scales(par);
        __syncthreads();
        if (j < T) load_v(j, par);
        if (j + 2 < T) load_k(j + 2, par);
        if (j + 1 < T) request_key_scales(j + 1);
    };
    int j = 0;
    if (DUMP) {
        for (; j < T; ++j) {
            turn(j, j & 1);
            dump_tile(j);
            qk_half((j + 1) & 1, std::integral_constant<int, 0>{});
            qk_half((j + 1) & 1, std::integral_constant<int, 1>{});
        }
        return;
    }
    // The inner loop holds nothing but the steady state: a tile whose maximum forces a rescale
    // leaves it, is finished on the slow path, and the inner loop is entered again.  (The empty
    // assembly statements carry a value around the loop that the compiler cannot see through; they
    // keep it from restructuring the loop nest, which made it spill registers.)
    unsigned opaque = 0;
    auto iteration = [&](int j, int par) {
        asm volatile("" : "+s"(opaque));
        turn(j, par);
        begin_tile(j);
        asm volatile("" : "+s"(opaque));
        step_a(par);
        if (must_raise()) {
            if constexpr (CLOCKS) ++n_raised;
            raise_maximum();
            set_bias();
        }
        asm volatile("" : "+s"(opaque));
        step_b(par);
        asm volatile("" : "+s"(opaque));
    };
    if constexpr (D == 128) {
        // two tiles per trip, so that the buffer parity is a compile-time constant inside the body
        // (12 address computations less per step; measured +2..4 % at D = 128, -3 % at D = 64)
        for (; j + 1 < Tw; j += 2) {
            iteration(j, 0);
            iteration(j + 1, 1);
        }
        if (j < Tw) {
            iteration(j, 0);
            ++j;
        }
    } else {
        for (; j < Tw; ++j) iteration(j, j & 1);
    }
    // The scores of tile Tw that the last step produced are never read: keep their registers
    // untouched until the matrix instructions have written them (the compiler would hand them out
    // as temporaries at once).
    score_fence();
    // the P~V of the wavefront's last tile ...
    turn(j, j & 1);
    {
        const int vbuf = (j - 1) & 1;
        static_for<4>([&](auto G) {
            pv_group(vbuf, std::integral_constant<int, (IDX(G) >> 1)>{}, std::integral_constant<int, (IDX(G) & 1)>{});
        });
    }
    // ... and the wavefront keeps feeding the workgroup's tile pipeline until all are done.
    for (++j; j <= T; ++j) turn(j, j & 1);

    // ---- O = diag(l)^-1 O, fp16 store
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
        const int q_row = qrow0 + 32 * qs + ql;
        refresh(acc_l[qs]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) refresh(acc_o[qs][dt]);
        const float l_row = (lane & 16) ? acc_l[qs][1] : acc_l[qs][0];       // the lane's own query, all keys
        const float inv = 1.0f / l_row;
        if (q_row < Nq) {
            if (lse != nullptr && g == 0) lse[slab_o + q_row] = m_run[qs] + __builtin_amdgcn_logf(l_row);
            _Float16* orow = og + (slab_o + q_row) * D;
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
    if constexpr (CLOCKS) {
        if (lane == 0) {
            unsigned long long* row = clocks + (((size_t)unit * tiles_q + (tiles_q - 1 - qt)) * NW + wave) * 4;
            row[0] = __builtin_readcyclecounter() - clock_t0;
            row[1] = wall_clock64() - clock_r0;
            row[2] = (unsigned long long)n_raised;
            row[3] = (unsigned long long)Tw;
        }
    }
}

// Causal launches: how many slabs (units) an XCD interleaves tile-major (0: none, slab-major as without a
// mask).  Only when every XCD's range is a whole number of units -- otherwise the ranges cut through slabs,
// which is what balances the XCDs then -- and only as many as keep their K^ and V (unit_bytes each) inside
// the XCD's 4 MB L2 together: interleaving more trades the shorter tail for re-fetches from HBM (measured at
// 16K keys, 6 MB per slab: 2.2 x the HBM traffic for 0-4 % of time, depending on the box; at 1.5K keys, where
// 16 slabs fit, +14 % and no extra traffic).
int tile_major_group(long total_tiles, int tiles_q, long unit_bytes) {
    if (total_tiles % (8l * tiles_q) != 0) return 0;
    const int units_per_xcd = (int)(total_tiles / 8 / tiles_q);
    const long fit = (4l << 20) / (unit_bytes > 0 ? unit_bytes : 1);
    int g = (int)(fit < units_per_xcd ? fit : units_per_xcd);
    while (g > 1 && units_per_xcd % g != 0) --g;
    return g > 1 ? g : 0;
}

template <int D, int NW>
static hipError_t launch_dn(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                            const void* v, void* o, int32_t* sdump, int BH, int Nq, int N, int causal,
                            int block_q, int block_k, const SplitPlan& sp, hipStream_t st,
                            unsigned long long* clocks = nullptr) {
    constexpr int QTILE = NW * WROWS, NTHREADS = NW * 64;
    const int tiles_q = (Nq + QTILE - 1) / QTILE;
    const long total = (long)BH * sp.n_splits * tiles_q;
    const int per_xcd = (int)((total + 7) / 8);
    dim3 grid((unsigned)(per_xcd * 8));
    const int shift_q = __builtin_ctz((unsigned)block_q), shift_k = __builtin_ctz((unsigned)block_k);
    const _Float16* vp = (const _Float16*)v;
    _Float16* op = (_Float16*)o;
    const bool ktok = block_k == 1;
    const int tm_group = causal && !sdump ? tile_major_group(total, tiles_q, (long)(sp.n_splits > 1 ? sp.chunk : N) * 3 * D) : 0;
#define SAGE_ARGS qq, qscale, kq, kscale, vp, op, sdump, sp.lse, clocks, Nq, N, shift_q, shift_k, tiles_q, per_xcd, total, BH, sp.n_splits, sp.chunk, tm_group
#define SAGE_LAUNCH(C, DMP, KT) sage_attn_kernel<D, NW, C, DMP, KT><<<grid, NTHREADS, 0, st>>>(SAGE_ARGS)
    if (clocks != nullptr) {
        // the measurement build exists for the headline shape only: D = 128, 256-row workgroups, block scales
        if constexpr (D == 128 && NW == 8) {
            if (sdump || ktok) return hipErrorInvalidValue;
            if (causal) sage_attn_kernel<D, NW, true, false, false, true><<<grid, NTHREADS, 0, st>>>(SAGE_ARGS);
            else sage_attn_kernel<D, NW, false, false, false, true><<<grid, NTHREADS, 0, st>>>(SAGE_ARGS);
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    // per-token key scales need a few more registers than 4-wavefront workgroups at D = 128 have
    // (two workgroups per CU: 128 + 128 registers); launch_d() never asks for that combination
    constexpr bool KTOK_OK = !(D == 128 && NW == 4);
    if (sdump) SAGE_LAUNCH(false, true, false);
    else if (ktok) {
        if constexpr (KTOK_OK) {
            if (causal) SAGE_LAUNCH(true, false, true);
            else SAGE_LAUNCH(false, false, true);
        } else {
            return hipErrorInvalidValue;
        }
    }
    else if (causal) SAGE_LAUNCH(true, false, false);
    else SAGE_LAUNCH(false, false, false);
#undef SAGE_LAUNCH
#undef SAGE_ARGS
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                           const void* v, void* o, int32_t* sdump, int BH, int Nq, int N, int causal,
                           int block_q, int block_k, const SplitPlan& sp, hipStream_t st, int wg_rows = 0,
                           unsigned long long* clocks = nullptr) {
    // 256-row workgroups (8 wavefronts sharing one set of LDS tiles) for long sequences at D = 128;
    // 128-row workgroups, two or three per CU, for D = 64, whenever the larger tile would leave CUs
    // without work (fewer than two workgroups per CU), and for short sequences, where a workgroup
    // visits few tiles and the finer causal staircase and the independent progress of the small
    // workgroups matter more than the sharing (measured at D = 128: +30 % at N = 1K causal, +11 %
    // non-causal; +19 % / +2 % at 2K; +4 % / -3 % at 4K).
    const long big_tiles = (long)BH * sp.n_splits * ((Nq + 8 * WROWS - 1) / (8 * WROWS));
    const int n_seen = sp.n_splits > 1 ? sp.chunk : N;           // keys a workgroup walks
    const bool short_seq = n_seen <= 2048 || (causal && n_seen <= 4096);
    bool small = QS == 1 && (D == 64 || ((big_tiles < 2 * 256 || short_seq) && block_k != 1 && !sdump));
    // the score dump may name the workgroup shape, so that a test reaches every instantiation
    if (sdump && wg_rows != 0) small = wg_rows == 4 * WROWS;
    if (clocks != nullptr) small = false;       // the measurement build has the 256-row shape only
    if (small) return launch_dn<D, 4>(qq, qscale, kq, kscale, v, o, sdump, BH, Nq, N, causal, block_q, block_k, sp, st);
    return launch_dn<D, 8>(qq, qscale, kq, kscale, v, o, sdump, BH, Nq, N, causal, block_q, block_k, sp, st, clocks);
}

hipError_t launch_attn(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                       const void* v, void* o, int32_t* sdump, int BH, int Nq, int N, int D, int causal,
                       int block_q, int block_k, hipStream_t st, int wg_rows) {
    const SplitPlan whole = {1, 0, nullptr};
    if (D == 64) return launch_d<64>(qq, qscale, kq, kscale, v, o, sdump, BH, Nq, N, causal, block_q, block_k, whole, st, wg_rows);
    return launch_d<128>(qq, qscale, kq, kscale, v, o, sdump, BH, Nq, N, causal, block_q, block_k, whole, st, wg_rows);
}

hipError_t launch_attn_clocks(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                              const void* v, void* o, unsigned long long* clocks, int BH, int N, int causal,
                              int block_q, int block_k, hipStream_t st) {
    const SplitPlan whole = {1, 0, nullptr};
    return launch_d<128>(qq, qscale, kq, kscale, v, o, nullptr, BH, N, N, causal, block_q, block_k, whole, st, 0, clocks);
}

// ---- split over the keys ------------------------------------------------------------------------
// With few query rows per slab a launch has too few workgroups for the chip and each walks every
// key tile.  The keys are cut into n_splits chunks, a workgroup per (slab, chunk, query tile) leaves
// the attention of its rows over its chunk -- O_s normalized by the chunk's own denominator, fp16,
// and lse_s = m_s + log2 l_s -- and the merge below forms
//     O = sum_s w_s O_s / sum_s w_s,   w_s = 2^(lse_s - max_s lse_s),
// which is the attention over all keys: w_s is the chunk's share of the softmax denominator.
SplitPlan plan_split(int BH, int Nq, int N, int causal, int requested) {
    if (requested <= 0) {
        // One 128-row workgroup per CU (measured: 256 to 512 workgroups are the fastest at every
        // shape tried; the launch is memory-bound from there on, and more chunks only add partial
        // results to write and merge); chunks of at least 8 key tiles.
        const long wg = (long)BH * ((Nq + 127) / 128);
        long want = (256 + wg - 1) / wg;
        const long most = N / 512 < 64 ? N / 512 : 64;
        requested = (int)(want < most ? want : most);
    }
    if (requested <= 1) return {1, 0, nullptr};
    // Every chunk but the last has `chunk` keys, a multiple of the 64-key tile and of the largest K
    // block (128); the last takes the rest.  It starts at or before key N - Nq when causal (N - 1
    // otherwise), so that every row sees at least one key of every chunk and no partial result is
    // empty (the merge relies on it: every lse is finite).
    // A chunk is at least one group of 128 keys, so a request beyond the number of groups is the same
    // plan as that number (and 128 * requested then cannot leave the int range: N <= 2^23).
    const int groups = (N + 127) / 128;
    if (requested > groups) requested = groups;
    if (requested <= 1) return {1, 0, nullptr};
    const int chunk = 128 * ((N + 128 * requested - 1) / (128 * requested));
    const int limit = causal ? N - Nq : N - 1;
    const int fit = limit / chunk + 1;
    const int n = requested < fit ? requested : fit;
    if (n <= 1) return {1, 0, nullptr};
    return {n, chunk, nullptr};
}

template <int D>
__global__ void __launch_bounds__(256) merge_splits_kernel(const _Float16* __restrict__ part, const float* __restrict__ lse,
                                                           _Float16* __restrict__ og, long rows, int n_splits) {
    constexpr int TPR = D / 8;                         // threads per row, 8 channels each
    const long row = (long)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    const int c8 = threadIdx.x % TPR;
    if (row >= rows) return;
    float top = -__builtin_inff();
    for (int s = 0; s < n_splits; ++s) top = __builtin_fmaxf(top, lse[(size_t)s * rows + row]);
    float acc[8], wsum = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    for (int s = 0; s < n_splits; ++s) {
        const float w = __builtin_amdgcn_exp2f(lse[(size_t)s * rows + row] - top);
        const v8h x = *(const v8h*)(part + ((size_t)s * rows + row) * D + c8 * 8);
        wsum += w;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(w, (float)x[e], acc[e]);
    }
    const float inv = 1.0f / wsum;
    v8h y;
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = (_Float16)(acc[e] * inv);
    *(v8h*)(og + (size_t)row * D + c8 * 8) = y;
}

hipError_t launch_merge_splits(const void* part, const float* lse, void* o, long rows, int D, int n_splits, hipStream_t st) {
    const _Float16* pp = (const _Float16*)part;
    _Float16* op = (_Float16*)o;
    if (D == 64) merge_splits_kernel<64><<<(unsigned)((rows + 31) / 32), 256, 0, st>>>(pp, lse, op, rows, n_splits);
    else merge_splits_kernel<128><<<(unsigned)((rows + 15) / 16), 256, 0, st>>>(pp, lse, op, rows, n_splits);
    return hipGetLastError();
}

hipError_t launch_attn_split(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                             const void* v, void* o, void* workspace, int BH, int Nq, int N, int D, int causal,
                             int block_q, int block_k, int requested, hipStream_t st) {
    SplitPlan sp = plan_split(BH, Nq, N, causal, requested);
    if (sp.n_splits == 1) return launch_attn(qq, qscale, kq, kscale, v, o, nullptr, BH, Nq, N, D, causal, block_q, block_k, st);
    const long rows = (long)BH * Nq;
    // workspace: partial O [n_splits, BH, Nq, D] fp16, then lse [n_splits, BH, Nq] fp32
    _Float16* part = (_Float16*)workspace;
    sp.lse = (float*)((char*)workspace + (size_t)sp.n_splits * rows * D * sizeof(_Float16));
    hipError_t e = D == 64
        ? launch_d<64>(qq, qscale, kq, kscale, v, part, nullptr, BH, Nq, N, causal, block_q, block_k, sp, st)
        : launch_d<128>(qq, qscale, kq, kscale, v, part, nullptr, BH, Nq, N, causal, block_q, block_k, sp, st);
    if (e != hipSuccess) return e;
    return launch_merge_splits(part, sp.lse, o, rows, D, sp.n_splits, st);
}

}  // namespace sage
