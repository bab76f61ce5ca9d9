// Internal launch interface between the C-ABI entry points and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sage {

// Pre-pass (HBM-bound).  All return the hipError_t of the launch.  cs / sn: RoPE tables [N, D/2]
// applied to the input rows on the fly, or both null for none.
hipError_t launch_quant_q(const void* q, int8_t* qq, float* qscale, int BH, int N, int D,
                          float sm_scale, int block, const float* cs, const float* sn, hipStream_t st);
// parts: scratch for the partial column sums, plan_colsum(BH, N).parts * BH * D 64-bit words
// (sequences short enough for the single-launch kernel use none: parts = 0).
struct ColsumPlan {
    int parts;      // partial sums per (batch, head) slab
    int chunk;      // tokens per partial sum
};
ColsumPlan plan_colsum(int BH, int N);
hipError_t launch_smooth_quant_k(const void* k, int8_t* kq, float* kscale, float* kmean,
                                 long long* parts, int BH, int N, int D, int block,
                                 const float* cs, const float* sn, hipStream_t st);
// Both pre-passes of a (Q, K) pair in one launch less: the K side's first half (or, for short key
// sequences, all of it) shares a launch with the Q quantizer.  No RoPE.  parts as above (for Nkv).
hipError_t launch_quant_qk(const void* q, const void* k, int8_t* qq, float* qscale, int8_t* kq, float* kscale,
                           float* kmean, long long* parts, int BH, int Nq, int Nkv, int D, float sm_scale,
                           int block_q, int block_k, hipStream_t st);

// Fused attention (MFMA-bound): Nq query rows against N keys per slab.  sdump != nullptr selects the
// int32 score dump; for the dump, wg_rows (128 or 256) names the workgroup shape instead of leaving
// it to the launcher (0).
hipError_t launch_attn(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                       const void* v, void* o, int32_t* sdump, int BH, int Nq, int N, int D, int causal,
                       int block_q, int block_k, hipStream_t st, int wg_rows = 0);
// Measurement build of the same kernel (D = 128, 256-row workgroups, one scale per key block): also
// writes, per wavefront, [shader-clock ticks, 100 MHz ticks, raises of the running maximum, key tiles
// visited] to clocks[(workgroup * 8 + wavefront) * 4 ..], workgroup = slab * ceil(N / 256) + query tile
// counted from the last.
hipError_t launch_attn_clocks(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                              const void* v, void* o, unsigned long long* clocks, int BH, int N, int causal,
                              int block_q, int block_k, hipStream_t st);

// The same with the keys of a slab cut into chunks (for few query rows): partial results per chunk in
// `workspace` (n_splits * BH * Nq * (2 D + 4) bytes), then a merge into o.  plan_split() resolves the
// requested number of chunks (0 = choose) into the one used and the chunk length; lse is filled in
// by the launcher.
struct SplitPlan {
    int n_splits;
    int chunk;
    float* lse;
};
// slabs an XCD interleaves tile-major in a causal launch (0: none); see sage_attn.hip
int tile_major_group(long total_tiles, int tiles_q, long unit_bytes);
SplitPlan plan_split(int BH, int Nq, int N, int causal, int requested);
hipError_t launch_attn_split(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                             const void* v, void* o, void* workspace, int BH, int Nq, int N, int D, int causal,
                             int block_q, int block_k, int requested, hipStream_t st);

hipError_t launch_merge_splits(const void* part, const float* lse, void* o, long rows, int D, int n_splits, hipStream_t st);
hipError_t launch_attn_pv8_split(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                                 const int8_t* vt, const float* vscale, void* o, void* workspace, int BH, int Nq, int N,
                                 int D, int causal, int block_q, int block_k, int requested, hipStream_t st);

// INT8 second product (Section 4.3): per-channel quantizer of V (transposed output, pitch
// 64 * ceil(N / 64)) and the attention kernel that consumes it.
hipError_t launch_quant_v(const void* v, int8_t* vt, float* vscale, unsigned* amax_bits,
                          int BH, int N, int D, hipStream_t st);
hipError_t launch_attn_pv8(const int8_t* qq, const float* qscale, const int8_t* kq, const float* kscale,
                           const int8_t* vt, const float* vscale, void* o, int BH, int Nq, int N, int D, int causal,
                           int block_q, int block_k, hipStream_t st);

// Instruction-stream probes (sage_microbench.hip): kind 0..6, 1 or 2 wavefronts per SIMD, `out` takes
// four 64-bit words per wavefront.
hipError_t launch_microbench(int kind, int waves_per_simd, int workgroups, int iters, const int* data,
                             unsigned long long* out, hipStream_t st);

}  // namespace sage
