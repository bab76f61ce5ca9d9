/*
 * libsage -- SageAttention forward pass (SAGEAttn-B, -T, -vB and -vT) for AMD gfx950, C ABI.
 *
 * The three calls are the three stages of Algorithm 1 of the SageAttention paper:
 *   sage_smooth_quant_k : "Preprocessing" K = K - mean(K) (Section 4.2) followed by the per-block
 *                         INT8 quantizer psi_K (Section 3.2);
 *   sage_quant_q        : psi_Q(Q / sqrt(d)) -- the softmax scale is folded into Q before
 *                         quantizing (Section 4.6, "Fusion Tricks");
 *   sage_attn_fwd       : the tiled loop of Algorithm 1: S = Q^ K^^T * dQ * dK, online softmax
 *                         (Section 3.1), O += P~.to(FP16) V (Section 4.4), O = diag(l)^-1 O.
 * A block size of 1 selects Section 3.2's per-token quantizer (one scale per token) instead of the
 * per-block one; block_q = block_k = 1 in all three calls is the SAGEAttn-T kernel of Section 4.5's
 * table of kernels.  The two sides are independent: any block_q goes with any block_k.
 * sage_quant_v and sage_attn_pv_int8_fwd are the same loop with Section 4.3's INT8 second product
 * (the -vB / -vT kernels of that table); sage_rope_* fuse RoPE into the two pre-pass calls.
 * The *_cross_fwd calls take different numbers of queries and keys, and the *_cross_split_fwd calls
 * cut the keys into chunks that run as separate workgroups (few queries against many keys); neither
 * is in the paper, which states everything for equal lengths.
 *
 * Conventions shared by every call
 *   - All pointers are DEVICE pointers (HIP global memory) unless stated; the library never
 *     allocates, frees or synchronizes.  Work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL is the default stream) and the call returns immediately.
 *   - Tensors are contiguous row-major [B, H, N, D] with D innermost; fp16 is IEEE binary16.
 *     Scales are fp32 [B, H, ceil(N/block)], the K mean is fp32 [B, H, D].
 *   - The caller owns every buffer.  Outputs are fully overwritten, inputs are never written.
 *   - Tensor pointers must be 16-byte aligned, scale/mean pointers 4-byte aligned.
 *   - Inputs must be finite.  N is any positive value up to 2^23 (it need not be a multiple of a
 *     block size: the last block is short).  D is 64 or 128.  B * H (the number of (batch, head)
 *     slabs) is at most 65535; more is SAGE_ERR_SHAPE.
 *   - Return value: SAGE_OK or an error code below.  Arguments are validated on the host before
 *     anything is launched, so a failing call has no device side effects.  Nothing throws or aborts.
 *
 * Arithmetic (fixed so that an independent implementation can reproduce the INT8 tensors, the
 * scales, the mean and the int32 scores bit for bit):
 *   mean[c]  = fp32( (exact sum over the N tokens of K[t,c]) / N ), the division done in fp64;
 *   Ks       = fp32(K) - mean                         (fp32, not re-rounded to fp16);
 *   Qs       = fp32(Q) * sm_scale                     (fp32);
 *   per block of `block` consecutive tokens (all D channels; block = 1: per token): amax = max |X|,
 *   delta    = amax / 127   (fp32 division),  r = amax > 0 ? 127 / amax : 0  (fp32 division),
 *   X^       = clamp(round_half_even(X * r), -127, 127);  an all-zero block has delta = 0, X^ = 0.
 *   S^       = Q^ K^^T in int32, exact.
 * The softmax/output stage is specified up to floating-point tolerance only.
 */
#ifndef SAGE_H_
#define SAGE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SAGE_OK = 0,
    SAGE_ERR_NULL = 1,        /* a required pointer is NULL                                    */
    SAGE_ERR_SHAPE = 2,       /* B, H, N or D <= 0, N > 2^23, B*H > 65535, or B*H*N*D overflows */
    SAGE_ERR_UNSUPPORTED = 3, /* D not in {64,128} or a block size the kernels do not cover    */
    SAGE_ERR_WORKSPACE = 4,   /* workspace_bytes smaller than the call's *_workspace() size   */
    SAGE_ERR_ALIGN = 5,       /* a pointer is not aligned as required                          */
    SAGE_ERR_LAUNCH = 6,      /* the HIP runtime reported an error at launch                   */
    SAGE_ERR_VALUE = 7,       /* sm_scale not finite or not positive                           */
    SAGE_ERR_SCRATCH = 8      /* sage_smooth_quant_k_noalloc: shape beyond the static scratch  */
};

/* Human-readable name of a status code (host pointer to a static string; never NULL). */
const char* sage_status_string(int status);

/*
 * Build identity: the SHA-256 (64 hex digits, host pointer to a static string) of the source files
 * the library was compiled from, so that a caller can refuse a binary that does not belong to the
 * sources beside it.  "unknown" if the build did not provide it.
 */
const char* sage_source_hash(void);

/*
 * The softmax scale of Section 4.6 when the caller has none of its own: 1 / sqrt(D), the fp32
 * division of 1 by the fp32 square root (0 for D <= 0).  Host-only helper; nothing is launched.
 */
float sage_default_sm_scale(int D);

/*
 * psi_Q(Q * sm_scale): Section 3.2 (per-block quantizer), Section 4.6 (scale folded into Q),
 * Algorithm 1 "Quantization".
 *   q_f16   in  [B,H,N,D] fp16
 *   q_i8    out [B,H,N,D] int8, values in [-127,127]
 *   q_scale out [B,H,ceil(N/block_q)] fp32 (delta_Q)
 *   sm_scale    the softmax scale, normally 1/sqrt(D); finite and > 0
 *   block_q     tokens per scale: 1 (per-token quantizer), 32, 64 or 128
 */
int sage_quant_q(const void* q_f16, int8_t* q_i8, float* q_scale,
                 int B, int H, int N, int D, float sm_scale, int block_q, void* stream);

/*
 * Bytes of device scratch sage_smooth_quant_k needs for this shape: the exact column sums of K over
 * chunks of tokens, at most 64 per (batch, head) slab, as 64-bit integers ([B*H, chunks, D]).
 * 0 for sequences short enough to be handled in one launch (and for arguments the call rejects).
 */
size_t sage_smooth_quant_k_workspace(int B, int H, int N, int D);

/*
 * phi_K = psi_K o gamma: Section 4.2 (gamma(K) = K - mean(K), mean over all N tokens of one
 * (batch, head), also when the attention is causal), then Section 3.2's per-block quantizer.
 *   k_f16   in  [B,H,N,D] fp16
 *   k_i8    out [B,H,N,D] int8
 *   k_scale out [B,H,ceil(N/block_k)] fp32 (delta_K)
 *   k_mean  out [B,H,D] fp32, or NULL if the caller does not want the mean
 *   workspace   device scratch of at least sage_smooth_quant_k_workspace() bytes, 8-byte aligned;
 *               contents on entry are ignored, contents on return are unspecified.  Two calls
 *               that share a workspace must be ordered on the same stream.  May be NULL when that
 *               size is 0.
 *   block_k     tokens per scale: 1 (per-token quantizer), 32, 64 or 128
 */
int sage_smooth_quant_k(const void* k_f16, int8_t* k_i8, float* k_scale, float* k_mean,
                        void* workspace, size_t workspace_bytes,
                        int B, int H, int N, int D, int block_k, void* stream);

/*
 * sage_quant_q and sage_smooth_quant_k of one (Q, K) pair in one launch less (Sections 3.2, 4.2, 4.6;
 * Algorithm 1 "Quantization"): the quantization of Q depends on nothing the K side computes, so it
 * shares a launch with the K side's first half (the column sums); for key sequences short enough for
 * the single-launch K pre-pass, with all of it.  Two launches instead of three, one instead of two --
 * which is most of the pre-pass's time for short sequences.  Results are those of the two separate
 * calls, bit for bit.
 *   q_f16 [B,H,Nq,D], k_f16 [B,H,Nkv,D]: the two lengths may differ (cross attention, decode)
 *   q_i8, q_scale   as in sage_quant_q (for Nq);  k_i8, k_scale, k_mean as in sage_smooth_quant_k (for Nkv)
 *   workspace       at least sage_smooth_quant_k_workspace(B, H, Nkv, D) bytes, as in sage_smooth_quant_k
 * Arguments, limits and error codes as in the two separate calls; nothing is launched when a check fails.
 */
int sage_quant_qk(const void* q_f16, const void* k_f16, int8_t* q_i8, float* q_scale,
                  int8_t* k_i8, float* k_scale, float* k_mean, void* workspace, size_t workspace_bytes,
                  int B, int H, int Nq, int Nkv, int D, float sm_scale, int block_q, int block_k, void* stream);

/*
 * sage_smooth_quant_k for callers that cannot allocate device memory or carry a workspace around:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels, same results bit for bit; the partial column sums go to a buffer that is part of the
 * library's device image (SAGE_NOALLOC_SCRATCH_BYTES = 4 MiB, held by every GPU the
 * library runs on until the process ends) instead of a caller-supplied workspace.  The call allocates
 * and frees nothing.
 *   - Shapes whose sage_smooth_quant_k_workspace() exceeds the limit are refused with
 *     SAGE_ERR_SCRATCH before anything is launched (the limit covers B*H*chunks*D <= 524288, e.g.
 *     every configuration with B*H <= 64 at D = 128).
 *   - All calls on one GPU share that GPU's buffer: calls that may overlap in time (different
 *     streams, or threads) race on it and must be ordered by the caller.  Nothing needs clearing
 *     between calls: every word that is read was written by the same call.
 *   - The first call on a device looks up the buffer's address (hipGetSymbolAddress, once per
 *     device, under a lock); SAGE_ERR_LAUNCH if that fails.
 * All other arguments, limits and error codes as sage_smooth_quant_k.
 */
#define SAGE_NOALLOC_SCRATCH_BYTES (4u << 20)
int sage_smooth_quant_k_noalloc(const void* k_f16, int8_t* k_i8, float* k_scale, float* k_mean,
                                int B, int H, int N, int D, int block_k, void* stream);

/*
 * The two pre-pass calls with the rotary position embedding applied on the fly -- Section 4.6
 * ("Fusion Tricks"): the quantizer is fused into the operator that produces Q and K, so that the
 * rotated fp16 tensors are never written to or re-read from memory.  The paper names RoPE without
 * defining it; this is the rotate-half form: channel c < D/2 is paired with channel c + D/2,
 *     y[t,c] = x[t,c] cos[t,c] - x[t,c+D/2] sin[t,c],   y[t,c+D/2] = x[t,c+D/2] cos[t,c] + x[t,c] sin[t,c],
 * products and sum rounded to fp32, y rounded to fp16 (round to nearest even) -- exactly the
 * tensor a separate RoPE kernel would store -- and then everything as in sage_quant_q /
 * sage_smooth_quant_k on y (the K mean is the mean of the rotated K).  The results are therefore
 * bit-identical to the unfused sequence.
 *   rope_cos, rope_sin  in  [N, D/2] fp32, row t = position of token t, shared by all (batch,
 *                       head) slabs; 16-byte aligned; required
 * All other arguments, limits and error codes as in the unfused calls.
 */
int sage_rope_quant_q(const void* q_f16, const float* rope_cos, const float* rope_sin,
                      int8_t* q_i8, float* q_scale,
                      int B, int H, int N, int D, float sm_scale, int block_q, void* stream);
int sage_rope_smooth_quant_k(const void* k_f16, const float* rope_cos, const float* rope_sin,
                             int8_t* k_i8, float* k_scale, float* k_mean,
                             void* workspace, size_t workspace_bytes,
                             int B, int H, int N, int D, int block_k, void* stream);

/*
 * The loop of Algorithm 1 (with Section 3.1's online softmax and Section 4.4's FP16 P~ V, here
 * accumulated in fp32 because gfx950's FP16 matrix instructions accumulate in fp32).
 *   q_i8, q_scale   from sage_quant_q (same block_q)
 *   k_i8, k_scale   from sage_smooth_quant_k (same block_k)
 *   v_f16   in  [B,H,N,D] fp16
 *   o_f16   out [B,H,N,D] fp16
 *   causal      0: every key is visible; non-zero: key j is visible to query t iff j <= t
 *   sm_scale    the value that was given to sage_quant_q; it is already inside q_i8/q_scale and is
 *               NOT applied again here -- it is only validated (finite, > 0)
 *   block_q     1, 32, 64 or 128;  block_k  1, 64 or 128 -- the values the scales were made with.
 *               With block_k = 1 every score is dequantized with its own key's scale before the
 *               row maximum is taken (a few percent slower); block_q = 1 costs nothing.
 */
int sage_attn_fwd(const int8_t* q_i8, const float* q_scale,
                  const int8_t* k_i8, const float* k_scale,
                  const void* v_f16, void* o_f16,
                  int B, int H, int N, int D, int causal, float sm_scale,
                  int block_q, int block_k, void* stream);

/*
 * psi_V of Section 4.3 for the kernels with an INT8 second product (SAGEAttn-vB / -vT, Section 4.5):
 * the per-channel quantizer of Section 3.2, one scale per channel of every (batch, head) slab, taken
 * over all N tokens; delta_V[c] = amax_c / 127, V^[t,c] = clamp(rne(V[t,c] * (127 / amax_c)), -127, 127);
 * an all-zero channel gives delta_V = 0, V^ = 0.
 *   v_f16    in  [B,H,N,D] fp16
 *   v_i8t    out [B,H,D,Np] int8: V^ TRANSPOSED, channel-major, Np = sage_quant_v_pitch(N) =
 *            64 * ceil(N / 64) tokens per channel row; tokens N .. Np-1 are written as 0
 *   v_scale  out [B,H,D] fp32
 *   workspace   device, >= sage_quant_v_workspace(B,H,N,D) bytes, 4-byte aligned; scratch, contents
 *               undefined on entry and exit
 * Same ownership, stream and error conventions as the calls above.
 */
size_t sage_quant_v_workspace(int B, int H, int N, int D);
int sage_quant_v_pitch(int N);
int sage_quant_v(const void* v_f16, int8_t* v_i8t, float* v_scale,
                 void* workspace, size_t workspace_bytes,
                 int B, int H, int N, int D, void* stream);

/*
 * The loop of Algorithm 1 with the second product of Section 4.3: P~ is quantized per block with
 * the static scale 1/127 (its row maxima are 1), P^ V^ is an INT8 product with an int32 result,
 * dequantized with 1/127 and delta_V[c].  m, l and the rescaling are those of Algorithm 1 (l sums the
 * unrounded P~).  block_q / block_k as in sage_attn_fwd: block sizes give SAGEAttn-vB, 1 gives -vT.
 * The block of P~ that is quantized together is the loop's block of 64 keys (the paper's kernel
 * setting), whatever the granularity of the K scales: a code is relative to the running maximum
 * after its own 64-key block.
 *   q_i8, q_scale, k_i8, k_scale   as for sage_attn_fwd
 *   v_i8t, v_scale                 from sage_quant_v (same N)
 *   o_f16   out [B,H,N,D] fp16
 * The codes of P~ depend on the last bits of the exponential, so two correct implementations can
 * differ by one code in a few elements; one code of one key is worth at most delta_V[c] / l in the
 * output (l = the row's softmax denominator relative to its maximum, >= 1).
 */
int sage_attn_pv_int8_fwd(const int8_t* q_i8, const float* q_scale,
                          const int8_t* k_i8, const float* k_scale,
                          const int8_t* v_i8t, const float* v_scale, void* o_f16,
                          int B, int H, int N, int D, int causal, float sm_scale,
                          int block_q, int block_k, void* stream);

/*
 * sage_attn_fwd with Nq queries against Nkv keys and values (cross-attention, or the last Nq tokens
 * of a sequence attending to all of it).  The paper states Algorithm 1 for Nq = Nkv; nothing but
 * the ranges changes.
 *   q_i8 [B,H,Nq,D], q_scale [B,H,ceil(Nq/block_q)]     from sage_quant_q with N = Nq
 *   k_i8 [B,H,Nkv,D], k_scale [B,H,ceil(Nkv/block_k)]   from sage_smooth_quant_k with N = Nkv
 *   v_f16 [B,H,Nkv,D], o_f16 out [B,H,Nq,D]
 *   causal   non-zero: query t is the token at position t + Nkv - Nq and sees keys j <= t + Nkv - Nq
 *            (mask aligned at the end); needs Nq <= Nkv, else SAGE_ERR_UNSUPPORTED
 * Everything else as sage_attn_fwd, which is this call with Nq = Nkv.
 */
int sage_attn_cross_fwd(const int8_t* q_i8, const float* q_scale,
                        const int8_t* k_i8, const float* k_scale,
                        const void* v_f16, void* o_f16,
                        int B, int H, int Nq, int Nkv, int D, int causal, float sm_scale,
                        int block_q, int block_k, void* stream);

/*
 * sage_attn_cross_fwd for few queries against many keys (decoding, the tail of a chunked prefill):
 * the keys of a slab are cut into n_splits chunks that run as separate workgroups, each leaving the
 * attention of its rows over its chunk and the chunk's share of the softmax denominator, and a
 * merge kernel combines them.  The result is that of Algorithm 1 over all keys up to the order
 * of the floating-point sums (the partial outputs pass through fp16); the paper has no such split.
 *   n_splits   requested number of chunks, 0 = chosen from the shape; the number actually used is
 *              sage_attn_split_count() (chunks are multiples of 128 keys, and with a causal mask the
 *              last chunk starts at or before key Nkv - Nq); 1 chunk is sage_attn_cross_fwd itself
 *   workspace  device, >= sage_attn_split_workspace() bytes (same arguments), 16-byte aligned;
 *              scratch, contents undefined on entry and exit; may be NULL when that size is 0
 * sage_attn_split_count returns 0 for arguments the call would reject.
 * Everything else as sage_attn_cross_fwd; SAGE_ERR_VALUE for n_splits < 0, SAGE_ERR_SHAPE if B * H * chunks
 * exceeds 2^30.
 */
int sage_attn_split_count(int B, int H, int Nq, int Nkv, int causal, int n_splits);
size_t sage_attn_split_workspace(int B, int H, int Nq, int Nkv, int D, int causal, int n_splits);
int sage_attn_cross_split_fwd(const int8_t* q_i8, const float* q_scale,
                              const int8_t* k_i8, const float* k_scale,
                              const void* v_f16, void* o_f16, void* workspace, size_t workspace_bytes,
                              int B, int H, int Nq, int Nkv, int D, int causal, float sm_scale,
                              int block_q, int block_k, int n_splits, void* stream);

/*
 * sage_attn_pv_int8_fwd with Nq queries against Nkv keys and values: the lengths, the layouts of
 * q_i8 / q_scale / o_f16 (Nq) and of k_i8 / k_scale / v_i8t / v_scale (Nkv; v_i8t from sage_quant_v
 * with N = Nkv) and the end-aligned causal mask are those of sage_attn_cross_fwd.
 */
int sage_attn_pv_int8_cross_fwd(const int8_t* q_i8, const float* q_scale,
                                const int8_t* k_i8, const float* k_scale,
                                const int8_t* v_i8t, const float* v_scale, void* o_f16,
                                int B, int H, int Nq, int Nkv, int D, int causal, float sm_scale,
                                int block_q, int block_k, void* stream);

/*
 * sage_attn_pv_int8_cross_fwd for few queries against many keys, with the keys cut into chunks as in
 * sage_attn_cross_split_fwd (same chunk plan: sage_attn_split_count; same workspace size:
 * sage_attn_split_workspace).  Every chunk runs the loop of Algorithm 1 with the second product of
 * Section 4.3 as if it were the whole key set, so a code of P~ is relative to the running maximum
 * WITHIN ITS CHUNK, not over all keys before it: the same attention as the unsplit call, but not the
 * same rounding of P~ (never coarser: a chunk's maximum is at most the running maximum over all keys).
 * One chunk is sage_attn_pv_int8_cross_fwd itself.
 */
int sage_attn_pv_int8_cross_split_fwd(const int8_t* q_i8, const float* q_scale,
                                      const int8_t* k_i8, const float* k_scale,
                                      const int8_t* v_i8t, const float* v_scale, void* o_f16,
                                      void* workspace, size_t workspace_bytes,
                                      int B, int H, int Nq, int Nkv, int D, int causal, float sm_scale,
                                      int block_q, int block_k, int n_splits, void* stream);

/*
 * Test hook: the raw int32 scores S^ = Q^ K^^T (Algorithm 1, the Matmul inside the S update)
 * produced by the same matrix-instruction code path as sage_attn_fwd, without mask.
 *   s_i32   out [B,H,N,N] int32 -- O(N^2) memory: meant for small N or for sub-problems.
 *   block_q, block_k   as in sage_attn_fwd (validated the same way; the scores themselves do not
 *                      depend on them: no scale is applied)
 *   wg_rows   query rows per workgroup: 128 (4 wavefronts) or 256 (8 wavefronts) -- the two shapes
 *             the attention kernel is built in; 0 leaves the choice to the launcher as sage_attn_fwd
 *             does.  Other values: SAGE_ERR_UNSUPPORTED.
 */
int sage_attn_qk_i32_debug(const int8_t* q_i8, const int8_t* k_i8, int32_t* s_i32,
                           int B, int H, int N, int D, int block_q, int block_k, int wg_rows, void* stream);

/*
 * Measurement hook: sage_attn_fwd's kernel at D = 128 in its 256-row workgroup shape (Algorithm 1; the
 * speed figures of Section 5 are quoted against the matrix unit's peak, which presumes a clock the
 * chip does not hold under this load), built with two counters read at the start and the end of every
 * wavefront.  Same arguments and the same output o_f16 as sage_attn_fwd (sm_scale is folded into
 * q_scale there and is no argument here), and in addition
 *   clocks  out [B*H * ceil(N/256) * 8][4] uint64, one row per wavefront, row index
 *           ((slab * ceil(N/256) + (ceil(N/256) - 1 - query tile)) * 8 + wavefront):
 *           [0] shader-clock ticks of the wavefront, [1] ticks of the constant 100 MHz counter over the
 *           same span ([0] / [1] * 0.1 = the clock in GHz the chip held), [2] how often the wavefront
 *           raised a running maximum (the rare path of the online softmax), [3] key tiles it visited.
 *           The caller zeroes it; device memory, 8-byte aligned.
 *   D must be 128 and block_k 64 or 128 (one scale per key block): otherwise SAGE_ERR_UNSUPPORTED.
 * The 256-row shape is used whatever the problem size (sage_attn_fwd picks 128-row workgroups for
 * short sequences and small launches).  Other errors as in sage_attn_fwd.
 */
int sage_attn_clock_debug(const int8_t* q_i8, const float* q_scale, const int8_t* k_i8, const float* k_scale,
                          const void* v_f16, void* o_f16, uint64_t* clocks,
                          int B, int H, int N, int D, int causal, int block_q, int block_k, void* stream);

/*
 * Measurement hook: instruction-stream probes of the matrix pipe, for the roofline the attention
 * kernels are quoted against (Section 5, "Kernel Speed", compares the kernel with the peak of the
 * GPU's INT8 matrix unit; this gives the rate gfx950 sustains with the same instructions).  One
 * launch of `workgroups` workgroups of 4 * waves_per_simd wavefronts; every wavefront repeats a fixed
 * group of instructions `iters` times:
 *   kind 0  8 INT8 32x32x32 matrix instructions        (8 * 65536 operations per group)
 *   kind 1  8 FP16 32x32x16 matrix instructions        (8 * 32768)
 *   kind 2  8 INT8 + 16 FP16: the matrix work of one 32-query x 64-key step of Algorithm 1 at D = 128
 *   kind 3  24 softmax chunks (2 fma, 2 exp2, 1 FP16 pack each), no matrix instruction
 *   kind 4  8 x (one FP16 matrix instruction + one chunk) in one instruction stream
 *   kind 5  wavefronts 0-3 of a workgroup run kind 1's group, wavefronts 4-7 (the same SIMDs) 8 chunks;
 *           needs waves_per_simd = 2
 *   kind 6  kind 2's instructions with 16 chunks and 8 three-way maxima spread between them
 *   kind 7  24 LDS reads of 16 bytes per lane (1 KB per wavefront each): the kernel's K^ operand reads
 *   kind 8  48 transposing LDS reads of 8 bytes per lane: the kernel's V^T operand reads (24 KB per group)
 *   kind 9  kind 6 with the A operand of every matrix instruction read from LDS three instructions
 *           ahead of its use, as the attention kernel reads them
 *   kind 10 16 of the 4x4x4 FP16 matrix instructions the kernel takes its row sums with
 *   kind 11 4 x (4 FP16 32x32x16 + 2 of the 4x4x4): the P~V part of a step with its row sums
 *   kind 12 4 x (4 FP16 32x32x16 + 1 FP16 16x16x32);  kind 13  4 x 5 FP16 32x32x16 (other ways to the row sums)
 *   kind 14 kind 0 with all 8 instructions accumulating into one register block (a dependent chain)
 *   kind 15 the step in the attention kernel's own order at D = 128: 16 FP16 instructions with a 16x16x32
 *           row-sum instruction after every fourth, then 8 INT8 ones, every operand read from LDS three
 *           ahead; 16 three-way maxima behind the first 4 instructions, the 16 chunks behind instructions
 *           4 .. 19 (the last 8 overwrite the scores the chunks read)
 *   kind 16 kind 15 with the chunks spread over instructions 4 .. 23 instead (what a second set of score
 *           registers would allow)
 *   kind 17 16 FP16 16x16x32 matrix instructions (kind 1's operations in the shape with a quarter of the result
 *           block and twice the contraction depth);  kind 18  16 INT8 16x16x64 instructions (kind 0's operations)
 *   kind 19 kind 15 built from the 16x16 instructions: every operand read from LDS feeds two of them (two
 *           16-query blocks), 32 FP16 + 16 INT8 + 4 row-sum instructions per step
 *   kind 20 kind 19 for a wavefront of 64 queries: every operand feeds four 16x16 instructions, twice the
 *           softmax work, the same LDS reads (twice kind 15's operations per group)
 *   data    in  1024 int32 of arbitrary (random) bits: the operands; 16-byte aligned
 *   out     out 4 uint64 per wavefront ([workgroups * 4 * waves_per_simd][4]): shader-clock ticks of the
 *           loop, constant-rate-counter ticks of the loop, a checksum, 0
 * Errors as everywhere; SAGE_ERR_UNSUPPORTED for an unknown kind (0 .. 20 exist) or waves_per_simd not in {1, 2}.
 */
int sage_microbench(int kind, int waves_per_simd, int workgroups, int iters,
                    const int32_t* data, uint64_t* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SAGE_H_ */
