/*
 * SageAttention forward pass -- CPU oracle (TEST INFRASTRUCTURE, not the product).
 *
 * Plain, slow, readable C that follows the paper's definitions step by step:
 *   Section 3.1 (attention, FlashAttention-2 online softmax), Section 3.2 (dynamic
 *   quantizers), Section 4.1 (quantized-attention formulation), Section 4.2 (smoothing K),
 *   Section 4.3 (INT8 P~ and V, the -vB / -vT kernels), Section 4.4 (FP16 P~V), Section 4.6 (1/sqrt(d) folded into Q before quantizing) and
 *   Algorithm 1 (SAGEAttn-B).
 *
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may call this file.
 * It shares no code with the HIP path.  OpenMP (if enabled) only spreads independent
 * (batch, head, Q-block) units over host cores; the arithmetic of each unit is unchanged.
 *
 * Arithmetic contract (the paper leaves these open; the readings taken are):
 *   - fp32 means IEEE binary32, round-to-nearest-even, one rounding per written operation,
 *     no FMA contraction (compile with -ffp-contract=off), denormals kept.
 *   - mean(K) is the exactly-summed column total (integer arithmetic in units of 2^-24),
 *     divided by N in double, rounded once to fp32.
 *   - K - mean(K) is formed in fp32 and is NOT rounded back to fp16.
 *   - Quantizer: delta = fl32(amax/127); X^ = clamp(rne(fl32(x * fl32(127/amax))), -127, 127);
 *     an all-zero block gives delta = 0 and X^ = 0.
 *   - Rounding to INT8 and to FP16 is round-half-to-even (switchable to truncation for P~).
 *
 * Levels:
 *   L0  exact fp64 softmax(Q K^T sm_scale [+ causal mask]) V on the fp16 input values.
 *   L1  quantized S = dQ dK (Q^ K^^T), then exact fp64 two-pass softmax and fp64 P V.
 *   L2  Algorithm 1 as written: block loop, fp32 online softmax, P~ -> fp16, fp32 (or
 *       emulated fp16) accumulation, final division, fp16 output; and the same loop with the
 *       INT8 second product of Section 4.3 (codes of P~ with the static scale 1/127, V per channel).
 *
 * Status of pins: every function here is pinned by tests/test_oracle_*.py against closed
 * forms, brute force, invariants and a hand-worked example (tests/golden/).  The output
 * tolerance used for GPU parity (2e-3 abs, cosine 0.9999) is a project target and is not
 * given by the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define SAGE_ORACLE_P_TRUNCATE 1u   /* P~ -> fp16 by truncation instead of nearest-even      */
#define SAGE_ORACLE_ACC_FP16   2u   /* emulate an fp16 accumulator for P~V (Algorithm 1)      */
#define SAGE_ORACLE_QUANT_DIV  4u   /* quantize with x / delta instead of x * fl32(127/amax)  */
#define SAGE_ORACLE_L_FROM_P16 8u   /* row sum l from the fp16-rounded P~ (not Algorithm 1)   */

/* ------------------------------------------------------------------ fp16 <-> fp32 */

static float f16_to_f32(uint16_t h) {
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    int e = (h >> 10) & 31;
    uint32_t m = h & 1023u;
    float mag;
    if (e == 0) mag = ldexpf((float)m, -24);                 /* zero / subnormal */
    else if (e == 31) mag = m ? NAN : INFINITY;
    else mag = ldexpf((float)(1024u + m), e - 25);
    uint32_t bits; memcpy(&bits, &mag, 4); bits |= sign;
    float out; memcpy(&out, &bits, 4);
    return out;
}

/* fp32 -> fp16; truncate = 0: round half to even, 1: toward zero.  Finite inputs. */
static uint16_t f32_to_f16(float x, int truncate) {
    uint16_t sign = (uint16_t)(signbit(x) ? 0x8000u : 0u);
    double a = fabs((double)x);
    if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
    if (a == 0.0) return sign;
    int e; (void)frexp(a, &e);                /* a = f * 2^e, f in [0.5, 1) */
    int exp_unb = e - 1;                      /* a = 1.xxx * 2^exp_unb */
    if (exp_unb < -14) exp_unb = -14;         /* subnormal range shares the 2^-24 step */
    double step = ldexp(1.0, exp_unb - 10);
    double q = a / step;                      /* exact: division by a power of two */
    double r = truncate ? floor(q) : nearbyint(q);   /* default rounding mode: ties to even */
    double v = r * step;
    if (v >= 65520.0) return (uint16_t)(sign | (truncate ? 0x7bffu : 0x7c00u));
    if (isinf(x)) return (uint16_t)(sign | 0x7c00u);
    if (v == 0.0) return sign;
    int e2; (void)frexp(v, &e2);
    int eu = e2 - 1;
    if (eu < -14) return (uint16_t)(sign | (uint16_t)(v / ldexp(1.0, -24)));
    uint32_t mant = (uint32_t)(v / ldexp(1.0, eu - 10)) - 1024u;
    return (uint16_t)(sign | (uint16_t)((eu + 15) << 10) | (uint16_t)mant);
}

void sage_oracle_f16_to_f32(const uint16_t* h, float* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = f16_to_f32(h[i]);
}
void sage_oracle_f32_to_f16(const float* x, uint16_t* out, int64_t n, int truncate) {
    for (int64_t i = 0; i < n; ++i) out[i] = f32_to_f16(x[i], truncate);
}

/* ------------------------------------------------------------------ Section 4.2: mean(K) */

/* An fp16 value as an exact integer count of 2^-24 (finite inputs). */
static int64_t f16_as_units(uint16_t h) {
    int e = (h >> 10) & 31;
    int64_t m = h & 1023;
    int64_t mag = (e == 0) ? m : ((1024 + m) << (e - 1));
    return (h & 0x8000u) ? -mag : mag;
}

/* mean(K)[c] = (1/N) sum_t K[t,c] for one (batch, head) slab K[N,D].
 * The sum is exact; one division and one rounding to fp32 follow.  N <= 2^23. */
void sage_oracle_k_mean(const uint16_t* k, int N, int D, float* mean) {
    for (int c = 0; c < D; ++c) {
        int64_t total = 0;
        for (int t = 0; t < N; ++t) total += f16_as_units(k[(int64_t)t * D + c]);
        double avg_units = (double)total / (double)N;
        mean[c] = (float)(avg_units * 0x1p-24);
    }
}

/* gamma(K) = K - mean(K), in fp32 (Section 4.2, Algorithm 1 preprocessing). */
void sage_oracle_smooth_k(const uint16_t* k, const float* mean, int N, int D, float* ks) {
    for (int t = 0; t < N; ++t)
        for (int c = 0; c < D; ++c) {
            volatile float d = f16_to_f32(k[(int64_t)t * D + c]) - mean[c];
            ks[(int64_t)t * D + c] = d;
        }
}

/* Q * sm_scale in fp32 (Section 4.6: the 1/sqrt(d) factor is applied before quantizing). */
void sage_oracle_scale_q(const uint16_t* q, float sm_scale, int N, int D, float* qs) {
    for (int64_t i = 0; i < (int64_t)N * D; ++i) {
        volatile float p = f16_to_f32(q[i]) * sm_scale;
        qs[i] = p;
    }
}

/* ------------------------------------------------------------------ Section 4.6: RoPE ahead of the quantizer */

/* Rotary position embedding of one slab x[N,D] (fp16), the operator Section 4.6 fuses the
 * quantizer into.  The paper only names it; the form taken here is the "rotate-half" one of the
 * Llama-family models it evaluates: channel c < D/2 is paired with channel c + D/2,
 *     y[t,c]       = x[t,c] cos[t,c] - x[t,c+D/2] sin[t,c]
 *     y[t,c+D/2]   = x[t,c+D/2] cos[t,c] + x[t,c] sin[t,c]
 * with the tables cos, sin [N, D/2] (fp32) given by the caller.  Each product and the sum are
 * rounded to fp32, and y is rounded to fp16: it is the tensor the unfused model hands to the
 * attention layer, so quantizing it "before it is written" gives what the unfused path gives. */
void sage_oracle_rope(const uint16_t* x, const float* cs, const float* sn, int N, int D, uint16_t* y) {
    int half = D / 2;
    for (int t = 0; t < N; ++t)
        for (int c = 0; c < half; ++c) {
            float a = f16_to_f32(x[(int64_t)t * D + c]), b = f16_to_f32(x[(int64_t)t * D + c + half]);
            float co = cs[(int64_t)t * half + c], si = sn[(int64_t)t * half + c];
            volatile float ac = a * co, bs = b * si, bc = b * co, as = a * si;
            volatile float lo = ac - bs, hi = bc + as;
            y[(int64_t)t * D + c] = f32_to_f16(lo, 0);
            y[(int64_t)t * D + c + half] = f32_to_f16(hi, 0);
        }
}

/* ------------------------------------------------------------------ Section 3.2: per-block quantizer psi */

/* x[N,D] fp32 -> xq[N,D] int8 and delta[ceil(N/block)]: one scale for every `block`
 * consecutive tokens (all D channels); the last block may be short. */
void sage_oracle_quant_per_block(const float* x, int N, int D, int block, unsigned flags,
                                 int8_t* xq, float* delta) {
    int nblk = (N + block - 1) / block;
    for (int g = 0; g < nblk; ++g) {
        int t0 = g * block, t1 = t0 + block < N ? t0 + block : N;
        float amax = 0.0f;
        for (int t = t0; t < t1; ++t)
            for (int c = 0; c < D; ++c) {
                float a = fabsf(x[(int64_t)t * D + c]);
                if (a > amax) amax = a;
            }
        volatile float d = amax / 127.0f;
        volatile float r = amax > 0.0f ? 127.0f / amax : 0.0f;
        delta[g] = d;
        for (int t = t0; t < t1; ++t)
            for (int c = 0; c < D; ++c) {
                float v = x[(int64_t)t * D + c];
                volatile float scaled;
                if (flags & SAGE_ORACLE_QUANT_DIV) scaled = (d > 0.0f) ? v / d : 0.0f;
                else scaled = v * r;
                float rounded = nearbyintf(scaled);          /* ties to even */
                if (rounded > 127.0f) rounded = 127.0f;
                if (rounded < -127.0f) rounded = -127.0f;
                xq[(int64_t)t * D + c] = (int8_t)rounded;
            }
    }
}

/* Pre-pass for one slab: phi_K = psi_K o gamma (Section 4.2). */
void sage_oracle_smooth_quant_k_slab(const uint16_t* k, int N, int D, int block_k, unsigned flags,
                                     int8_t* kq, float* k_scale, float* k_mean) {
    float* ks = (float*)malloc((size_t)N * D * sizeof(float));
    sage_oracle_k_mean(k, N, D, k_mean);
    sage_oracle_smooth_k(k, k_mean, N, D, ks);
    sage_oracle_quant_per_block(ks, N, D, block_k, flags, kq, k_scale);
    free(ks);
}

/* Pre-pass for one slab: psi_Q(Q * sm_scale). */
void sage_oracle_quant_q_slab(const uint16_t* q, int N, int D, float sm_scale, int block_q,
                              unsigned flags, int8_t* qq, float* q_scale) {
    float* qs = (float*)malloc((size_t)N * D * sizeof(float));
    sage_oracle_scale_q(q, sm_scale, N, D, qs);
    sage_oracle_quant_per_block(qs, N, D, block_q, flags, qq, q_scale);
    free(qs);
}

/* Whole tensors [B,H,N,D]; slabs are independent. */
void sage_oracle_smooth_quant_k(const uint16_t* k, int B, int H, int N, int D, int block_k,
                                unsigned flags, int8_t* kq, float* k_scale, float* k_mean) {
    int nblk = (N + block_k - 1) / block_k;
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < B * H; ++s)
        sage_oracle_smooth_quant_k_slab(k + (int64_t)s * N * D, N, D, block_k, flags,
                                        kq + (int64_t)s * N * D, k_scale + (int64_t)s * nblk,
                                        k_mean + (int64_t)s * D);
}
void sage_oracle_quant_q(const uint16_t* q, int B, int H, int N, int D, float sm_scale, int block_q,
                         unsigned flags, int8_t* qq, float* q_scale) {
    int nblk = (N + block_q - 1) / block_q;
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < B * H; ++s)
        sage_oracle_quant_q_slab(q + (int64_t)s * N * D, N, D, sm_scale, block_q, flags,
                                 qq + (int64_t)s * N * D, q_scale + (int64_t)s * nblk);
}

/* ------------------------------------------------------------------ Algorithm 1: S^ = Q^ K^^T */

/* Raw integer scores for query rows [row0, row0+nrows) of one slab against all N keys. */
void sage_oracle_qk_i32(const int8_t* qq, const int8_t* kq, int N, int D, int row0, int nrows,
                        int32_t* s /* [nrows, N] */) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < nrows; ++i)
        for (int j = 0; j < N; ++j) {
            int32_t acc = 0;
            for (int c = 0; c < D; ++c)
                acc += (int32_t)qq[(int64_t)(row0 + i) * D + c] * (int32_t)kq[(int64_t)j * D + c];
            s[(int64_t)i * N + j] = acc;
        }
}

/* ------------------------------------------------------------------ L2: Algorithm 1, one Q block */

/* Q block `i` (rows i*bq .. min(N,(i+1)*bq)-1) of one slab; writes those rows of o (fp16 bits, [N,D]).
 * Causal reading: key j is visible to query t iff j <= t; kv blocks entirely above the diagonal
 * are not visited.
 * gq / gk = tokens per scale of Q^ / K^: equal to bq / bkv for Algorithm 1 (one scale per block of
 * the loop), 1 for the per-token quantizer of Section 3.2 (SAGEAttn-T): query t is dequantized
 * with q_scale[t / gq], key j with k_scale[j / gk].
 * Nq queries against N keys: the paper treats Nq = N only (Section 3.1); with Nq != N nothing in
 * Algorithm 1 changes except the ranges, and the causal mask is aligned at the end (query t is the
 * token at position t + N - Nq, as when the last Nq tokens of a sequence attend to all of it). */
static void l2_q_block(const int8_t* qq, const float* q_scale, const int8_t* kq, const float* k_scale,
                       const uint16_t* v, int Nq, int N, int D, int causal, int bq, int bkv, int gq, int gk,
                       unsigned flags, int i, uint16_t* o) {
    int r0 = i * bq, r1 = r0 + bq < Nq ? r0 + bq : Nq, nr = r1 - r0;
    int Tn = (N + bkv - 1) / bkv;
    int shift = N - Nq;          /* causal with Nq != N: query t sits at position t + (N - Nq) among the keys */
    float* m = (float*)malloc(sizeof(float) * nr);
    float* l = (float*)malloc(sizeof(float) * nr);
    float* O = (float*)calloc((size_t)nr * D, sizeof(float));
    float* S = (float*)malloc(sizeof(float) * (size_t)nr * bkv);
    float* Pt = (float*)malloc(sizeof(float) * (size_t)bkv);
    for (int a = 0; a < nr; ++a) { m[a] = -INFINITY; l[a] = 0.0f; }

    for (int j = 0; j < Tn; ++j) {
        int c0 = j * bkv, c1 = c0 + bkv < N ? c0 + bkv : N, nc = c1 - c0;
        if (causal && c0 > r1 - 1 + shift) break;
        /* S = Matmul(Q^_i, K^_j^T) * dQ[i] * dK[j], then the mask */
        for (int a = 0; a < nr; ++a)
            for (int b = 0; b < nc; ++b) {
                int32_t acc = 0;
                for (int c = 0; c < D; ++c)
                    acc += (int32_t)qq[(int64_t)(r0 + a) * D + c] * (int32_t)kq[(int64_t)(c0 + b) * D + c];
                volatile float t1 = (float)acc * q_scale[(r0 + a) / gq];
                volatile float t2 = t1 * k_scale[(c0 + b) / gk];
                S[a * bkv + b] = (causal && (c0 + b) > (r0 + a + shift)) ? -INFINITY : t2;
            }
        /* online softmax and O update, row by row */
        for (int a = 0; a < nr; ++a) {
            float m_old = m[a], m_new = m_old;
            for (int b = 0; b < nc; ++b) if (S[a * bkv + b] > m_new) m_new = S[a * bkv + b];
            float alpha = (m_old == -INFINITY) ? 0.0f : expf(m_old - m_new);
            float rowsum = 0.0f;
            for (int b = 0; b < nc; ++b) {
                float p = (S[a * bkv + b] == -INFINITY) ? 0.0f : expf(S[a * bkv + b] - m_new);
                float p16 = f16_to_f32(f32_to_f16(p, (flags & SAGE_ORACLE_P_TRUNCATE) ? 1 : 0));
                Pt[b] = p16;
                volatile float acc = rowsum + ((flags & SAGE_ORACLE_L_FROM_P16) ? p16 : p);
                rowsum = acc;
            }
            volatile float lnew = alpha * l[a];
            lnew = lnew + rowsum;
            l[a] = lnew;
            m[a] = m_new;
            for (int c = 0; c < D; ++c) {
                volatile float oc = alpha * O[(int64_t)a * D + c];
                if (flags & SAGE_ORACLE_ACC_FP16) {
                    /* fp16 accumulator: the running value is re-rounded to fp16 after every
                     * 16-key slice of the product (one matrix-instruction step). */
                    float acc = f16_to_f32(f32_to_f16(oc, 0));
                    for (int b0 = 0; b0 < nc; b0 += 16) {
                        float part = 0.0f;
                        for (int b = b0; b < nc && b < b0 + 16; ++b) {
                            volatile float pv = Pt[b] * f16_to_f32(v[(int64_t)(c0 + b) * D + c]);
                            volatile float s2 = part + pv; part = s2;
                        }
                        volatile float s3 = acc + part;
                        acc = f16_to_f32(f32_to_f16(s3, 0));
                    }
                    O[(int64_t)a * D + c] = acc;
                } else {
                    float acc = oc;
                    for (int b = 0; b < nc; ++b) {
                        volatile float pv = Pt[b] * f16_to_f32(v[(int64_t)(c0 + b) * D + c]);
                        volatile float s2 = acc + pv; acc = s2;
                    }
                    O[(int64_t)a * D + c] = acc;
                }
            }
        }
    }
    /* O_i = diag(l)^-1 O_i, written as fp16 */
    for (int a = 0; a < nr; ++a)
        for (int c = 0; c < D; ++c) {
            volatile float q = O[(int64_t)a * D + c] / l[a];
            o[(int64_t)(r0 + a) * D + c] = f32_to_f16(q, 0);
        }
    free(m); free(l); free(O); free(S); free(Pt);
}

/* L2 on one slab for a list of Q blocks (nblocks < 0: all of them). Rows of other blocks in
 * `o` are left untouched.  gran_q / gran_k: tokens per scale (see l2_q_block). */
void sage_oracle_attn_l2_slab_g(const int8_t* qq, const float* q_scale, const int8_t* kq,
                                const float* k_scale, const uint16_t* v, int N, int D, int causal,
                                int block_q, int block_k, int gran_q, int gran_k, unsigned flags,
                                const int* blocks, int nblocks, uint16_t* o) {
    int Tm = (N + block_q - 1) / block_q;
    int n = nblocks < 0 ? Tm : nblocks;
#pragma omp parallel for schedule(dynamic)
    for (int u = 0; u < n; ++u) {
        int i = nblocks < 0 ? u : blocks[u];
        l2_q_block(qq, q_scale, kq, k_scale, v, N, N, D, causal, block_q, block_k, gran_q, gran_k, flags, i, o);
    }
}
/* Algorithm 1 proper: one scale per block of the loop. */
void sage_oracle_attn_l2_slab(const int8_t* qq, const float* q_scale, const int8_t* kq,
                              const float* k_scale, const uint16_t* v, int N, int D, int causal,
                              int block_q, int block_k, unsigned flags,
                              const int* blocks, int nblocks, uint16_t* o) {
    sage_oracle_attn_l2_slab_g(qq, q_scale, kq, k_scale, v, N, D, causal, block_q, block_k,
                               block_q, block_k, flags, blocks, nblocks, o);
}

/* L2 on whole tensors [B,H,N,D]; scales [B,H,ceil(N/gran)]. */
void sage_oracle_attn_l2_g(const int8_t* qq, const float* q_scale, const int8_t* kq, const float* k_scale,
                           const uint16_t* v, int B, int H, int N, int D, int causal,
                           int block_q, int block_k, int gran_q, int gran_k, unsigned flags, uint16_t* o) {
    int Tm = (N + block_q - 1) / block_q;
    int nsq = (N + gran_q - 1) / gran_q, nsk = (N + gran_k - 1) / gran_k;
    int64_t units = (int64_t)B * H * Tm;
#pragma omp parallel for schedule(dynamic)
    for (int64_t u = 0; u < units; ++u) {
        int64_t s = u / Tm; int i = (int)(u % Tm);
        l2_q_block(qq + s * N * D, q_scale + s * nsq, kq + s * N * D, k_scale + s * nsk,
                   v + s * N * D, N, N, D, causal, block_q, block_k, gran_q, gran_k, flags, i,
                   o + s * N * D);
    }
}
void sage_oracle_attn_l2(const int8_t* qq, const float* q_scale, const int8_t* kq, const float* k_scale,
                         const uint16_t* v, int B, int H, int N, int D, int causal,
                         int block_q, int block_k, unsigned flags, uint16_t* o) {
    sage_oracle_attn_l2_g(qq, q_scale, kq, k_scale, v, B, H, N, D, causal, block_q, block_k,
                          block_q, block_k, flags, o);
}

/* Algorithm 1 with Nq queries against Nk keys on whole tensors: Q^ [B,H,Nq,D], K^ and V [B,H,Nk,D],
 * scales [B,H,ceil(Nq/gran_q)] and [B,H,ceil(Nk/gran_k)], output [B,H,Nq,D].  Causal needs Nq <= Nk. */
void sage_oracle_attn_l2_cross_g(const int8_t* qq, const float* q_scale, const int8_t* kq, const float* k_scale,
                                 const uint16_t* v, int B, int H, int Nq, int Nk, int D, int causal,
                                 int block_q, int block_k, int gran_q, int gran_k, unsigned flags, uint16_t* o) {
    int Tm = (Nq + block_q - 1) / block_q;
    int nsq = (Nq + gran_q - 1) / gran_q, nsk = (Nk + gran_k - 1) / gran_k;
    int64_t units = (int64_t)B * H * Tm;
#pragma omp parallel for schedule(dynamic)
    for (int64_t u = 0; u < units; ++u) {
        int64_t s = u / Tm; int i = (int)(u % Tm);
        l2_q_block(qq + s * Nq * D, q_scale + s * nsq, kq + s * Nk * D, k_scale + s * nsk,
                   v + s * Nk * D, Nq, Nk, D, causal, block_q, block_k, gran_q, gran_k, flags, i,
                   o + s * Nq * D);
    }
}

/* ------------------------------------------------------------------ Section 4.3: INT8 P~ and V (SAGEAttn-vB / -vT) */

/* psi_V, the per-channel quantizer of Section 3.2 applied to V (Section 4.3): one scale per channel
 * c of one (batch, head) slab v[N,D], taken over ALL N tokens (also when the mask is causal: the
 * scale belongs to the tensor, not to a query).  Same arithmetic as the per-block quantizer:
 * delta[c] = fl32(amax_c / 127), V^[t,c] = clamp(rne(fl32(v[t,c] * fl32(127 / amax_c)))), an
 * all-zero channel gives delta = 0 and V^ = 0.  vq is token-major [N,D] like v. */
void sage_oracle_quant_v_slab(const uint16_t* v, int N, int D, int8_t* vq, float* v_scale) {
    for (int c = 0; c < D; ++c) {
        float amax = 0.0f;
        for (int t = 0; t < N; ++t) {
            float a = fabsf(f16_to_f32(v[(int64_t)t * D + c]));
            if (a > amax) amax = a;
        }
        volatile float d = amax / 127.0f;
        volatile float r = amax > 0.0f ? 127.0f / amax : 0.0f;
        v_scale[c] = d;
        for (int t = 0; t < N; ++t) {
            volatile float scaled = f16_to_f32(v[(int64_t)t * D + c]) * r;
            float rounded = nearbyintf(scaled);              /* ties to even */
            if (rounded > 127.0f) rounded = 127.0f;
            if (rounded < -127.0f) rounded = -127.0f;
            vq[(int64_t)t * D + c] = (int8_t)rounded;
        }
    }
}
void sage_oracle_quant_v(const uint16_t* v, int B, int H, int N, int D, int8_t* vq, float* v_scale) {
#pragma omp parallel for schedule(dynamic)
    for (int s = 0; s < B * H; ++s)
        sage_oracle_quant_v_slab(v + (int64_t)s * N * D, N, D, vq + (int64_t)s * N * D, v_scale + (int64_t)s * D);
}

/* One Q block of the kernels with an INT8 second product (Section 4.3, the -vB / -vT rows of the
 * kernel table in Section 4.5).  Algorithm 1 with its P~V line replaced:
 *   P^ = rne(fl32(P~ * 127))            psi_P: per-block with the static scale 1/127 (row maxima of
 *                                       P~ are <= 1 because the running maximum is subtracted)
 *   A  = P^ V^_j                        exact int32
 *   O  = alpha * O + fl32(fl32((float)A * (1/127)) * delta_V[c])
 * m, l and alpha are those of Algorithm 1: l sums the fp32 P~, not the codes.
 * lsum (may be NULL) receives the final l of every row of the block (rows i*bq ...), which bounds
 * what one code of P^ is worth in the output: delta_V[c] * |V^| / (127 l) * 127 <= delta_V[c] / l. */
static void l2_pv8_q_block(const int8_t* qq, const float* q_scale, const int8_t* kq, const float* k_scale,
                           const int8_t* vq, const float* v_scale, int Nq, int N, int D, int causal,
                           int bq, int bkv, int gq, int gk, int i, uint16_t* o, float* lsum, float* mrow) {
    int r0 = i * bq, r1 = r0 + bq < Nq ? r0 + bq : Nq, nr = r1 - r0;
    int Tn = (N + bkv - 1) / bkv;
    int shift = N - Nq;          /* Nq queries against N keys: end-aligned causal mask, as in l2_q_block */
    float* m = (float*)malloc(sizeof(float) * nr);
    float* l = (float*)malloc(sizeof(float) * nr);
    float* O = (float*)calloc((size_t)nr * D, sizeof(float));
    float* S = (float*)malloc(sizeof(float) * (size_t)nr * bkv);
    int32_t* Pq = (int32_t*)malloc(sizeof(int32_t) * (size_t)bkv);
    const float inv127 = 1.0f / 127.0f;
    for (int a = 0; a < nr; ++a) { m[a] = -INFINITY; l[a] = 0.0f; }

    for (int j = 0; j < Tn; ++j) {
        int c0 = j * bkv, c1 = c0 + bkv < N ? c0 + bkv : N, nc = c1 - c0;
        if (causal && c0 > r1 - 1 + shift) break;
        for (int a = 0; a < nr; ++a)
            for (int b = 0; b < nc; ++b) {
                int32_t acc = 0;
                for (int c = 0; c < D; ++c)
                    acc += (int32_t)qq[(int64_t)(r0 + a) * D + c] * (int32_t)kq[(int64_t)(c0 + b) * D + c];
                volatile float t1 = (float)acc * q_scale[(r0 + a) / gq];
                volatile float t2 = t1 * k_scale[(c0 + b) / gk];
                S[a * bkv + b] = (causal && (c0 + b) > (r0 + a + shift)) ? -INFINITY : t2;
            }
        for (int a = 0; a < nr; ++a) {
            float m_old = m[a], m_new = m_old;
            for (int b = 0; b < nc; ++b) if (S[a * bkv + b] > m_new) m_new = S[a * bkv + b];
            float alpha = (m_old == -INFINITY) ? 0.0f : expf(m_old - m_new);
            float rowsum = 0.0f;
            for (int b = 0; b < nc; ++b) {
                float p = (S[a * bkv + b] == -INFINITY) ? 0.0f : expf(S[a * bkv + b] - m_new);
                volatile float scaled = p * 127.0f;
                Pq[b] = (int32_t)nearbyintf(scaled);             /* 0 .. 127 */
                volatile float acc = rowsum + p;
                rowsum = acc;
            }
            volatile float lnew = alpha * l[a];
            lnew = lnew + rowsum;
            l[a] = lnew;
            m[a] = m_new;
            for (int c = 0; c < D; ++c) {
                int32_t A = 0;
                for (int b = 0; b < nc; ++b) A += Pq[b] * (int32_t)vq[(int64_t)(c0 + b) * D + c];
                volatile float t1 = (float)A * inv127;
                volatile float t2 = t1 * v_scale[c];
                volatile float oc = alpha * O[(int64_t)a * D + c];
                volatile float sum = oc + t2;
                O[(int64_t)a * D + c] = sum;
            }
        }
    }
    for (int a = 0; a < nr; ++a) {
        for (int c = 0; c < D; ++c) {
            volatile float q = O[(int64_t)a * D + c] / l[a];
            o[(int64_t)(r0 + a) * D + c] = f32_to_f16(q, 0);
        }
        if (lsum) lsum[r0 + a] = l[a];
        if (mrow) mrow[r0 + a] = m[a];
    }
    free(m); free(l); free(O); free(S); free(Pq);
}

/* One slab, a list of Q blocks (nblocks < 0: all).  gran_q / gran_k as in the FP16 variant:
 * block sizes for -vB, 1 for -vT.  lsum [N] may be NULL. */
void sage_oracle_attn_pv8_slab_g(const int8_t* qq, const float* q_scale, const int8_t* kq,
                                 const float* k_scale, const int8_t* vq, const float* v_scale,
                                 int N, int D, int causal, int block_q, int block_k, int gran_q, int gran_k,
                                 const int* blocks, int nblocks, uint16_t* o, float* lsum) {
    int Tm = (N + block_q - 1) / block_q;
    int n = nblocks < 0 ? Tm : nblocks;
#pragma omp parallel for schedule(dynamic)
    for (int u = 0; u < n; ++u) {
        int i = nblocks < 0 ? u : blocks[u];
        l2_pv8_q_block(qq, q_scale, kq, k_scale, vq, v_scale, N, N, D, causal, block_q, block_k,
                       gran_q, gran_k, i, o, lsum, NULL);
    }
}

/* Whole tensors [B,H,N,D]; v_scale [B,H,D]; lsum [B,H,N] or NULL. */
void sage_oracle_attn_pv8_g(const int8_t* qq, const float* q_scale, const int8_t* kq, const float* k_scale,
                            const int8_t* vq, const float* v_scale, int B, int H, int N, int D, int causal,
                            int block_q, int block_k, int gran_q, int gran_k, uint16_t* o, float* lsum) {
    int Tm = (N + block_q - 1) / block_q;
    int nsq = (N + gran_q - 1) / gran_q, nsk = (N + gran_k - 1) / gran_k;
    int64_t units = (int64_t)B * H * Tm;
#pragma omp parallel for schedule(dynamic)
    for (int64_t u = 0; u < units; ++u) {
        int64_t s = u / Tm; int i = (int)(u % Tm);
        l2_pv8_q_block(qq + s * N * D, q_scale + s * nsq, kq + s * N * D, k_scale + s * nsk,
                       vq + s * N * D, v_scale + s * D, N, N, D, causal, block_q, block_k, gran_q, gran_k,
                       i, o + s * N * D, lsum ? lsum + s * N : NULL, NULL);
    }
}

/* The same with Nq queries against Nk keys: Q^ [B,H,Nq,D], K^ and V^ [B,H,Nk,D], output, lsum and
 * mrow (the final row maxima m of Algorithm 1, in the units of S; may be NULL) over Nq rows. */
void sage_oracle_attn_pv8_cross_g(const int8_t* qq, const float* q_scale, const int8_t* kq, const float* k_scale,
                                  const int8_t* vq, const float* v_scale, int B, int H, int Nq, int Nk, int D,
                                  int causal, int block_q, int block_k, int gran_q, int gran_k,
                                  uint16_t* o, float* lsum, float* mrow) {
    int Tm = (Nq + block_q - 1) / block_q;
    int nsq = (Nq + gran_q - 1) / gran_q, nsk = (Nk + gran_k - 1) / gran_k;
    int64_t units = (int64_t)B * H * Tm;
#pragma omp parallel for schedule(dynamic)
    for (int64_t u = 0; u < units; ++u) {
        int64_t s = u / Tm; int i = (int)(u % Tm);
        l2_pv8_q_block(qq + s * Nq * D, q_scale + s * nsq, kq + s * Nk * D, k_scale + s * nsk,
                       vq + s * Nk * D, v_scale + s * D, Nq, Nk, D, causal, block_q, block_k, gran_q, gran_k,
                       i, o + s * Nq * D, lsum ? lsum + s * Nq : NULL, mrow ? mrow + s * Nq : NULL);
    }
}

/* ------------------------------------------------------------------ L1: quantized S, exact softmax */

/* Rows [row0,row0+nrows) of one slab: S = dQ dK S^ in fp64, two-pass softmax, fp64 P V.
 * block_q / block_k are the tokens per scale here (1 = per-token quantizer); L1 has no block loop. */
void sage_oracle_attn_l1_slab(const int8_t* qq, const float* q_scale, const int8_t* kq,
                              const float* k_scale, const uint16_t* v, int N, int D, int causal,
                              int block_q, int block_k, int row0, int nrows, double* o /* [nrows,D] */) {
#pragma omp parallel for schedule(dynamic)
    for (int a = 0; a < nrows; ++a) {
        int t = row0 + a;
        int last = causal ? t : N - 1;
        double* s = (double*)malloc(sizeof(double) * (size_t)(last + 1));
        double mx = -INFINITY;
        for (int j = 0; j <= last; ++j) {
            int64_t acc = 0;
            for (int c = 0; c < D; ++c) acc += (int64_t)qq[(int64_t)t * D + c] * (int64_t)kq[(int64_t)j * D + c];
            s[j] = (double)acc * (double)q_scale[t / block_q] * (double)k_scale[j / block_k];
            if (s[j] > mx) mx = s[j];
        }
        double den = 0.0;
        for (int j = 0; j <= last; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
        for (int c = 0; c < D; ++c) {
            double acc = 0.0;
            for (int j = 0; j <= last; ++j) acc += s[j] * (double)f16_to_f32(v[(int64_t)j * D + c]);
            o[(int64_t)a * D + c] = acc / den;
        }
        free(s);
    }
}

/* ------------------------------------------------------------------ L0: exact attention (Section 3.1) */

/* Rows [row0,row0+nrows) of softmax(Q K^T sm_scale) V for one slab, all in fp64.
 * q, k, v are fp32 arrays holding the values to use (so that smoothed or shifted K can be fed). */
void sage_oracle_attn_l0_slab(const float* q, const float* k, const float* v, int N, int D,
                              int causal, double sm_scale, int row0, int nrows, double* o) {
#pragma omp parallel for schedule(dynamic)
    for (int a = 0; a < nrows; ++a) {
        int t = row0 + a;
        int last = causal ? t : N - 1;
        double* s = (double*)malloc(sizeof(double) * (size_t)(last + 1));
        double mx = -INFINITY;
        for (int j = 0; j <= last; ++j) {
            double acc = 0.0;
            for (int c = 0; c < D; ++c) acc += (double)q[(int64_t)t * D + c] * (double)k[(int64_t)j * D + c];
            s[j] = acc * sm_scale;
            if (s[j] > mx) mx = s[j];
        }
        double den = 0.0;
        for (int j = 0; j <= last; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
        for (int c = 0; c < D; ++c) {
            double acc = 0.0;
            for (int j = 0; j <= last; ++j) acc += s[j] * (double)v[(int64_t)j * D + c];
            o[(int64_t)a * D + c] = acc / den;
        }
        free(s);
    }
}

int sage_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
