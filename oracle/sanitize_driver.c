/*
 * Sanitizer driver for the CPU oracle (TEST INFRASTRUCTURE): calls every exported function of
 * sage_oracle.c on small ragged shapes so that AddressSanitizer / UndefinedBehaviorSanitizer see
 * every loop bound and index expression.  Built and run by tests/test_oracle_sanitizers.py; it
 * checks nothing numerically (the pins in tests/ do that) and prints a checksum only so that the
 * work cannot be optimised away.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void sage_oracle_f16_to_f32(const uint16_t*, float*, int64_t);
void sage_oracle_f32_to_f16(const float*, uint16_t*, int64_t, int);
void sage_oracle_k_mean(const uint16_t*, int, int, float*);
void sage_oracle_smooth_k(const uint16_t*, const float*, int, int, float*);
void sage_oracle_scale_q(const uint16_t*, float, int, int, float*);
void sage_oracle_rope(const uint16_t*, const float*, const float*, int, int, uint16_t*);
void sage_oracle_quant_per_block(const float*, int, int, int, unsigned, int8_t*, float*);
void sage_oracle_smooth_quant_k(const uint16_t*, int, int, int, int, int, unsigned, int8_t*, float*, float*);
void sage_oracle_quant_q(const uint16_t*, int, int, int, int, float, int, unsigned, int8_t*, float*);
void sage_oracle_qk_i32(const int8_t*, const int8_t*, int, int, int, int, int32_t*);
void sage_oracle_attn_l2_g(const int8_t*, const float*, const int8_t*, const float*, const uint16_t*, int, int, int, int,
                           int, int, int, int, int, unsigned, uint16_t*);
void sage_oracle_attn_l2(const int8_t*, const float*, const int8_t*, const float*, const uint16_t*, int, int, int, int,
                         int, int, int, unsigned, uint16_t*);
void sage_oracle_attn_l2_slab_g(const int8_t*, const float*, const int8_t*, const float*, const uint16_t*, int, int, int,
                                int, int, int, int, unsigned, const int*, int, uint16_t*);
void sage_oracle_attn_l1_slab(const int8_t*, const float*, const int8_t*, const float*, const uint16_t*, int, int, int,
                              int, int, int, int, double*);
void sage_oracle_attn_l0_slab(const float*, const float*, const float*, int, int, int, double, int, int, double*);
void sage_oracle_attn_l2_cross_g(const int8_t*, const float*, const int8_t*, const float*, const uint16_t*, int, int, int,
                                 int, int, int, int, int, int, int, unsigned, uint16_t*);
void sage_oracle_quant_v(const uint16_t*, int, int, int, int, int8_t*, float*);
void sage_oracle_attn_pv8_g(const int8_t*, const float*, const int8_t*, const float*, const int8_t*, const float*, int, int,
                            int, int, int, int, int, int, int, uint16_t*, float*);
void sage_oracle_attn_pv8_slab_g(const int8_t*, const float*, const int8_t*, const float*, const int8_t*, const float*,
                                 int, int, int, int, int, int, int, const int*, int, uint16_t*, float*);

static uint32_t rng = 12345u;
static float unit(void) { rng = rng * 1664525u + 1013904223u; return (float)(rng >> 8) / 16777216.0f * 4.0f - 2.0f; }

static void one_case(int B, int H, int N, int D, int bq, int bk, int gq, int gk, int causal, double* sum) {
    int64_t E = (int64_t)B * H * N * D;
    float* f = malloc(sizeof(float) * E);
    uint16_t *q = malloc(2 * E), *k = malloc(2 * E), *v = malloc(2 * E), *o = malloc(2 * E), *kr = malloc(2 * E);
    int8_t *qq = malloc(E), *kq = malloc(E);
    int nq = (N + gq - 1) / gq, nk = (N + gk - 1) / gk;
    float *qs = malloc(sizeof(float) * B * H * nq), *ks = malloc(sizeof(float) * B * H * nk), *km = malloc(sizeof(float) * B * H * D);
    float *cs = malloc(sizeof(float) * N * (D / 2)), *sn = malloc(sizeof(float) * N * (D / 2));
    for (int64_t i = 0; i < E; ++i) f[i] = unit();
    sage_oracle_f32_to_f16(f, q, E, 0);
    for (int64_t i = 0; i < E; ++i) f[i] = unit() + 1.5f;
    sage_oracle_f32_to_f16(f, k, E, 1);
    for (int64_t i = 0; i < E; ++i) f[i] = unit();
    sage_oracle_f32_to_f16(f, v, E, 0);
    sage_oracle_f16_to_f32(v, f, E);
    for (int i = 0; i < N * (D / 2); ++i) { cs[i] = 0.6f; sn[i] = 0.8f; }
    for (int s = 0; s < B * H; ++s) sage_oracle_rope(k + (int64_t)s * N * D, cs, sn, N, D, kr + (int64_t)s * N * D);
    sage_oracle_smooth_quant_k(kr, B, H, N, D, gk, 0, kq, ks, km);
    sage_oracle_quant_q(q, B, H, N, D, 0.25f, gq, 4u, qq, qs);
    sage_oracle_attn_l2_g(qq, qs, kq, ks, v, B, H, N, D, causal, bq, bk, gq, gk, 1u | 8u, o);
    if (gq == bq && gk == bk) sage_oracle_attn_l2(qq, qs, kq, ks, v, B, H, N, D, causal, bq, bk, 2u, o);
    int Tm = (N + bq - 1) / bq, blocks[2] = {Tm - 1, 0};
    sage_oracle_attn_l2_slab_g(qq, qs, kq, ks, v, N, D, causal, bq, bk, gq, gk, 0, blocks, 2, o);
    /* fewer queries than keys: the first Nq rows of Q^ of every slab are repacked as a [B,H,Nq,D] tensor */
    {
        int Nq = N > 3 ? N - 3 : N, nqc = (Nq + gq - 1) / gq;
        int8_t* qc = malloc((size_t)B * H * Nq * D);
        float* qsc = malloc(sizeof(float) * B * H * nqc);
        uint16_t* oc = malloc(2 * (size_t)B * H * Nq * D);
        for (int s = 0; s < B * H; ++s) {
            memcpy(qc + (size_t)s * Nq * D, qq + (size_t)s * N * D, (size_t)Nq * D);
            for (int g = 0; g < nqc; ++g) qsc[s * nqc + g] = qs[s * nq + g];
        }
        sage_oracle_attn_l2_cross_g(qc, qsc, kq, ks, v, B, H, Nq, N, D, causal, bq, bk, gq, gk, 0, oc);
        *sum += oc[0];
        free(qc); free(qsc); free(oc);
    }
    int8_t* vq = malloc(E);
    float *vs = malloc(sizeof(float) * B * H * D), *ls = malloc(sizeof(float) * B * H * N);
    sage_oracle_quant_v(v, B, H, N, D, vq, vs);
    sage_oracle_attn_pv8_g(qq, qs, kq, ks, vq, vs, B, H, N, D, causal, bq, bk, gq, gk, o, ls);
    sage_oracle_attn_pv8_slab_g(qq, qs, kq, ks, vq, vs, N, D, causal, bq, bk, gq, gk, blocks, 2, o, NULL);
    *sum += ls[B * H * N - 1] + vs[0];
    free(vq); free(vs); free(ls);
    int row0 = N / 3, nrows = N - row0;
    double* o1 = malloc(sizeof(double) * nrows * D);
    sage_oracle_attn_l1_slab(qq, qs, kq, ks, v, N, D, causal, gq, gk, row0, nrows, o1);
    int32_t* s32 = malloc(sizeof(int32_t) * nrows * N);
    sage_oracle_qk_i32(qq, kq, N, D, row0, nrows, s32);
    float *qf = malloc(sizeof(float) * N * D), *kf = malloc(sizeof(float) * N * D), *mean = malloc(sizeof(float) * D);
    sage_oracle_scale_q(q, 0.25f, N, D, qf);
    sage_oracle_k_mean(k, N, D, mean);
    sage_oracle_smooth_k(k, mean, N, D, kf);
    sage_oracle_attn_l0_slab(qf, kf, f, N, D, causal, 1.0, row0, nrows, o1);
    float* xs = malloc(sizeof(float) * nk);
    sage_oracle_quant_per_block(kf, N, D, gk, 0, kq, xs);
    for (int i = 0; i < nrows * D; ++i) *sum += o1[i];
    *sum += s32[nrows * N - 1] + o[0] + ks[0] + km[0];
    free(f); free(q); free(k); free(v); free(o); free(kr); free(qq); free(kq); free(qs); free(ks); free(km);
    free(cs); free(sn); free(o1); free(s32); free(qf); free(kf); free(mean); free(xs);
}

int main(void) {
    double sum = 0.0;
    one_case(1, 1, 1, 8, 4, 4, 4, 4, 1, &sum);
    one_case(2, 2, 37, 16, 16, 8, 16, 8, 0, &sum);
    one_case(1, 3, 70, 8, 32, 16, 1, 1, 1, &sum);
    one_case(1, 2, 65, 32, 64, 32, 1, 32, 0, &sum);
    one_case(2, 1, 129, 16, 128, 64, 128, 1, 1, &sum);
    printf("checksum %.6f\n", sum);
    return 0;
}
