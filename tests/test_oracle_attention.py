"""Pins for the attention half of the CPU oracle (levels L0, L1, L2).

Expected values come from: an independent numpy fp64 brute force of Section 3.1's definition,
the shift-invariance identity of Section 4.2, closed-form special cases, error bounds that
follow from the quantizer's definition, and the accuracy figures the paper prints."""
import os

import numpy as np
import pytest

import oracle
import sage_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_attention(q, k, v, causal, sm_scale):
    """softmax(Q K^T sm_scale) V with numpy in fp64 -- independent of the C code."""
    q, k, v = (np.asarray(a, np.float64) for a in (q, k, v))
    s = (q @ k.T) * sm_scale
    if causal:
        n = s.shape[0]
        s = np.where(np.arange(n)[None, :] > np.arange(n)[:, None], -np.inf, s)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    return (p / p.sum(axis=1, keepdims=True)) @ v


def quantized_inputs(q, k, v, sm_scale, bq, bk, flags=0):
    mean = oracle.k_mean(k)
    kq, kd = oracle.quant_per_block(oracle.smooth_k(k, mean), bk, flags)
    qq, qd = oracle.quant_per_block(oracle.scale_q(q, sm_scale), bq, flags)
    return qq, qd, kq, kd


def rand_qkv(seed, N, D, k_bias=0.0, k_noise=1.0):
    g = np.random.default_rng(seed)
    q = g.standard_normal((N, D), dtype=np.float32).astype(np.float16)
    k = (g.standard_normal((N, D), dtype=np.float32) * k_noise + g.standard_normal(D, dtype=np.float32) * k_bias).astype(np.float16)
    v = g.standard_normal((N, D), dtype=np.float32).astype(np.float16)
    return q, k, v


def paper_numbers():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_kernel_accuracy.txt")):
        if line.strip() and not line.startswith("#"):
            name, cos, l1, rmse = line.split()
            out[name] = (float(cos), float(l1), float(rmse))
    return out


# ------------------------------------------------------------------ L0

@pytest.mark.parametrize("N,D,causal", [(1, 4, False), (5, 3, True), (37, 16, False), (64, 8, True), (50, 16, True)])
def test_l0_matches_numpy_brute_force(N, D, causal):
    q, k, v = rand_qkv(N * 7 + D, N, D, k_bias=2.0)
    ref = brute_attention(q, k, v, causal, 0.3)
    got = oracle.attn_l0_slab(q, k, v, causal, 0.3)
    assert np.abs(got - ref).max() <= 1e-12
    sub = oracle.attn_l0_slab(q, k, v, causal, 0.3, row0=N // 2, nrows=N - N // 2)
    assert np.array_equal(sub, got[N // 2:])


@pytest.mark.parametrize("causal", [False, True])
def test_smoothing_k_leaves_exact_attention_unchanged(causal):
    # sigma(q (K - mean)^T) = sigma(q K^T): the shift is constant along every row
    q, k, v = rand_qkv(21, 96, 16, k_bias=5.0)
    ks = oracle.smooth_k(k, oracle.k_mean(k))
    a = oracle.attn_l0_slab(q, k, v, causal, 0.25)
    b = oracle.attn_l0_slab(q, ks, v, causal, 0.25)
    assert np.abs(a - b).max() <= 1e-6          # ks carries one fp32 rounding per element
    # and with an exactly representable shift the identity holds to fp64 rounding
    shift = np.float32(2.0)
    c = oracle.attn_l0_slab(q, k.astype(np.float32) - shift, v, causal, 0.25)
    assert np.abs(a - c).max() <= 1e-10


# ------------------------------------------------------------------ S^ and S

def test_integer_scores_match_int64_matmul_and_bound():
    g = np.random.default_rng(5)
    N, D = 150, 64
    qq = g.integers(-127, 128, (N, D), dtype=np.int8); kq = g.integers(-127, 128, (N, D), dtype=np.int8)
    kq[3] = 127; qq[7] = -127                      # extreme corner: -127*127*D
    s = oracle.qk_i32(qq, kq)
    ref = qq.astype(np.int64) @ kq.astype(np.int64).T
    assert s.dtype == np.int32 and np.array_equal(s, ref)
    assert s[7, 3] == -127 * 127 * D and np.abs(s).max() <= 127 * 127 * D
    assert np.array_equal(oracle.qk_i32(qq, kq, 10, 20), ref[10:30])


def test_dequantized_scores_obey_the_quantization_error_bound():
    # |S - Qs Ks^T| <= (dQ/2) sum|Ks| + (dK/2) sum|Qs| + D dQ dK / 4  (+ fp32 slack)
    N, D, bq, bk = 256, 64, 128, 64
    q, k, v = rand_qkv(8, N, D, k_bias=3.0, k_noise=0.5)
    sm = 0.125
    qs = oracle.scale_q(q, sm).astype(np.float64)
    ks = oracle.smooth_k(k, oracle.k_mean(k)).astype(np.float64)
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, bq, bk)
    s_hat = oracle.qk_i32(qq, kq).astype(np.float64)
    dq = np.repeat(qd.astype(np.float64), bq)[:N, None]; dk = np.repeat(kd.astype(np.float64), bk)[None, :N]
    s = s_hat * dq * dk
    exact = qs @ ks.T
    bound = 0.5 * dq * np.abs(ks).sum(1)[None, :] + 0.5 * dk * np.abs(qs).sum(1)[:, None] + D * dq * dk / 4
    assert np.all(np.abs(s - exact) <= bound * (1 + 1e-3))
    assert np.abs(s - exact).max() > 0.01 * bound.max()          # the bound is not vacuous


# ------------------------------------------------------------------ L1 against L0 (the method's accuracy)

def test_l1_accuracy_on_normal_inputs_matches_the_papers_order_of_magnitude():
    cos_p, l1_p, rmse_p = paper_numbers()["sageattn_b_normal"]
    q, k, v = rand_qkv(0, 1024, 64)
    sm = 0.125
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, 128, 64)
    m = oracle.accuracy_metrics(oracle.attn_l0_slab(q, k, v, False, sm),
                                oracle.attn_l1_slab(qq, qd, kq, kd, v, False, 128, 64))
    assert m["cos"] > 0.9999 and round(m["cos"], 3) == cos_p
    assert l1_p / 4 < m["rel_l1"] < l1_p * 2
    assert rmse_p / 4 < m["rmse"] < rmse_p * 2


def test_smoothing_rescues_per_block_int8_on_channel_biased_k():
    """Qualitative pin to the appendix table: without smoothing per-block INT8 attention collapses
    on K with large shared per-channel bias; with smoothing it recovers."""
    nums = paper_numbers()
    q, k, v = rand_qkv(3, 512, 64, k_bias=100.0, k_noise=0.5)
    sm = 0.5
    ref = oracle.attn_l0_slab(q, k, v, False, sm)
    qq, qd = oracle.quant_per_block(oracle.scale_q(q, sm), 128)
    kq_raw, kd_raw = oracle.quant_per_block(k.astype(np.float32), 64)           # psi_K without gamma
    kq_s, kd_s = oracle.quant_per_block(oracle.smooth_k(k, oracle.k_mean(k)), 64)
    without = oracle.accuracy_metrics(ref, oracle.attn_l1_slab(qq, qd, kq_raw, kd_raw, v, False, 128, 64))
    with_s = oracle.accuracy_metrics(ref, oracle.attn_l1_slab(qq, qd, kq_s, kd_s, v, False, 128, 64))
    assert with_s["cos"] > nums["per_block_with_smoothing"][0]
    assert without["cos"] < 0.6 and without["rel_l1"] > 10 * with_s["rel_l1"]
    assert abs(without["cos"] - nums["per_block_without_smoothing"][0]) < 0.3       # same regime as the paper's 30.6 %


# ------------------------------------------------------------------ L2 (Algorithm 1) against L1

@pytest.mark.parametrize("N,D,bq,bk,causal", [(256, 64, 64, 64, False), (300, 64, 128, 64, True),
                                               (200, 128, 128, 64, False), (130, 32, 32, 16, True)])
def test_l2_online_softmax_agrees_with_two_pass_l1(N, D, bq, bk, causal):
    q, k, v = rand_qkv(N + D, N, D, k_bias=3.0, k_noise=0.5)
    sm = float(1 / np.sqrt(D))
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, bq, bk)
    o2 = oracle.attn_l2_slab(qq, qd, kq, kd, v, causal, bq, bk).astype(np.float64)
    o1 = oracle.attn_l1_slab(qq, qd, kq, kd, v, causal, bq, bk)
    assert np.abs(o2 - o1).max() <= 1e-3 + 2.0 ** -11 * np.abs(o1).max()        # fp16 output + fp16 P~
    assert oracle.accuracy_metrics(o1, o2)["cos"] > 0.999999


def test_l2_whole_tensor_entry_equals_slab_entry_and_block_subsets():
    w = si.custom("t", 2, 2, 200, 32, True, 64, 32)
    q, k, v = si.full(w)
    kq, ks, km = oracle.smooth_quant_k(k, w.block_k)
    qq, qs = oracle.quant_q(q, w.sm_scale, w.block_q)
    o = oracle.attn_l2(qq, qs, kq, ks, v, True, w.block_q, w.block_k)
    for b in range(2):
        for h in range(2):
            o_s = oracle.attn_l2_slab(qq[b, h], qs[b, h], kq[b, h], ks[b, h], v[b, h], True, 64, 32)
            assert np.array_equal(o[b, h].view(np.uint16), o_s.view(np.uint16))
    part = oracle.attn_l2_slab(qq[1, 0], qs[1, 0], kq[1, 0], ks[1, 0], v[1, 0], True, 64, 32, q_blocks=[3, 1])
    assert np.array_equal(part[64:128], o[1, 0, 64:128]) and np.array_equal(part[192:], o[1, 0, 192:])
    assert np.all(part[:64] == 0) and np.all(part[128:192] == 0)


def test_constant_k_gives_running_or_global_mean_of_v():
    """K identical for all tokens => K - mean(K) = 0 exactly => S = 0 => uniform attention."""
    N, D = 192, 16
    g = np.random.default_rng(2)
    q = g.standard_normal((N, D)).astype(np.float16)
    k = np.tile(g.standard_normal((1, D)).astype(np.float16), (N, 1))
    v = g.standard_normal((N, D)).astype(np.float16)
    qq, qd, kq, kd = quantized_inputs(q, k, v, 0.25, 64, 64)
    assert np.all(kq == 0) and np.all(kd == 0)                                   # all-zero blocks
    v64 = v.astype(np.float64)
    o = oracle.attn_l2_slab(qq, qd, kq, kd, v, False, 64, 64).astype(np.float64)
    assert np.abs(o - v64.mean(0)[None]).max() <= 2e-3
    oc = oracle.attn_l2_slab(qq, qd, kq, kd, v, True, 64, 64).astype(np.float64)
    prefix = np.cumsum(v64, 0) / np.arange(1, N + 1)[:, None]
    assert np.abs(oc - prefix).max() <= 2e-3


def test_causal_first_row_is_v0_bit_exactly_and_rows_only_see_their_prefix():
    q, k, v = rand_qkv(4, 160, 32, k_bias=2.0)
    qq, qd, kq, kd = quantized_inputs(q, k, v, 0.2, 64, 32)
    o = oracle.attn_l2_slab(qq, qd, kq, kd, v, True, 64, 32)
    assert np.array_equal(o[0].view(np.uint16), v[0].view(np.uint16))
    # changing V (not K: K feeds the mean) strictly after row t leaves rows <= t untouched
    v2 = v.copy(); v2[100:] = 7.0
    o2 = oracle.attn_l2_slab(qq, qd, kq, kd, v2, True, 64, 32)
    assert np.array_equal(o[:100], o2[:100]) and not np.array_equal(o[100:], o2[100:])


def test_output_is_a_convex_combination_of_v_rows():
    q, k, v = rand_qkv(6, 130, 16, k_bias=1.0)
    qq, qd, kq, kd = quantized_inputs(q, k, v, 0.25, 64, 64)
    o = oracle.attn_l2_slab(qq, qd, kq, kd, v, False, 64, 64).astype(np.float64)
    lo, hi = v.astype(np.float64).min(0), v.astype(np.float64).max(0)
    assert np.all(o >= lo - 2e-3) and np.all(o <= hi + 2e-3)
    vc = np.full_like(v, 1.25)
    oc = oracle.attn_l2_slab(qq, qd, kq, kd, vc, False, 64, 64)
    assert np.abs(oc.astype(np.float64) - 1.25).max() <= 1e-3


def test_one_hot_attention_selects_the_matching_value_row():
    """Keys that are +/- large along private channels make softmax pick one row: O[t] ~= V[pi(t)]."""
    N, D = 64, 64
    perm = np.random.default_rng(1).permutation(N)
    k = np.zeros((N, D), np.float16); q = np.zeros((N, D), np.float16)
    for t in range(N):
        k[t, t] = 8.0
        q[t, perm[t]] = 8.0
    k[:, :] -= 0.0
    v = np.random.default_rng(2).standard_normal((N, D)).astype(np.float16)
    qq, qd, kq, kd = quantized_inputs(q, k, v, 1.0, 64, 64)
    o = oracle.attn_l2_slab(qq, qd, kq, kd, v, False, 64, 64).astype(np.float32)
    assert np.abs(o - v[perm].astype(np.float32)).max() <= 2e-3     # a transposed operand would give V[perm^-1]


def test_tail_blocks_do_not_leak_padding():
    # N not a multiple of either block: the result for the first rows must not depend on how the
    # tensors would be padded, and must match the two-pass level.
    q, k, v = rand_qkv(12, 177, 32, k_bias=2.0)
    qq, qd, kq, kd = quantized_inputs(q, k, v, 0.2, 128, 64)
    assert qd.shape == (2,) and kd.shape == (3,)
    o2 = oracle.attn_l2_slab(qq, qd, kq, kd, v, False, 128, 64).astype(np.float64)
    o1 = oracle.attn_l1_slab(qq, qd, kq, kd, v, False, 128, 64)
    assert np.abs(o2 - o1).max() <= 2e-3


def test_fp16_accumulator_and_rounding_switches_stay_close_to_algorithm_1():
    """Section 4.4's claim: an fp16 accumulator for P~V loses no accuracy against fp32."""
    q, k, v = rand_qkv(13, 512, 64, k_bias=3.0, k_noise=0.5)
    sm = 0.125
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, 128, 64)
    ref = oracle.attn_l0_slab(q, k, v, False, sm)
    base = oracle.attn_l2_slab(qq, qd, kq, kd, v, False, 128, 64)
    acc16 = oracle.attn_l2_slab(qq, qd, kq, kd, v, False, 128, 64, flags=oracle.ACC_FP16)
    m32, m16 = oracle.accuracy_metrics(ref, base), oracle.accuracy_metrics(ref, acc16)
    assert abs(m32["cos"] - m16["cos"]) < 1e-4 and m16["rmse"] < 2 * m32["rmse"] + 1e-3
    trunc = oracle.attn_l2_slab(qq, qd, kq, kd, v, False, 128, 64, flags=oracle.P_TRUNCATE | oracle.L_FROM_P16)
    assert np.abs(trunc.astype(np.float64) - base.astype(np.float64)).max() <= 1e-3


def test_cfg1_end_to_end_accuracy_against_exact_attention():
    w = si.WORKLOADS["cfg1_tiny"]
    q, k, v = si.full(w)
    kq, ks, km = oracle.smooth_quant_k(k, w.block_k)
    qq, qs = oracle.quant_q(q, w.sm_scale, w.block_q)
    o = oracle.attn_l2(qq, qs, kq, ks, v, w.causal, w.block_q, w.block_k)
    ref = np.stack([oracle.attn_l0_slab(q[0, h], k[0, h], v[0, h], False, w.sm_scale) for h in range(w.H)])[None]
    m = oracle.accuracy_metrics(ref, o)
    assert m["cos"] > 0.9999 and m["rel_l1"] < 0.03


# ------------------------------------------------------------------ per-token scales (SAGEAttn-T)

def brute_quantized_attention(qq, dq_tok, kq, dk_tok, v, causal):
    """softmax(diag(dQ) Q^ K^^T diag(dK)) V with numpy in fp64, one scale per token -- Section 4.1's
    formula with Section 3.2's per-token quantizer, independent of the C code."""
    s = (qq.astype(np.float64) @ kq.astype(np.float64).T) * dq_tok.astype(np.float64)[:, None] * dk_tok.astype(np.float64)[None, :]
    if causal:
        n = s.shape[0]
        s = np.where(np.arange(n)[None, :] > np.arange(n)[:, None], -np.inf, s)
    p = np.exp(s - s.max(axis=1, keepdims=True))
    return (p / p.sum(axis=1, keepdims=True)) @ v.astype(np.float64)


@pytest.mark.parametrize("N,D,bq,bk,causal", [(200, 32, 64, 32, False), (177, 64, 128, 64, True)])
def test_per_token_scales_repeated_from_block_scales_reproduce_algorithm_1_bit_for_bit(N, D, bq, bk, causal):
    # a per-token scale vector that is constant inside every block IS the per-block method
    q, k, v = rand_qkv(31 + N, N, D, k_bias=2.0)
    qq, qd, kq, kd = quantized_inputs(q, k, v, 0.2, bq, bk)
    base = oracle.attn_l2_slab(qq, qd, kq, kd, v, causal, bq, bk)
    qd_tok, kd_tok = np.repeat(qd, bq)[:N], np.repeat(kd, bk)[:N]
    tok = oracle.attn_l2_slab(qq, qd_tok, kq, kd_tok, v, causal, bq, bk, gran_q=1, gran_k=1)
    assert np.array_equal(base.view(np.uint16), tok.view(np.uint16))
    mixed = oracle.attn_l2_slab(qq, qd_tok, kq, kd, v, causal, bq, bk, gran_q=1)
    assert np.array_equal(base.view(np.uint16), mixed.view(np.uint16))


@pytest.mark.parametrize("causal", [False, True])
def test_per_token_levels_match_the_numpy_definition_with_unrelated_scale_vectors(causal):
    # random codes and two unrelated scale vectors: a scale applied along the wrong axis, or
    # indexed by the block instead of the token, changes the result by far more than the tolerance
    g = np.random.default_rng(77)
    N, D = 150, 32
    qq = g.integers(-127, 128, (N, D), dtype=np.int8); kq = g.integers(-127, 128, (N, D), dtype=np.int8)
    dq = (g.uniform(0.2, 3.0, N) * 2e-3).astype(np.float32); dk = (g.uniform(0.2, 3.0, N) * 2e-3).astype(np.float32)
    v = g.standard_normal((N, D)).astype(np.float16)
    ref = brute_quantized_attention(qq, dq, kq, dk, v, causal)
    o1 = oracle.attn_l1_slab(qq, dq, kq, dk, v, causal, 1, 1)
    assert np.abs(o1 - ref).max() <= 1e-12
    o2 = oracle.attn_l2_slab(qq, dq, kq, dk, v, causal, 64, 32, gran_q=1, gran_k=1).astype(np.float64)
    assert np.abs(o2 - ref).max() <= 1e-3 + 2.0 ** -11 * np.abs(ref).max()
    swapped = brute_quantized_attention(qq, dk, kq, dq, v, causal)
    assert np.abs(swapped - ref).max() > 0.05           # the inputs do tell the two axes apart
    # the loop's block sizes do not matter once the scales are per token
    o3 = oracle.attn_l2_slab(qq, dq, kq, dk, v, causal, 32, 64, gran_q=1, gran_k=1).astype(np.float64)
    assert np.abs(o3 - o2).max() <= 1e-3


def test_per_token_whole_tensor_entry_equals_slab_entry():
    w = si.custom("t", 2, 2, 150, 32, True, 64, 32)
    q, k, v = si.full(w)
    kq, ks, km = oracle.smooth_quant_k(k, 1)
    qq, qs = oracle.quant_q(q, w.sm_scale, 1)
    assert ks.shape == (2, 2, 150) and qs.shape == (2, 2, 150)
    o = oracle.attn_l2(qq, qs, kq, ks, v, True, 64, 32, gran_q=1, gran_k=1)
    for b in range(2):
        for h in range(2):
            o_s = oracle.attn_l2_slab(qq[b, h], qs[b, h], kq[b, h], ks[b, h], v[b, h], True, 64, 32, gran_q=1, gran_k=1)
            assert np.array_equal(o[b, h].view(np.uint16), o_s.view(np.uint16))


def test_per_token_accuracy_on_normal_inputs_matches_the_papers_order_of_magnitude():
    nums = paper_numbers()
    cos_p, l1_p, rmse_p = nums["sageattn_t_normal"]
    q, k, v = rand_qkv(0, 1024, 64)
    sm = 0.125
    ref = oracle.attn_l0_slab(q, k, v, False, sm)
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, 1, 1)
    m_t = oracle.accuracy_metrics(ref, oracle.attn_l1_slab(qq, qd, kq, kd, v, False, 1, 1))
    assert m_t["cos"] > 0.9999 and round(m_t["cos"], 3) == cos_p
    assert l1_p / 4 < m_t["rel_l1"] < l1_p * 2 and rmse_p / 4 < m_t["rmse"] < rmse_p * 2
    # the paper's ordering: per-token is (slightly) more accurate than per-block on the same inputs
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, 128, 64)
    m_b = oracle.accuracy_metrics(ref, oracle.attn_l1_slab(qq, qd, kq, kd, v, False, 128, 64))
    assert m_t["rel_l1"] < m_b["rel_l1"] and m_t["rmse"] < m_b["rmse"]
    assert m_t["rel_l1"] > 0.5 * m_b["rel_l1"]          # ... but of the same order (paper: 0.019 against 0.021)


def test_per_token_scales_absorb_token_outliers_that_hurt_per_block_scales():
    """A few tokens 30x larger than the rest share their block's scale under the per-block
    quantizer and crush the other tokens' codes; the per-token quantizer is immune."""
    q, k, v = rand_qkv(9, 512, 64)
    g = np.random.default_rng(10)
    big = g.choice(512, 16, replace=False)
    q = q.copy(); k = k.copy()
    q[big] *= np.float16(30.0); k[g.choice(512, 16, replace=False)] *= np.float16(30.0)
    sm = 0.02
    ref = oracle.attn_l0_slab(q, k, v, False, sm)
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, 1, 1)
    m_t = oracle.accuracy_metrics(ref, oracle.attn_l1_slab(qq, qd, kq, kd, v, False, 1, 1))
    qq, qd, kq, kd = quantized_inputs(q, k, v, sm, 128, 64)
    m_b = oracle.accuracy_metrics(ref, oracle.attn_l1_slab(qq, qd, kq, kd, v, False, 128, 64))
    assert m_t["rmse"] < 0.5 * m_b["rmse"] and m_t["cos"] > 0.99 > m_b["cos"]
