"""GPU parity of the per-token variant (SAGEAttn-T: Section 3.2's per-token quantizer for Q and K
inside Algorithm 1's loop) against the CPU oracle, through the C ABI with block_q = block_k = 1.

Bit-exact: INT8 tensors, per-token scales, K mean.  Output: max-abs <= 2e-3, cosine >= 0.9999
against the oracle's Algorithm-1 level run with one scale per token and the paper's 128 x 64 loop
blocks."""
import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import assert_output_close, assert_prepass_bit_exact, bits, to_dev, with_token_outliers

pytestmark = pytest.mark.gpu

LOOP_Q, LOOP_K = 128, 64          # Algorithm 1's block sizes; they no longer fix the scales

SMALL = [
    si.WORKLOADS["cfg1_tiny"],
    si.custom("ragged_d128", 1, 3, 333, 128, False, 128, 64, seed=si.BASE_SEED + 31),
    si.custom("ragged_d64_causal", 2, 2, 457, 64, True, 128, 64, seed=si.BASE_SEED + 32),
    si.custom("causal_d128", 1, 2, 640, 128, True, 128, 64, k_noise=1.0, k_bias=4.0, outlier_frac=0.01,
              outlier_gain=8.0, seed=si.BASE_SEED + 33),
    si.custom("one_token", 1, 1, 1, 64, True, 128, 64, seed=si.BASE_SEED + 34),
    si.custom("short", 2, 1, 31, 128, False, 128, 64, seed=si.BASE_SEED + 35),
    si.custom("whole_tiles", 2, 2, 512, 128, False, 128, 64, seed=si.BASE_SEED + 36),
    si.custom("one_past_a_tile", 1, 2, 257, 64, True, 128, 64, seed=si.BASE_SEED + 37),
]


def run_and_compare(q, k, v, w, block_q, block_k, what):
    (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km) = assert_prepass_bit_exact(
        q, k, w.sm_scale, block_q, block_k)
    o_gpu = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), w.causal, w.sm_scale, block_q, block_k)
    torch.cuda.synchronize()
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, w.causal, LOOP_Q, LOOP_K,
                           gran_q=block_q if block_q == 1 else LOOP_Q, gran_k=block_k if block_k == 1 else LOOP_K)
    return assert_output_close(o_gpu.cpu().numpy(), o_ref, what)


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_small_workloads_per_token_parity(w):
    print(f"[case] per-token {w.name} B{w.B} H{w.H} N{w.N} D{w.D} causal={w.causal}", flush=True)
    q, k, v = si.full(w)
    run_and_compare(q, k, v, w, 1, 1, w.name)


@pytest.mark.parametrize("D,causal", [(128, False), (64, True)])
def test_token_outliers_per_token_parity(D, causal):
    print(f"[case] per-token, outlier tokens D{D} causal={causal}", flush=True)
    w = si.custom("outlier_tokens", 1, 2, 900, D, causal, 128, 64, seed=si.BASE_SEED + 40 + D)
    q, k, v = with_token_outliers(w)
    run_and_compare(q, k, v, w, 1, 1, w.name)
    # the scales inside one 64-key tile do differ by about the planted gain
    ks = oracle.smooth_quant_k(k, 1)[1][0, 0]
    spread = [ks[i:i + 64].max() / ks[i:i + 64].min() for i in range(0, 896, 64)]
    assert max(spread) > 6.0


@pytest.mark.parametrize("block_q,block_k", [(1, 64), (128, 1), (1, 128), (32, 1)])
def test_per_token_on_one_side_only(block_q, block_k):
    """Q per token with K per block and the reverse: both granularities are independent arguments."""
    print(f"[case] mixed granularity {block_q} x {block_k}", flush=True)
    w = si.custom("mixed", 1, 2, 700, 128, True, 128, 64, seed=si.BASE_SEED + 50)
    q, k, v = with_token_outliers(w)
    (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km) = assert_prepass_bit_exact(
        q, k, w.sm_scale, block_q, block_k)
    o_gpu = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), True, w.sm_scale, block_q, block_k)
    torch.cuda.synchronize()
    # loop blocks: multiples of the scale blocks, so that every scale block sits inside one loop block
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, True, 128, 128, gran_q=block_q, gran_k=block_k)
    assert_output_close(o_gpu.cpu().numpy(), o_ref, f"mixed {block_q}x{block_k}")


def test_per_token_all_zero_tokens_and_constant_k():
    """K constant over tokens: every smoothed token is exactly zero, every per-token scale is 0 and
    attention is uniform; causal row 0 returns V[0] bit for bit."""
    print("[case] per-token, constant K", flush=True)
    N, D = 300, 128
    g = np.random.default_rng(6)
    q = g.standard_normal((1, 1, N, D)).astype(np.float16)
    v = g.standard_normal((1, 1, N, D)).astype(np.float16)
    k = np.tile(g.standard_normal((1, 1, 1, D)).astype(np.float16), (1, 1, N, 1))
    q[0, 0, 17] = 0                                       # an all-zero query token as well
    (q_i8, q_scale, k_i8, k_scale, k_mean), _ = assert_prepass_bit_exact(q, k, 0.1, 1, 1)
    assert float(k_scale.abs().max()) == 0.0 and float(q_scale[0, 0, 17]) == 0.0
    o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), True, 0.1, 1, 1).cpu().numpy()
    assert np.array_equal(bits(o[0, 0, 0]), bits(v[0, 0, 0]))
    prefix = np.cumsum(v[0, 0].astype(np.float64), 0) / np.arange(1, N + 1)[:, None]
    assert np.abs(o[0, 0].astype(np.float64) - prefix).max() <= 2e-3


@pytest.mark.parametrize("D,causal", [(128, True), (64, False)])
def test_per_token_scores_that_keep_rising_force_a_rescale_at_every_tile(D, causal):
    print(f"[case] per-token rising scores D{D} causal={causal}", flush=True)
    N = 1100
    g = np.random.default_rng(17 + D)
    u = g.standard_normal(D); u /= np.linalg.norm(u)
    t = (np.arange(N) - N / 2)[:, None]
    k = (t * 0.05 * u[None, :] + 0.01 * g.standard_normal((N, D))).astype(np.float16)[None, None]
    q = (4.0 * np.sqrt(D) * u[None, :] + 0.1 * g.standard_normal((N, D))).astype(np.float16)[None, None]
    v = g.standard_normal((1, 1, N, D)).astype(np.float16)
    sm = float(np.float32(1.0) / np.sqrt(np.float32(D)))
    (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km) = assert_prepass_bit_exact(q, k, sm, 1, 1)
    o_gpu = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), causal, sm, 1, 1)
    torch.cuda.synchronize()
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, causal, LOOP_Q, LOOP_K, gran_q=1, gran_k=1)
    assert_output_close(o_gpu.cpu().numpy(), o_ref, f"rising_d{D}")


FULL = [("cfg3_prefill16k", 2, 5), ("cfg4_video", 1, 4)]


@pytest.mark.parametrize("name,n_heads,n_blocks", FULL, ids=[c[0] for c in FULL])
def test_full_size_per_token_parity(name, n_heads, n_blocks):
    """The benchmark shapes with per-token scales: whole-tensor pre-pass bit-exact, attention on
    sampled Q blocks of the first and last head."""
    w = si.WORKLOADS[name]
    print(f"[case] per-token {name} B{w.B} H{w.H} N{w.N} D{w.D} causal={w.causal}", flush=True)
    q, k, v = si.full(w)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(kd, 1)
    q_i8, q_scale = sage.sage_quant_q(qd, w.sm_scale, 1)
    o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, vd, w.causal, w.sm_scale, 1, 1)
    torch.cuda.synchronize()
    print("  gpu done", flush=True)
    kq, ks, km = oracle.smooth_quant_k(k, 1)
    qq, qs = oracle.quant_q(q, w.sm_scale, 1)
    assert np.array_equal(bits(k_mean.cpu().numpy()), bits(km))
    assert np.array_equal(bits(k_scale.cpu().numpy()), bits(ks))
    assert np.array_equal(bits(q_scale.cpu().numpy()), bits(qs))
    assert np.array_equal(k_i8.cpu().numpy(), kq)
    assert np.array_equal(q_i8.cpu().numpy(), qq)
    print("  pre-pass bit-exact", flush=True)
    Tm = (w.N + LOOP_Q - 1) // LOOP_Q
    o_host = o.cpu().numpy()
    for hi, (b, h) in enumerate([(0, 0), (w.B - 1, w.H - 1)][:n_heads]):
        g = np.random.default_rng(200 + hi)
        blocks = sorted({0, Tm - 1, Tm // 2} | {int(x) for x in g.integers(0, Tm, n_blocks - 3)})
        ref = oracle.attn_l2_slab(qq[b, h], qs[b, h], kq[b, h], ks[b, h], v[b, h], w.causal,
                                  LOOP_Q, LOOP_K, q_blocks=blocks, gran_q=1, gran_k=1)
        rows = np.concatenate([np.arange(i * LOOP_Q, min(w.N, (i + 1) * LOOP_Q)) for i in blocks])
        err, cos = assert_output_close(o_host[b, h][rows], ref[rows], f"{name} head ({b},{h}) blocks {blocks}")
        print(f"  head ({b},{h}) blocks {blocks}: max_abs {err:.2e} cos {cos:.7f}", flush=True)
