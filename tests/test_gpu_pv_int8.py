"""GPU parity of the kernels with an INT8 second product (Section 4.3; SAGEAttn-vB, and -vT with
per-token Q/K scales) against the CPU oracle, through the C ABI.

Bit-exact: the per-channel INT8 codes of V (transposed layout, zero padding included) and delta_V.
Output: the codes of P~ are decided by the last bits of an fp32 exponential, which the two sides
compute differently (hardware exp2 against libm expf), so a code can differ by one here and there;
one code of one key is worth at most delta_V[c] / l in the output (l = the row's softmax denominator
relative to its maximum, returned by the oracle).  The bar is therefore
    |O_gpu - O_oracle| <= 2e-3 + 2 delta_V[c] / l[row]      for every element,
    |O_gpu - O_oracle| <= 2e-3                              for all but at most 1 element in 100 000,
    cosine >= 0.9999."""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import ABS_TOL, COS_TOL, assert_prepass_bit_exact, bits, to_dev, with_token_outliers

pytestmark = pytest.mark.gpu

SMALL = [
    si.WORKLOADS["cfg1_tiny"],
    si.custom("ragged_d128", 1, 3, 333, 128, False, 128, 64, seed=si.BASE_SEED + 61),
    si.custom("ragged_d64_causal", 2, 2, 457, 64, True, 128, 64, seed=si.BASE_SEED + 62),
    si.custom("causal_d128", 1, 2, 640, 128, True, 128, 64, k_noise=1.0, k_bias=4.0, outlier_frac=0.01,
              outlier_gain=8.0, seed=si.BASE_SEED + 63),
    si.custom("one_token", 1, 1, 1, 64, True, 128, 64, seed=si.BASE_SEED + 64),
    si.custom("short", 2, 1, 31, 128, False, 128, 64, seed=si.BASE_SEED + 65),
    si.custom("whole_tiles", 2, 2, 512, 128, False, 128, 64, seed=si.BASE_SEED + 66),
    si.custom("one_past_a_tile", 1, 2, 257, 64, True, 128, 64, seed=si.BASE_SEED + 67),
    si.custom("many_tiles_d64", 1, 2, 2100, 64, False, 128, 64, seed=si.BASE_SEED + 68),
]


def channel_scaled(v, seed):
    """V with channel-wise magnitudes spread over 1.5 decades (what a per-channel scale is for) and
    one all-zero channel."""
    g = np.random.default_rng(seed)
    gain = np.exp(g.uniform(np.log(0.1), np.log(4.0), v.shape[-1])).astype(np.float32)
    gain[3] = 0.0
    return (v.astype(np.float32) * gain).astype(np.float16)


def assert_v_quant_bit_exact(v):
    B, H, N, D = v.shape
    v_i8t, v_scale = sage.sage_quant_v(to_dev(v))
    torch.cuda.synchronize()
    vq, vs = oracle.quant_v(v)
    Np = sage.sage_quant_v_pitch(N)
    assert Np == 64 * ((N + 63) // 64) and tuple(v_i8t.shape) == (B, H, D, Np)
    got = v_i8t.cpu().numpy()
    assert np.array_equal(bits(v_scale.cpu().numpy()), bits(vs)), "v_scale differs"
    assert np.array_equal(got[..., :N], vq.transpose(0, 1, 3, 2)), "v_i8t differs"
    assert not got[..., N:].any(), "padding of v_i8t is not zero"
    return (v_i8t, v_scale), (vq, vs)


def assert_pv8_close(o_gpu, o_ref, l_ref, vs, what):
    """The bar of the FP16-product kernels (max-abs 2e-3, cosine 0.9999), except that a code of P~ may
    fall on the other side of a rounding boundary in the two implementations (the decision hangs on the
    last bits of an fp32 exponential): such an element may be off by up to two codes of one key,
    2 * delta_V[c] / l, and at most one element in 100 000 may need that allowance."""
    a = o_gpu.astype(np.float64); b = o_ref.astype(np.float64)
    assert np.all(np.isfinite(a)), f"{what}: non-finite output"
    diff = np.abs(a - b)
    tol = ABS_TOL + 2.0 * vs[..., None, :].astype(np.float64) / l_ref[..., :, None].astype(np.float64)
    worst = float((diff - tol).max())
    assert worst <= 0.0, f"{what}: an element is {worst:.3e} beyond 2e-3 + two codes"
    beyond = int(np.count_nonzero(diff > ABS_TOL))
    frac = 1.0 - beyond / diff.size
    assert beyond <= diff.size // 100000, f"{what}: {beyond} of {diff.size} elements beyond {ABS_TOL} (only {frac:.6f} within)"
    cos = float((a * b).sum() / (np.sqrt((a * a).sum()) * np.sqrt((b * b).sum())))
    assert cos >= COS_TOL, f"{what}: cosine {cos:.7f} < {COS_TOL}"
    return float(diff.max()), cos, frac


def run_and_compare(w, block_q, block_k, what, v_seed=None, qkv=None):
    q, k, v = si.full(w) if qkv is None else qkv
    if v_seed is not None:
        v = channel_scaled(v, v_seed)
    (q_i8, q_scale, k_i8, k_scale, _), (qq, qs, kq, ks, _) = assert_prepass_bit_exact(q, k, w.sm_scale, block_q, block_k)
    (v_i8t, v_scale), (vq, vs) = assert_v_quant_bit_exact(v)
    o_gpu = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, w.causal, w.sm_scale,
                                       block_q, block_k)
    torch.cuda.synchronize()
    o_ref, l_ref = oracle.attn_pv8(qq, qs, kq, ks, vq, vs, w.causal, 128, 64,
                                   gran_q=block_q, gran_k=block_k, return_l=True)
    return assert_pv8_close(o_gpu.cpu().numpy(), o_ref, l_ref, vs, what)


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_small_workloads_vb_parity(w):
    print(f"[case] INT8 PV, per-block {w.name} B{w.B} H{w.H} N{w.N} D{w.D} causal={w.causal}", flush=True)
    err, cos, frac = run_and_compare(w, 128, 64, w.name)
    print(f"  max_abs {err:.2e} cos {cos:.7f} within 2e-3: {frac:.5f}", flush=True)


@pytest.mark.parametrize("w", SMALL[1:5] + SMALL[7:], ids=lambda w: w.name)
def test_small_workloads_vt_parity(w):
    print(f"[case] INT8 PV, per-token {w.name} B{w.B} H{w.H} N{w.N} D{w.D} causal={w.causal}", flush=True)
    err, cos, frac = run_and_compare(w, 1, 1, w.name)
    print(f"  max_abs {err:.2e} cos {cos:.7f} within 2e-3: {frac:.5f}", flush=True)


@pytest.mark.parametrize("D,causal", [(128, True), (64, False)])
def test_channel_scaled_v_parity(D, causal):
    print(f"[case] INT8 PV, V channels spread over 1.5 decades D{D} causal={causal}", flush=True)
    w = si.custom("v_channels", 1, 2, 700, D, causal, 128, 64, seed=si.BASE_SEED + 70 + D)
    run_and_compare(w, 128, 64, w.name, v_seed=5 + D)


@pytest.mark.parametrize("D,causal,bq,bk", [(128, False, 128, 64), (64, True, 128, 64), (128, True, 1, 1)])
def test_token_outliers_parity(D, causal, bq, bk):
    # a few tokens 12x larger: large block scales, so that one unit of an integer score is a large
    # step of the softmax argument and rows are sharply peaked (small l: every code counts)
    print(f"[case] INT8 PV, outlier tokens D{D} causal={causal} scales {bq}x{bk}", flush=True)
    w = si.custom("outlier_tokens", 1, 2, 900, D, causal, 128, 64, seed=si.BASE_SEED + 80 + D)
    err, cos, frac = run_and_compare(w, bq, bk, w.name, qkv=with_token_outliers(w))
    print(f"  max_abs {err:.2e} cos {cos:.7f} within 2e-3: {frac:.5f}", flush=True)


def test_causal_first_row_is_the_dequantized_v0():
    # code 127 on key 0 only, l = 1: the first output row is delta_V V^[0] rounded to fp16
    w = si.custom("row0", 1, 2, 200, 64, True, 128, 64, seed=si.BASE_SEED + 75)
    q, k, v = si.full(w)
    q_i8, q_scale = sage.sage_quant_q(to_dev(q), w.sm_scale, 128)
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(to_dev(k), 64)
    v_i8t, v_scale = sage.sage_quant_v(to_dev(v))
    o = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, True, w.sm_scale, 128, 64)
    torch.cuda.synchronize()
    want = v_i8t[:, :, :, 0].cpu().numpy().astype(np.float64) * v_scale.cpu().numpy().astype(np.float64)
    got = o[:, :, 0, :].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= 2.0 ** -11 * np.abs(want) + 1e-6)


def test_int32_accumulator_is_flushed_periodically_when_the_maximum_never_changes():
    # key 0 wins every row by a margin (channel 0 of Q is a constant 16, of K it is 3 at token 0 and 0
    # elsewhere), so no row raises its maximum after the first tile; with 1094 key tiles the kernel's
    # periodic flush (every 1024 tiles, against int32 overflow) is the only flush that runs
    w = si.custom("flat_max", 1, 1, 70000, 64, False, 128, 64, seed=si.BASE_SEED + 90)
    print(f"[case] INT8 PV periodic flush N{w.N} D{w.D}", flush=True)
    q, k, v = si.full(w)
    g = np.random.default_rng(90)
    k = (g.standard_normal(k.shape) * 0.5).astype(np.float16)
    q[..., 0] = 16.0
    k[..., 0] = 0.0
    k[..., 0, 0] = 3.0
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(kd, 64)
    q_i8, q_scale = sage.sage_quant_q(qd, w.sm_scale, 128)
    v_i8t, v_scale = sage.sage_quant_v(vd)
    o = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, False, w.sm_scale, 128, 64)
    torch.cuda.synchronize()
    kq, ks, _ = oracle.smooth_quant_k(k, 64)
    qq, qs = oracle.quant_q(q, w.sm_scale, 128)
    vq, vs = oracle.quant_v(v)
    Tm = (w.N + 127) // 128
    blocks = [0, Tm // 2, Tm - 1]
    ref, l_ref = oracle.attn_pv8_slab(qq[0, 0], qs[0, 0], kq[0, 0], ks[0, 0], vq[0, 0], vs[0, 0], False, 128, 64,
                                      q_blocks=blocks, return_l=True)
    rows = np.concatenate([np.arange(i * 128, min(w.N, (i + 1) * 128)) for i in blocks])
    # the premise: the running maximum of these rows is the score of key 0 (first tile) -- then
    # 127 P~ of key 0 is 127 and l >= 1 is small because every other key is far below
    s0 = oracle.qk_i32(qq[0, 0], kq[0, 0], 0, 128)
    assert np.all(s0.argmax(axis=1) == 0)
    err, cos, frac = assert_pv8_close(o[0, 0].cpu().numpy()[rows], ref[rows], l_ref[rows], vs[0, 0], "flat_max")
    print(f"  max_abs {err:.2e} cos {cos:.7f} within 2e-3: {frac:.5f}; l in [{l_ref[rows].min():.2f}, {l_ref[rows].max():.2f}]", flush=True)


# cfg5 (2048 key tiles per row) also exercises the periodic flush of the int32 accumulator: late rows go
# more than 1024 tiles without a new maximum
FULL = [("cfg3_prefill16k", 5), ("cfg4_video", 4), ("cfg5_prefill128k", 4)]


@pytest.mark.parametrize("name,n_blocks", FULL, ids=[c[0] for c in FULL])
def test_full_size_vb_parity(name, n_blocks):
    w = si.WORKLOADS[name]
    t0 = time.time()
    print(f"[case] INT8 PV full size {name} B{w.B} H{w.H} N{w.N} D{w.D} causal={w.causal}", flush=True)
    q, k, v = si.full(w)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(kd, w.block_k)
    q_i8, q_scale = sage.sage_quant_q(qd, w.sm_scale, w.block_q)
    v_i8t, v_scale = sage.sage_quant_v(vd)
    o = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, w.causal, w.sm_scale,
                                   w.block_q, w.block_k)
    torch.cuda.synchronize()
    print(f"  gpu done {time.time() - t0:.1f}s", flush=True)
    vq, vs = oracle.quant_v(v)
    got = v_i8t.cpu().numpy()
    assert np.array_equal(bits(v_scale.cpu().numpy()), bits(vs))
    assert np.array_equal(got[..., :w.N], vq.transpose(0, 1, 3, 2)) and not got[..., w.N:].any()
    print(f"  V quantizer bit-exact {time.time() - t0:.1f}s", flush=True)
    Tm = (w.N + w.block_q - 1) // w.block_q
    g = np.random.default_rng(7)
    for b, h in [(0, 0), (w.B - 1, w.H - 1)]:
        kq, ks, _ = oracle.smooth_quant_k(k[b:b + 1, h:h + 1], w.block_k)
        qq, qs = oracle.quant_q(q[b:b + 1, h:h + 1], w.sm_scale, w.block_q)
        blocks = sorted({0, Tm - 1, Tm // 2} | {int(x) for x in g.integers(0, Tm, n_blocks - 3)})
        ref, l_ref = oracle.attn_pv8_slab(qq[0, 0], qs[0, 0], kq[0, 0], ks[0, 0], vq[b, h], vs[b, h], w.causal,
                                          w.block_q, w.block_k, q_blocks=blocks, return_l=True)
        rows = np.concatenate([np.arange(i * w.block_q, min(w.N, (i + 1) * w.block_q)) for i in blocks])
        err, cos, frac = assert_pv8_close(o[b, h].cpu().numpy()[rows], ref[rows], l_ref[rows], vs[b, h],
                                          f"{name} head ({b},{h}) blocks {blocks}")
        print(f"  head ({b},{h}) blocks {blocks}: max_abs {err:.2e} cos {cos:.7f} within 2e-3: {frac:.5f}"
              f"  {time.time() - t0:.1f}s", flush=True)


@pytest.mark.parametrize("pv8", [True, False], ids=["int8_pv", "fp16_pv"])
def test_a_cliff_in_the_scores_leaves_finite_exact_results(pv8):
    # the first 64 keys score about -400 (natural units) for every query, all later keys about 0: the
    # running maximum rises by about 577 in log2 units between the first and the second tile, far
    # beyond what exp2 can represent; the earlier accumulation must vanish, not overflow
    w = si.custom("cliff", 1, 2, 400, 64, False, 128, 64, seed=si.BASE_SEED + 95)
    print(f"[case] score cliff, int8_pv={pv8}", flush=True)
    q, k, v = si.full(w)
    g = np.random.default_rng(95)
    k = (g.standard_normal(k.shape) * 0.5).astype(np.float16)
    q[..., 0] = 40.0
    k[..., 0] = 40.0
    k[..., :64, 0] = -40.0
    (q_i8, q_scale, k_i8, k_scale, _), (qq, qs, kq, ks, _) = assert_prepass_bit_exact(q, k, w.sm_scale, 128, 64)
    s = oracle.qk_i32(qq[0, 0], kq[0, 0], 0, 4).astype(np.float64) * qs[0, 0, 0]
    assert (s[:, 64:] * ks[0, 0, 1]).max() - (s[:, :64] * ks[0, 0, 0]).max() > 300.0      # the premise
    if pv8:
        (v_i8t, v_scale), (vq, vs) = assert_v_quant_bit_exact(v)
        o = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, False, w.sm_scale, 128, 64)
        torch.cuda.synchronize()
        o_ref, l_ref = oracle.attn_pv8(qq, qs, kq, ks, vq, vs, False, 128, 64, return_l=True)
        assert_pv8_close(o.cpu().numpy(), o_ref, l_ref, vs, "cliff")
    else:
        from gpu_util import assert_output_close
        o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), False, w.sm_scale, 128, 64)
        torch.cuda.synchronize()
        assert_output_close(o.cpu().numpy(), oracle.attn_l2(qq, qs, kq, ks, v, False, 128, 64), "cliff")


@pytest.mark.parametrize("causal", [False, True])
def test_all_zero_blocks_give_uniform_attention_over_the_dequantized_v(causal):
    # K constant over tokens (smoothed K = 0: zero codes, zero scales) and one all-zero block of Q:
    # every visible key gets code 127, O = (prefix) mean of delta_V V^
    w = si.custom("zeros", 1, 2, 300, 128, causal, 128, 64, seed=si.BASE_SEED + 96)
    print(f"[case] INT8 PV zero blocks causal={causal}", flush=True)
    q, k, v = si.full(w)
    k[...] = k[:, :, :1, :]
    q[:, :, 128:256, :] = 0
    (q_i8, q_scale, k_i8, k_scale, _), (qq, qs, kq, ks, _) = assert_prepass_bit_exact(q, k, w.sm_scale, 128, 64)
    assert not kq.any() and not ks.any() and qs[0, 0, 1] == 0.0
    (v_i8t, v_scale), (vq, vs) = assert_v_quant_bit_exact(v)
    o = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal, w.sm_scale, 128, 64)
    torch.cuda.synchronize()
    deq = vq.astype(np.float64) * vs[:, :, None, :].astype(np.float64)
    want = np.cumsum(deq, 2) / np.arange(1, 301)[None, None, :, None] if causal else np.broadcast_to(deq.mean(2, keepdims=True), deq.shape)
    assert np.abs(o.cpu().numpy().astype(np.float64) - want).max() <= 2e-3
    o_ref, l_ref = oracle.attn_pv8(qq, qs, kq, ks, vq, vs, causal, 128, 64, return_l=True)
    assert_pv8_close(o.cpu().numpy(), o_ref, l_ref, vs, "zeros")
