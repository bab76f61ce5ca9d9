"""GPU parity: libsage (through its C ABI) against the CPU oracle on the same seeded inputs.

Bit-exact: INT8 tensors, scales, K mean, int32 scores.  Output: max-abs <= 2e-3 and cosine >= 0.9999
against the oracle's Algorithm-1 level (which emulates the same quantization)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import ABS_TOL, assert_output_close, assert_prepass_bit_exact, bits, to_dev, with_token_outliers

pytestmark = pytest.mark.gpu

SMALL = [
    si.WORKLOADS["cfg1_tiny"],
    si.custom("ragged_d128", 1, 3, 333, 128, False, 128, 64, seed=si.BASE_SEED + 11),
    si.custom("ragged_d64_causal", 2, 2, 457, 64, True, 128, 64, seed=si.BASE_SEED + 12),
    si.custom("causal_d128", 1, 2, 640, 128, True, 128, 64, k_noise=1.0, k_bias=4.0, outlier_frac=0.01,
              outlier_gain=8.0, seed=si.BASE_SEED + 13),
    si.custom("blocks_64_128", 1, 2, 300, 64, True, 64, 128, seed=si.BASE_SEED + 14),
    si.custom("blocks_32_64", 1, 1, 200, 128, False, 32, 64, seed=si.BASE_SEED + 15),
    si.custom("one_token", 1, 1, 1, 64, True, 128, 64, seed=si.BASE_SEED + 16),
    si.custom("short", 2, 1, 31, 128, False, 128, 64, seed=si.BASE_SEED + 17),
    si.custom("blocks_64_128_d128", 1, 2, 700, 128, True, 64, 128, seed=si.BASE_SEED + 18),
    si.custom("whole_tiles", 2, 2, 512, 128, False, 128, 64, seed=si.BASE_SEED + 19),
    si.custom("one_short_of_a_tile", 1, 2, 255, 64, True, 128, 64, seed=si.BASE_SEED + 21),
    si.custom("one_past_a_tile", 1, 2, 257, 128, True, 128, 64, seed=si.BASE_SEED + 22),
    # 512 tokens is the last size whose K pre-pass runs as a single launch, 513 the first that does not
    si.custom("single_launch_limit", 1, 3, 513, 64, False, 128, 64, seed=si.BASE_SEED + 23),
    si.custom("single_launch_blocks_128", 2, 2, 500, 128, False, 128, 128, seed=si.BASE_SEED + 25),
    si.custom("two_launch_blocks_128", 1, 2, 2049, 128, True, 128, 128, seed=si.BASE_SEED + 24),
    si.custom("blocks_32", 1, 2, 700, 64, True, 32, 64, seed=si.BASE_SEED + 26),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_small_workloads_full_parity(w):
    print(f"[case] {w.name} B{w.B} H{w.H} N{w.N} D{w.D} causal={w.causal} blocks {w.block_q}x{w.block_k}", flush=True)
    q, k, v = si.full(w)
    (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km) = assert_prepass_bit_exact(
        q, k, w.sm_scale, w.block_q, w.block_k)
    # int32 scores through the attention kernel's MFMA path, in both workgroup shapes the kernel is
    # built in (4 and 8 wavefronts) and in the one the launcher picks for this shape
    s_ref = [[oracle.qk_i32(qq[b, h], kq[b, h]) for h in range(w.H)] for b in range(w.B)]
    for wg_rows in (128, 256, 0):
        s_gpu = sage.sage_attn_qk_i32_debug(q_i8, k_i8, block_q=w.block_q, block_k=w.block_k, wg_rows=wg_rows)
        torch.cuda.synchronize()
        s_gpu = s_gpu.cpu().numpy()
        for b in range(w.B):
            for h in range(w.H):
                assert np.array_equal(s_gpu[b, h], s_ref[b][h]), f"int32 scores differ (workgroup rows {wg_rows})"
    # output
    o_gpu = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), w.causal, w.sm_scale, w.block_q, w.block_k)
    torch.cuda.synchronize()
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, w.causal, w.block_q, w.block_k)
    assert_output_close(o_gpu.cpu().numpy(), o_ref, w.name)


def test_causal_first_row_is_v0_bit_exact_and_constant_k_gives_prefix_means():
    print("[case] causal row 0 / constant K", flush=True)
    N, D = 300, 64
    g = np.random.default_rng(5)
    q = g.standard_normal((1, 1, N, D)).astype(np.float16)
    v = g.standard_normal((1, 1, N, D)).astype(np.float16)
    k = np.tile(g.standard_normal((1, 1, 1, D)).astype(np.float16), (1, 1, N, 1))
    (q_i8, q_scale, k_i8, k_scale, k_mean), _ = assert_prepass_bit_exact(q, k, 0.125, 128, 64)
    assert int(k_i8.abs().max()) == 0 and float(k_scale.abs().max()) == 0.0     # all-zero blocks
    o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), True, 0.125, 128, 64).cpu().numpy()
    assert np.array_equal(bits(o[0, 0, 0]), bits(v[0, 0, 0]))
    prefix = np.cumsum(v[0, 0].astype(np.float64), 0) / np.arange(1, N + 1)[:, None]
    assert np.abs(o[0, 0].astype(np.float64) - prefix).max() <= ABS_TOL
    o_nc = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), False, 0.125, 128, 64).cpu().numpy()
    assert np.abs(o_nc[0, 0].astype(np.float64) - v[0, 0].astype(np.float64).mean(0)[None]).max() <= ABS_TOL


@pytest.mark.parametrize("D,causal", [(128, False), (128, True), (64, True)])
def test_scores_that_keep_rising_force_a_rescale_at_every_tile(D, causal):
    """Scores grow linearly with the key index (about 13 nats per 64-key tile), so the running
    maximum has to be raised -- and O, l rescaled -- at every tile a row visits."""
    print(f"[case] rising scores D{D} causal={causal}", flush=True)
    N = 1100
    g = np.random.default_rng(7 + D)
    u = g.standard_normal(D); u /= np.linalg.norm(u)
    t = (np.arange(N) - N / 2)[:, None]
    k = (t * 0.05 * u[None, :] + 0.01 * g.standard_normal((N, D))).astype(np.float16)[None, None]
    q = (4.0 * np.sqrt(D) * u[None, :] + 0.1 * g.standard_normal((N, D))).astype(np.float16)[None, None]
    v = g.standard_normal((1, 1, N, D)).astype(np.float16)
    sm = float(np.float32(1.0) / np.sqrt(np.float32(D)))
    (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km) = assert_prepass_bit_exact(q, k, sm, 128, 64)
    o_gpu = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), causal, sm, 128, 64)
    torch.cuda.synchronize()
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, causal, 128, 64)
    assert_output_close(o_gpu.cpu().numpy(), o_ref, f"rising_d{D}")
    # the construction does what it says: the last tile's scores exceed the first tile's by far
    s = oracle.qk_i32(qq[0, 0], kq[0, 0])[N - 1].astype(np.float64) * qs[0, 0, -1] * np.repeat(ks[0, 0], 64)[:N]
    assert s[-64:].max() - s[:64].max() > 100.0


@pytest.mark.parametrize("D,causal,bq,bk", [(128, True, 128, 64), (64, False, 128, 64), (128, False, 64, 128)])
def test_outlier_tokens_make_coarse_integer_scores_and_the_softmax_stays_exact(D, causal, bq, bk):
    """A few tokens 12x larger than the rest: the other tokens of their blocks get small codes, the
    product of the two scales is large, and one unit of S^ is a visible step of the softmax
    argument.  The kernel folds dequantization, the fp32 seed of the integer accumulator and the
    running maximum into one fma; that is only as exact as the oracle's two multiplications if the
    folded constant is exact."""
    print(f"[case] outlier tokens D{D} causal={causal} blocks {bq}x{bk}", flush=True)
    w = si.custom("outlier_tokens_b", 1, 2, 900, D, causal, bq, bk, seed=si.BASE_SEED + 60 + D)
    q, k, v = with_token_outliers(w)
    (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km) = assert_prepass_bit_exact(q, k, w.sm_scale, bq, bk)
    o_gpu = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), causal, w.sm_scale, bq, bk)
    torch.cuda.synchronize()
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, causal, bq, bk)
    assert_output_close(o_gpu.cpu().numpy(), o_ref, w.name)
    # the regime is the intended one: the largest product of scales is far above the usual 1e-4
    assert float(qs.max()) * float(ks.max()) > 0.02


def test_results_are_deterministic_run_to_run():
    print("[case] determinism", flush=True)
    w = si.custom("det", 1, 4, 1000, 128, True, 128, 64, seed=si.BASE_SEED + 20)
    q, k, v = si.full(w)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    outs = []
    for _ in range(3):
        k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(kd, w.block_k)
        q_i8, q_scale = sage.sage_quant_q(qd, w.sm_scale, w.block_q)
        o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, vd, True, w.sm_scale, w.block_q, w.block_k)
        outs.append([x.cpu().numpy().copy() for x in (k_i8, k_scale, k_mean, q_i8, q_scale, o)])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


def test_host_side_errors_leave_no_side_effects():
    print("[case] error paths", flush=True)
    q = torch.zeros((1, 1, 64, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(sage.SageError) as e:
        sage.sage_quant_q(q, 0.125, block_q=48)
    assert e.value.status == 3
    with pytest.raises(sage.SageError) as e:
        sage.sage_quant_q(q, float("nan"), block_q=64)
    assert e.value.status == 7
    q96 = torch.zeros((1, 1, 64, 96), dtype=torch.float16, device="cuda")
    with pytest.raises(sage.SageError) as e:
        sage.sage_quant_q(q96, 0.125, block_q=64)
    assert e.value.status == 3
    # a sequence long enough to need scratch for its partial column sums, and a workspace too small for them
    k_long = torch.zeros((1, 1, 1024, 64), dtype=torch.float16, device="cuda")
    assert sage.sage_smooth_quant_k_workspace(1, 1, 1024, 64) > 8
    ws = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(sage.SageError) as e:
        sage.sage_smooth_quant_k(k_long, 64, workspace=ws)
    assert e.value.status == 4
    torch.cuda.synchronize()


@pytest.mark.parametrize("N,block_k", [(300, 64), (3000, 64), (3000, 1)])
def test_k_mean_output_is_optional(N, block_k):
    """sage_smooth_quant_k with k_mean = NULL (straight through the C ABI): same codes and scales as with it,
    on the single-launch path for short sequences and on the two-launch path."""
    import ctypes
    w = si.custom("nomean", 2, 2, N, 128, False, seed=si.BASE_SEED + 60 + N)
    _, k, _ = si.full(w)
    kd = to_dev(k)
    k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(kd, block_k)
    lib = sage.load()
    B, H, D = w.B, w.H, w.D
    k_i8_b = torch.full_like(k_i8, 5)
    k_scale_b = torch.full_like(k_scale, -1.0)
    ws = torch.empty(max(lib.sage_smooth_quant_k_workspace(B, H, N, D), 16), dtype=torch.uint8, device="cuda")
    st = lib.sage_smooth_quant_k(ctypes.c_void_p(kd.data_ptr()), ctypes.c_void_p(k_i8_b.data_ptr()),
                                 ctypes.c_void_p(k_scale_b.data_ptr()), None, ctypes.c_void_p(ws.data_ptr()), ws.numel(),
                                 B, H, N, D, block_k, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    assert st == 0
    assert torch.equal(k_i8, k_i8_b) and torch.equal(k_scale.view(torch.int32), k_scale_b.view(torch.int32))
    kq, ks, km = oracle.smooth_quant_k(k, block_k)
    assert np.array_equal(k_i8_b.cpu().numpy(), kq) and np.array_equal(bits(k_mean.cpu().numpy()), bits(km))
