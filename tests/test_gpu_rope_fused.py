"""GPU parity of the pre-pass with RoPE applied on the fly (Section 4.6: the quantizer fused into
the operator that produces Q and K) against the CPU oracle: oracle RoPE -> fp16 -> oracle pre-pass.
Everything is integer or single-rounded fp32 work, so every output is compared bit for bit; and the
fused calls must return exactly what the library's unfused calls return on the rotated tensors."""
import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import assert_output_close, bits, to_dev

pytestmark = pytest.mark.gpu


def tables(N, D, base=10000.0):
    t = np.arange(N, dtype=np.float64)[:, None]
    w = base ** (-2.0 * np.arange(D // 2, dtype=np.float64) / D)[None, :]
    return np.cos(t * w).astype(np.float32), np.sin(t * w).astype(np.float32)


CASES = [
    si.custom("rope_d64", 2, 2, 457, 64, True, 128, 64, seed=si.BASE_SEED + 71),
    si.custom("rope_d128", 1, 3, 333, 128, False, 128, 64, seed=si.BASE_SEED + 72),
    si.custom("rope_blocks_32_128", 1, 2, 300, 128, False, 32, 128, seed=si.BASE_SEED + 73),
    si.custom("rope_per_token", 2, 1, 700, 128, True, 1, 1, seed=si.BASE_SEED + 74),
    si.custom("rope_per_token_d64", 1, 2, 130, 64, False, 1, 1, seed=si.BASE_SEED + 75),
    si.custom("rope_one_token", 1, 1, 1, 64, True, 128, 64, seed=si.BASE_SEED + 76),
]


def check_fused_prepass(q, k, cos, sin, sm_scale, block_q, block_k):
    qd, kd, cd, sd = to_dev(q), to_dev(k), to_dev(cos), to_dev(sin)
    k_i8, k_scale, k_mean = sage.sage_rope_smooth_quant_k(kd, cd, sd, block_k)
    q_i8, q_scale = sage.sage_rope_quant_q(qd, cd, sd, sm_scale, block_q)
    torch.cuda.synchronize()
    q_rot, k_rot = oracle.rope(q, cos, sin), oracle.rope(k, cos, sin)
    kq, ks, km = oracle.smooth_quant_k(k_rot, block_k)
    qq, qs = oracle.quant_q(q_rot, sm_scale, block_q)
    assert np.array_equal(bits(k_mean.cpu().numpy()), bits(km)), "k_mean differs"
    assert np.array_equal(bits(k_scale.cpu().numpy()), bits(ks)), "k_scale differs"
    assert np.array_equal(k_i8.cpu().numpy(), kq), "k_i8 differs"
    assert np.array_equal(bits(q_scale.cpu().numpy()), bits(qs)), "q_scale differs"
    assert np.array_equal(q_i8.cpu().numpy(), qq), "q_i8 differs"
    return (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km), (q_rot, k_rot)


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_fused_rope_prepass_is_bit_exact_and_equals_the_unfused_calls(w):
    print(f"[case] {w.name} B{w.B} H{w.H} N{w.N} D{w.D} blocks {w.block_q}x{w.block_k}", flush=True)
    q, k, v = si.full(w)
    cos, sin = tables(w.N, w.D)
    dev, ref, (q_rot, k_rot) = check_fused_prepass(q, k, cos, sin, w.sm_scale, w.block_q, w.block_k)
    # the library's own unfused calls on the rotated fp16 tensors give the same bits
    k2 = sage.sage_smooth_quant_k(to_dev(k_rot), w.block_k)
    q2 = sage.sage_quant_q(to_dev(q_rot), w.sm_scale, w.block_q)
    torch.cuda.synchronize()
    for a, b in zip((dev[2], dev[3], dev[4], dev[0], dev[1]), (*k2, *q2)):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    # and the attention that follows agrees with the oracle's
    q_i8, q_scale, k_i8, k_scale, _ = dev
    qq, qs, kq, ks, _ = ref
    o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), w.causal, w.sm_scale, w.block_q, w.block_k)
    torch.cuda.synchronize()
    lq, lk = (128, 64) if w.block_q == 1 else (w.block_q, w.block_k)
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, w.causal, lq, lk, gran_q=w.block_q, gran_k=w.block_k)
    assert_output_close(o.cpu().numpy(), o_ref, w.name)


def test_rotation_is_really_applied():
    """Zero angles reproduce the unfused pre-pass of the unrotated tensors; real angles do not."""
    w = si.custom("rope_identity", 1, 2, 200, 64, False, 128, 64, seed=si.BASE_SEED + 77)
    q, k, v = si.full(w)
    one, zero = np.ones((w.N, w.D // 2), np.float32), np.zeros((w.N, w.D // 2), np.float32)
    a = sage.sage_rope_smooth_quant_k(to_dev(k), to_dev(one), to_dev(zero), 64)
    b = sage.sage_smooth_quant_k(to_dev(k), 64)
    cos, sin = tables(w.N, w.D)
    c = sage.sage_rope_smooth_quant_k(to_dev(k), to_dev(cos), to_dev(sin), 64)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))
    assert not torch.equal(a[0], c[0])


@pytest.mark.parametrize("name", ["cfg3_prefill16k", "cfg4_video"])
def test_fused_rope_prepass_full_size(name):
    w = si.WORKLOADS[name]
    print(f"[case] fused RoPE pre-pass {name} B{w.B} H{w.H} N{w.N} D{w.D}", flush=True)
    q, k, v = si.full(w)
    cos, sin = tables(w.N, w.D)
    check_fused_prepass(q, k, cos, sin, w.sm_scale, w.block_q, w.block_k)
