"""Seeded sweep over shapes the fixed cases do not name: sequence lengths around every tile and
block boundary, both head dimensions, causal or not, every scale granularity, with and without
RoPE in the pre-pass.  Each case goes through the C ABI and is compared with the oracle as in
test_gpu_parity.py (pre-pass bit for bit, output within the tolerance)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import assert_output_close, bits, to_dev
from test_gpu_pv_int8 import assert_pv8_close, assert_v_quant_bit_exact

pytestmark = pytest.mark.gpu

BOUNDARIES = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 319, 383, 384, 385,
              511, 512, 513, 575, 640, 767, 769, 1023, 1025, 1280, 1409]
GRANULARITIES = [(128, 64), (64, 64), (32, 128), (64, 128), (1, 1), (1, 64), (128, 1)]


def cases(n=36, seed=20241002):
    g = np.random.default_rng(seed)
    out = []
    for i in range(n):
        N = int(g.choice(BOUNDARIES)) if i % 3 else int(g.integers(1, 1500))
        D = int(g.choice([64, 128]))
        bq, bk = GRANULARITIES[int(g.integers(0, len(GRANULARITIES)))]
        out.append((i, int(g.integers(1, 3)), int(g.integers(1, 4)), N, D, bool(g.integers(0, 2)), bq, bk, bool(i % 4 == 0)))
    return out


@pytest.mark.parametrize("i,B,H,N,D,causal,bq,bk,rope", cases(),
                         ids=lambda v: str(int(v)) if isinstance(v, (bool, int)) else None)
def test_random_shape(i, B, H, N, D, causal, bq, bk, rope):
    print(f"[case] {i}: B{B} H{H} N{N} D{D} causal={causal} scales {bq}x{bk} rope={rope}", flush=True)
    w = si.custom(f"sweep{i}", B, H, N, D, causal, 128, 64, k_noise=1.0, k_bias=3.0, seed=si.BASE_SEED + 500 + i)
    q, k, v = si.full(w)
    if rope:
        t = np.arange(N, dtype=np.float64)[:, None] * (10000.0 ** (-2.0 * np.arange(D // 2, dtype=np.float64) / D))[None, :]
        cos, sin = np.cos(t).astype(np.float32), np.sin(t).astype(np.float32)
        k_i8, k_scale, k_mean = sage.sage_rope_smooth_quant_k(to_dev(k), to_dev(cos), to_dev(sin), bk)
        q_i8, q_scale = sage.sage_rope_quant_q(to_dev(q), to_dev(cos), to_dev(sin), w.sm_scale, bq)
        q, k = oracle.rope(q, cos, sin), oracle.rope(k, cos, sin)
    else:
        k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(to_dev(k), bk)
        q_i8, q_scale = sage.sage_quant_q(to_dev(q), w.sm_scale, bq)
    torch.cuda.synchronize()
    kq, ks, km = oracle.smooth_quant_k(k, bk)
    qq, qs = oracle.quant_q(q, w.sm_scale, bq)
    assert np.array_equal(bits(k_mean.cpu().numpy()), bits(km)), "k_mean differs"
    assert np.array_equal(bits(k_scale.cpu().numpy()), bits(ks)), "k_scale differs"
    assert np.array_equal(k_i8.cpu().numpy(), kq), "k_i8 differs"
    assert np.array_equal(bits(q_scale.cpu().numpy()), bits(qs)), "q_scale differs"
    assert np.array_equal(q_i8.cpu().numpy(), qq), "q_i8 differs"
    o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), causal, w.sm_scale, bq, bk)
    torch.cuda.synchronize()
    # loop blocks of the oracle: multiples of the scale blocks (their order of visiting keys does not
    # change the result beyond rounding; the scales are what is semantic)
    lq, lk = max(bq, 64) if bq != 1 else 128, max(bk, 64) if bk != 1 else 64
    o_ref = oracle.attn_l2(qq, qs, kq, ks, v, causal, lq, lk, gran_q=bq, gran_k=bk)
    assert_output_close(o.cpu().numpy(), o_ref, f"sweep{i}")
    # the same case with the INT8 second product (Section 4.3).  Its codes of P~ are relative to the
    # running maximum after each 64-key block of the loop, so the oracle's kv block is the kernel's
    # 64 whatever the granularity of the K scales.
    (v_i8t, v_scale), (vq, vs) = assert_v_quant_bit_exact(v)
    o8 = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal, w.sm_scale, bq, bk)
    torch.cuda.synchronize()
    o8_ref, l_ref = oracle.attn_pv8(qq, qs, kq, ks, vq, vs, causal, 128, 64, gran_q=bq, gran_k=bk, return_l=True)
    assert_pv8_close(o8.cpu().numpy(), o8_ref, l_ref, vs, f"sweep{i} INT8 PV")
