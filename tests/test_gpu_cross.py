"""GPU parity of sage_attn_cross_fwd (Nq queries against Nkv keys; end-aligned causal mask) against
the CPU oracle, through the C ABI: cross-attention shapes, decode-like shapes (few queries at the end
of a long sequence) and the cases that reduce to self-attention.  Pre-pass tensors bit-exact, output
max-abs <= 2e-3 and cosine >= 0.9999, as for the self-attention call."""
import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import assert_output_close, bits, to_dev

pytestmark = pytest.mark.gpu

# (name, B, H, Nq, Nkv, D, causal, block_q, block_k)
CASES = [
    ("text_to_image_cross", 2, 3, 1024, 77, 64, False, 128, 64),
    ("image_to_text_cross", 1, 2, 77, 1500, 128, False, 128, 64),
    ("decode_one_query", 2, 4, 1, 3000, 128, True, 128, 64),
    ("decode_one_query_nc", 2, 4, 1, 3000, 64, False, 128, 64),
    ("chunked_prefill_tail", 1, 2, 300, 1333, 128, True, 128, 64),
    ("chunked_prefill_d64", 2, 2, 257, 900, 64, True, 64, 64),
    ("chunk_crossing_tiles", 1, 2, 130, 131, 128, True, 128, 64),
    ("per_token_cross", 1, 2, 200, 700, 128, True, 1, 1),
    ("per_token_cross_d64", 1, 3, 333, 100, 64, False, 1, 1),
    ("long_queries_short_keys", 1, 2, 2500, 40, 128, False, 128, 64),
]


def make(name, B, H, Nq, Nkv, D, seed):
    wq = si.custom(name + "_q", B, H, Nq, D, False, seed=si.BASE_SEED + 700 + seed)
    wk = si.custom(name + "_k", B, H, Nkv, D, False, k_noise=1.0, k_bias=3.0, seed=si.BASE_SEED + 800 + seed)
    q, _, _ = si.full(wq)
    _, k, v = si.full(wk)
    return q, k, v, wq.sm_scale


@pytest.mark.parametrize("name,B,H,Nq,Nkv,D,causal,bq,bk", CASES, ids=[c[0] for c in CASES])
def test_cross_parity(name, B, H, Nq, Nkv, D, causal, bq, bk):
    print(f"[case] cross {name} B{B} H{H} Nq{Nq} Nkv{Nkv} D{D} causal={causal} scales {bq}x{bk}", flush=True)
    q, k, v, sm = make(name, B, H, Nq, Nkv, D, len(name))
    k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(to_dev(k), bk)
    q_i8, q_scale = sage.sage_quant_q(to_dev(q), sm, bq)
    o = sage.sage_attn_cross_fwd(q_i8, q_scale, k_i8, k_scale, to_dev(v), causal, sm, bq, bk)
    torch.cuda.synchronize()
    kq, ks, km = oracle.smooth_quant_k(k, bk)
    qq, qs = oracle.quant_q(q, sm, bq)
    assert np.array_equal(k_i8.cpu().numpy(), kq) and np.array_equal(q_i8.cpu().numpy(), qq)
    assert np.array_equal(bits(k_scale.cpu().numpy()), bits(ks)) and np.array_equal(bits(q_scale.cpu().numpy()), bits(qs))
    lq, lk = (128, 64) if bq == 1 else (max(bq, 64), max(bk, 64))
    o_ref = oracle.attn_l2_cross(qq, qs, kq, ks, v, causal, lq, lk, gran_q=bq, gran_k=bk)
    err, cos = assert_output_close(o.cpu().numpy(), o_ref, name)
    print(f"  max_abs {err:.2e} cos {cos:.7f}", flush=True)


@pytest.mark.parametrize("causal", [False, True])
def test_equal_lengths_give_the_self_attention_result_bit_for_bit(causal):
    w = si.custom("same", 2, 2, 457, 128, causal, seed=si.BASE_SEED + 750)
    q, k, v = si.full(w)
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(to_dev(k), 64)
    q_i8, q_scale = sage.sage_quant_q(to_dev(q), w.sm_scale, 128)
    vd = to_dev(v)
    a = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, vd, causal, w.sm_scale, 128, 64)
    b = sage.sage_attn_cross_fwd(q_i8, q_scale, k_i8, k_scale, vd, causal, w.sm_scale, 128, 64)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_causal_with_more_queries_than_keys_is_refused():
    q_i8 = torch.zeros((1, 1, 128, 64), dtype=torch.int8, device="cuda")
    k_i8 = torch.zeros((1, 1, 64, 64), dtype=torch.int8, device="cuda")
    sc = torch.ones((1, 1, 1), dtype=torch.float32, device="cuda")
    v = torch.zeros((1, 1, 64, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(sage.SageError) as e:
        sage.sage_attn_cross_fwd(q_i8, sc, k_i8, sc, v, True, 0.125, 128, 64)
    assert e.value.status == 3


# ------------------------------------------------------------------ the INT8 second product with two lengths

from test_gpu_pv_int8 import assert_pv8_close  # noqa: E402

PV8_CASES = [c for c in CASES if c[0] in ("text_to_image_cross", "image_to_text_cross", "decode_one_query",
                                          "chunked_prefill_tail", "chunked_prefill_d64", "chunk_crossing_tiles",
                                          "per_token_cross")]


@pytest.mark.parametrize("name,B,H,Nq,Nkv,D,causal,bq,bk", PV8_CASES, ids=[c[0] for c in PV8_CASES])
def test_cross_parity_int8_second_product(name, B, H, Nq, Nkv, D, causal, bq, bk):
    print(f"[case] INT8 PV cross {name} B{B} H{H} Nq{Nq} Nkv{Nkv} D{D} causal={causal} scales {bq}x{bk}", flush=True)
    q, k, v, sm = make(name, B, H, Nq, Nkv, D, len(name))
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(to_dev(k), bk)
    q_i8, q_scale = sage.sage_quant_q(to_dev(q), sm, bq)
    v_i8t, v_scale = sage.sage_quant_v(to_dev(v))
    o = sage.sage_attn_pv_int8_cross_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal, sm, bq, bk)
    torch.cuda.synchronize()
    kq, ks, _ = oracle.smooth_quant_k(k, bk)
    qq, qs = oracle.quant_q(q, sm, bq)
    vq, vs = oracle.quant_v(v)
    assert np.array_equal(v_i8t.cpu().numpy()[..., :Nkv], vq.transpose(0, 1, 3, 2))
    o_ref, l_ref = oracle.attn_pv8_cross(qq, qs, kq, ks, vq, vs, causal, 128, 64, gran_q=bq, gran_k=bk, return_l=True)
    err, cos, frac = assert_pv8_close(o.cpu().numpy(), o_ref, l_ref, vs, name)
    print(f"  max_abs {err:.2e} cos {cos:.7f} within 2e-3: {frac:.5f}", flush=True)


def test_int8_second_product_equal_lengths_give_the_self_attention_result_bit_for_bit():
    w = si.custom("same8", 2, 2, 457, 128, True, seed=si.BASE_SEED + 760)
    q, k, v = si.full(w)
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(to_dev(k), 64)
    q_i8, q_scale = sage.sage_quant_q(to_dev(q), w.sm_scale, 128)
    v_i8t, v_scale = sage.sage_quant_v(to_dev(v))
    a = sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, True, w.sm_scale, 128, 64)
    b = sage.sage_attn_pv_int8_cross_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, True, w.sm_scale, 128, 64)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
