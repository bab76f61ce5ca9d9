"""Pins for the oracle's Algorithm-1 loop with Nq queries against Nk keys (cross-attention, decode).
The paper treats Nq = Nk only; nothing but the ranges changes, and the causal mask is aligned at the
end (query t is token t + Nk - Nq).  Expected values: an independent numpy fp64 evaluation, the
self-attention oracle on the cases that reduce to it, and closed forms."""
import numpy as np
import pytest

import oracle
from test_oracle_attention import rand_qkv


def brute(qq, dq_tok, kq, dk_tok, v, causal):
    Nq, Nk = qq.shape[0], kq.shape[0]
    s = (qq.astype(np.float64) @ kq.astype(np.float64).T) * dq_tok.astype(np.float64)[:, None] * dk_tok.astype(np.float64)[None, :]
    if causal:
        s = np.where(np.arange(Nk)[None, :] > (np.arange(Nq) + Nk - Nq)[:, None], -np.inf, s)
    p = np.exp(s - s.max(axis=1, keepdims=True))
    return (p / p.sum(axis=1, keepdims=True)) @ v.astype(np.float64)


@pytest.mark.parametrize("Nq,Nk,causal", [(1, 200, True), (1, 200, False), (77, 300, False), (130, 131, True), (300, 77, False)])
def test_cross_matches_the_numpy_definition(Nq, Nk, causal):
    g = np.random.default_rng(Nq * 1000 + Nk)
    D = 32
    qq = g.integers(-127, 128, (1, 1, Nq, D), dtype=np.int8); kq = g.integers(-127, 128, (1, 1, Nk, D), dtype=np.int8)
    dq = (g.uniform(0.2, 3.0, Nq) * 2e-3).astype(np.float32); dk = (g.uniform(0.2, 3.0, Nk) * 2e-3).astype(np.float32)
    v = g.standard_normal((1, 1, Nk, D)).astype(np.float16)
    ref = brute(qq[0, 0], dq, kq[0, 0], dk, v[0, 0], causal)
    o = oracle.attn_l2_cross(qq, dq[None, None], kq, dk[None, None], v, causal, 64, 32, gran_q=1, gran_k=1)[0, 0]
    assert np.abs(o.astype(np.float64) - ref).max() <= 1e-3 + 2.0 ** -11 * np.abs(ref).max()
    if causal and Nq > 1:
        # a mask aligned at the start instead of the end is far outside that
        wrong = np.where(np.arange(Nk)[None, :] > np.arange(Nq)[:, None], -np.inf,
                         (qq[0, 0].astype(np.float64) @ kq[0, 0].astype(np.float64).T) * dq[:, None] * dk[None, :])
        p = np.exp(wrong - wrong.max(axis=1, keepdims=True))
        assert np.abs((p / p.sum(1, keepdims=True)) @ v[0, 0].astype(np.float64) - ref).max() > 0.05


@pytest.mark.parametrize("causal", [False, True])
def test_equal_lengths_reproduce_the_self_attention_entry_bit_for_bit(causal):
    q, k, v = rand_qkv(5, 333, 64, k_bias=2.0)
    kq, ks, _ = oracle.smooth_quant_k(k[None, None], 64)
    qq, qs = oracle.quant_q(q[None, None], 0.125, 128)
    a = oracle.attn_l2(qq, qs, kq, ks, v[None, None], causal, 128, 64)
    b = oracle.attn_l2_cross(qq, qs, kq, ks, v[None, None], causal, 128, 64)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_the_last_rows_of_causal_self_attention_are_a_causal_cross_attention():
    # per-token Q scales, so that cutting rows off Q does not change the scales of the rest; a Q
    # block boundary at the cut, so that the loop visits the same kv blocks
    q, k, v = rand_qkv(6, 320, 64, k_bias=2.0)
    kq, ks, _ = oracle.smooth_quant_k(k[None, None], 64)
    qq, qs = oracle.quant_q(q[None, None], 0.125, 1)
    full = oracle.attn_l2(qq, qs, kq, ks, v[None, None], True, 64, 64, gran_q=1)
    tail = oracle.attn_l2_cross(np.ascontiguousarray(qq[:, :, 256:]), np.ascontiguousarray(qs[:, :, 256:]), kq, ks,
                                v[None, None], True, 64, 64, gran_q=1)
    assert np.array_equal(full[:, :, 256:].view(np.uint16), tail.view(np.uint16))
    # decode: one query at the end sees every key, causal or not
    one = [oracle.attn_l2_cross(np.ascontiguousarray(qq[:, :, 319:]), np.ascontiguousarray(qs[:, :, 319:]), kq, ks,
                                v[None, None], c, 64, 64, gran_q=1) for c in (True, False)]
    assert np.array_equal(one[0].view(np.uint16), one[1].view(np.uint16))
    assert np.abs(one[0].astype(np.float64) - full[:, :, 319:].astype(np.float64)).max() <= 2e-3


def test_constant_k_gives_the_mean_of_the_visible_values():
    g = np.random.default_rng(8)
    Nq, Nk, D = 40, 100, 32
    qq = g.integers(-127, 128, (1, 1, Nq, D), dtype=np.int8)
    kq = np.zeros((1, 1, Nk, D), np.int8)
    v = g.standard_normal((1, 1, Nk, D)).astype(np.float16)
    ones_q, ones_k = np.ones((1, 1, 1), np.float32), np.ones((1, 1, 4), np.float32)
    o = oracle.attn_l2_cross(qq, ones_q, kq, ones_k, v, True, 64, 32).astype(np.float64)[0, 0]
    vf = v[0, 0].astype(np.float64)
    want = np.stack([vf[:Nk - Nq + t + 1].mean(0) for t in range(Nq)])
    assert np.abs(o - want).max() <= 1e-3


# ------------------------------------------------------------------ the same for the INT8 second product

def test_pv8_cross_reduces_to_the_self_attention_entry_and_to_its_last_rows():
    q, k, v = rand_qkv(16, 320, 64, k_bias=2.0)
    kq, ks, _ = oracle.smooth_quant_k(k[None, None], 64)
    qq, qs = oracle.quant_q(q[None, None], 0.125, 1)
    vq, vs = oracle.quant_v(v[None, None])
    for causal in (False, True):
        a, la = oracle.attn_pv8(qq, qs, kq, ks, vq, vs, causal, 64, 64, gran_q=1, return_l=True)
        b, lb = oracle.attn_pv8_cross(qq, qs, kq, ks, vq, vs, causal, 64, 64, gran_q=1, return_l=True)
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16)) and np.array_equal(la, lb)
    tail, lt = oracle.attn_pv8_cross(np.ascontiguousarray(qq[:, :, 256:]), np.ascontiguousarray(qs[:, :, 256:]), kq, ks,
                                     vq, vs, True, 64, 64, gran_q=1, return_l=True)
    assert np.array_equal(a[:, :, 256:].view(np.uint16), tail.view(np.uint16)) and np.array_equal(la[:, :, 256:], lt)


def test_pv8_cross_matches_the_numpy_recursion():
    from test_oracle_pv8 import brute_pv8
    g = np.random.default_rng(31)
    Nq, Nk, D = 90, 210, 32
    qq = g.integers(-127, 128, (Nk, D), dtype=np.int8); kq = g.integers(-127, 128, (Nk, D), dtype=np.int8)
    vq = g.integers(-127, 128, (Nk, D), dtype=np.int8)
    dq = (g.uniform(0.2, 3.0, Nk) * 2e-3).astype(np.float32); dk = (g.uniform(0.2, 3.0, Nk) * 2e-3).astype(np.float32)
    dv = g.uniform(0.01, 0.1, D).astype(np.float32)
    # the numpy recursion on the full square problem; its last Nq rows are the causal cross problem when
    # the Q block boundaries coincide (Nk - Nq = 120 is not a multiple of 64: use Q blocks of 30 rows)
    ref, l_ref = brute_pv8(qq, dq, kq, dk, vq, dv, True, 30, 32)
    o, l = oracle.attn_pv8_cross(np.ascontiguousarray(qq[None, None, Nk - Nq:]), dq[None, None, Nk - Nq:], kq[None, None],
                                 dk[None, None], vq[None, None], dv[None, None], True, 30, 32, gran_q=1, gran_k=1, return_l=True)
    assert np.allclose(l[0, 0], l_ref[Nk - Nq:], rtol=1e-5)
    diff = np.abs(o[0, 0].astype(np.float64) - ref[Nk - Nq:])
    assert np.all(diff <= 1e-3 + 2.0 * dv[None, :] / l_ref[Nk - Nq:, None])
