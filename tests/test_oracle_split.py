"""Pins for the oracle of the INT8-second-product kernels with the keys cut into chunks
(oracle.attn_pv8_cross_split: Algorithm 1 with the second product of Section 4.3 on every chunk of
keys, then a merge by the chunks' shares of the softmax denominator).  The paper has no such split;
what fixes the result is (a) the recursion of Sections 3.1 / 4.3 per chunk and (b) the identity
softmax over all keys = sum over chunks of (chunk denominator / total denominator) x softmax over the chunk.

Expected values come from: an independent numpy fp64 evaluation (unnormalized partial sums, merged
in one expression), the unsplit oracle for one chunk, a closed form (constant K), and the exact
attention over the dequantized V with the error bound of the code rounding."""
import numpy as np
import pytest

import oracle


def scores(qq, dq, kq, dk, causal):
    Nq, Nk = qq.shape[0], kq.shape[0]
    s = (qq.astype(np.float64) @ kq.astype(np.float64).T) * dq.astype(np.float64)[:, None] * dk.astype(np.float64)[None, :]
    if causal:
        s = np.where(np.arange(Nk)[None, :] > np.arange(Nq)[:, None] + (Nk - Nq), -np.inf, s)
    return s


def brute_split(qq, dq, kq, dk, vq, dv, causal, bkv, starts):
    """Per row and chunk: running maximum over the chunk's kv blocks, codes round(127 exp(S - m)),
    UNNORMALIZED o_s = sum of code products / 127 * dv, l_s, m_s; merged as
    sum_s e^(m_s - M) o_s / sum_s e^(m_s - M) l_s.  Per-token scales; fp64 throughout."""
    Nq, Nk, D = qq.shape[0], kq.shape[0], vq.shape[1]
    s = scores(qq, dq, kq, dk, causal)
    ends = list(starts[1:]) + [Nk]
    out = np.zeros((Nq, D)); big_l = np.zeros(Nq)
    for i in range(Nq):
        parts = []
        for a, b in zip(starts, ends):
            m, l, o = -np.inf, 0.0, np.zeros(D)
            for c0 in range(a, b, bkv):
                blk = s[i, c0:min(c0 + bkv, b)]
                m_new = max(m, blk.max())
                if m_new == -np.inf:
                    continue
                alpha = np.exp(m - m_new)
                p = np.exp(blk - m_new)
                l = alpha * l + p.sum()
                o = alpha * o + (np.rint(127.0 * p) @ vq[c0:min(c0 + bkv, b)].astype(np.float64)) / 127.0 * dv.astype(np.float64)
                m = m_new
            parts.append((m, l, o))
        top = max(p[0] for p in parts)
        num = sum(np.exp(m - top) * o for m, l, o in parts)
        den = sum(np.exp(m - top) * l for m, l, o in parts)
        out[i] = num / den
        big_l[i] = den
    return out, big_l


def random_case(seed, Nq, Nk, D, shift_at=None):
    g = np.random.default_rng(seed)
    qq = g.integers(-127, 128, (Nq, D), dtype=np.int8); kq = g.integers(-127, 128, (Nk, D), dtype=np.int8)
    vq = g.integers(-127, 128, (Nk, D), dtype=np.int8)
    dq = (g.uniform(0.5, 1.5, Nq) * 6e-3).astype(np.float32); dk = (g.uniform(0.5, 1.5, Nk) * 6e-3).astype(np.float32)
    dv = g.uniform(0.01, 0.1, D).astype(np.float32)
    if shift_at is not None:           # keys from shift_at on spread twice as wide: the chunk maxima differ by units
        dk[shift_at:] *= 2.0
    return qq, dq, kq, dk, vq, dv


def as4(*xs):
    return [x[None, None] for x in xs]


@pytest.mark.parametrize("Nq,Nk,D,bkv,starts,causal", [
    (5, 200, 32, 32, [0, 64, 128], False),
    (40, 200, 32, 32, [0, 96, 160], True),
    (2, 130, 16, 64, [0, 64, 128], True),
    (70, 333, 32, 32, [0, 32, 256], False),
])
def test_split_matches_the_numpy_evaluation(Nq, Nk, D, bkv, starts, causal):
    qq, dq, kq, dk, vq, dv = random_case(500 + Nk, Nq, Nk, D, shift_at=starts[-1] - 16)
    ref, l_ref = brute_split(qq, dq, kq, dk, vq, dv, causal, bkv, starts)
    o, big_l = oracle.attn_pv8_cross_split(*as4(qq, dq, kq, dk, vq, dv), causal, 64, bkv, starts, gran_q=1, gran_k=1,
                                           return_l=True)
    o, big_l = o[0, 0].astype(np.float64), big_l[0, 0]
    assert np.allclose(big_l, l_ref, rtol=1e-5)
    # one code of one key is worth at most dv / L; the partial outputs pass through fp16
    tol = 1e-3 + 2.0 * dv[None, :] / l_ref[:, None] + 2.0 ** -10 * np.abs(ref)
    diff = np.abs(o - ref)
    assert np.all(diff <= tol)
    assert np.mean(diff <= 1e-3 + 2.0 ** -10 * np.abs(ref)) > 0.99
    # the chunk maxima really differ, so a merge without the exp(m_s - M) factors is far off
    s = scores(qq, dq, kq, dk, causal)
    ends = starts[1:] + [Nk]
    tops = np.stack([s[:, a:b].max(1) for a, b in zip(starts, ends)])
    assert np.median(tops.max(0) - tops.min(0)) > 1.0
    # and the split is NOT the unsplit kernel: codes relative to chunk maxima differ from codes
    # relative to the running maximum over all keys (same attention, different rounding)
    whole = oracle.attn_pv8_cross(*as4(qq, dq, kq, dk, vq, dv), causal, 64, bkv, gran_q=1, gran_k=1)[0, 0].astype(np.float64)
    assert np.abs(whole - ref).max() <= 0.2 and not np.array_equal(whole, o)


@pytest.mark.parametrize("causal", [False, True])
def test_one_chunk_is_the_unsplit_oracle_bit_for_bit(causal):
    qq, dq, kq, dk, vq, dv = random_case(77, 50, 190, 32)
    a = oracle.attn_pv8_cross(*as4(qq, dq, kq, dk, vq, dv), causal, 64, 32, gran_q=1, gran_k=1)
    b = oracle.attn_pv8_cross_split(*as4(qq, dq, kq, dk, vq, dv), causal, 64, 32, [0], gran_q=1, gran_k=1)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_constant_k_gives_the_mean_of_the_dequantized_v_whatever_the_chunks():
    # S = 0 everywhere -> P~ = 1, code 127 for every visible key, m_s = 0, l_s = visible keys of the chunk:
    # the merge must weight chunks by l_s (unequal chunk sizes: equal weights would be wrong)
    g = np.random.default_rng(5)
    Nq, Nk, D = 20, 300, 32
    qq = g.integers(-127, 128, (Nq, D), dtype=np.int8)
    kq = np.zeros((Nk, D), np.int8)
    v = g.standard_normal((Nk, D)).astype(np.float16)
    v[200:] += np.float16(3.0)           # the small last chunk has a different mean
    vq, vs = oracle.quant_v(v)
    deq = vq.astype(np.float64) * vs.astype(np.float64)
    dq = np.full(Nq, 1e-3, np.float32); dk = np.full(Nk, 1e-3, np.float32)
    for causal in (False, True):
        o = oracle.attn_pv8_cross_split(*as4(qq, dq, kq, dk, vq, vs), causal, 64, 32, [0, 32, 256], gran_q=1, gran_k=1)
        o = o[0, 0].astype(np.float64)
        if causal:
            want = np.stack([deq[:Nk - Nq + i + 1].mean(0) for i in range(Nq)])
        else:
            want = np.tile(deq.mean(0), (Nq, 1))
        assert np.abs(o - want).max() <= 2e-3
        equal_weights = (deq[:32].mean(0) + deq[32:256].mean(0) + deq[256:].mean(0)) / 3
        assert np.abs(equal_weights - deq.mean(0)).max() > 0.1


def test_split_is_within_the_code_rounding_of_the_exact_attention_over_the_dequantized_v():
    # |code / 127 - P~| <= 1 / 254 per key, relative to the chunk's own maximum: chunk s is off by at
    # most sum_j |deq V_jc| / (254 l_s), and the merge averages the chunks with weights w_s / sum w
    qq, dq, kq, dk, vq, dv = random_case(901, 30, 400, 32, shift_at=250)
    starts = [0, 128, 256]
    for causal in (False, True):
        o = oracle.attn_pv8_cross_split(*as4(qq, dq, kq, dk, vq, dv), causal, 64, 32, starts, gran_q=1, gran_k=1)
        o = o[0, 0].astype(np.float64)
        s = scores(qq, dq, kq, dk, causal)
        p = np.exp(s - s.max(1, keepdims=True))
        deq = vq.astype(np.float64) * dv.astype(np.float64)
        exact = (p @ deq) / p.sum(1, keepdims=True)
        bound = np.zeros_like(exact)
        for a, b in zip(starts, starts[1:] + [400]):
            visible = np.isfinite(s[:, a:b]).astype(np.float64)
            l_s = np.exp(s[:, a:b] - s[:, a:b].max(1, keepdims=True)).sum(1)
            share = p[:, a:b].sum(1) / p.sum(1)
            bound += share[:, None] * (visible @ np.abs(deq[a:b])) / (254.0 * l_s[:, None])
        diff = np.abs(o - exact)
        assert np.all(diff <= bound + 2e-3)
        assert diff.max() > 0.02 * bound.max()
