"""Pins for the pre-pass half of the CPU oracle (mean(K), smoothing, per-block INT8 quantizer).

None of the expected values here comes from the oracle itself or from the GPU path: they are
closed forms, exact rational arithmetic, numpy's own fp16 conversion, invariants of the
definitions in Sections 3.2 and 4.2, and a hand-worked fixture."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ fp16 conversions

def _c_f16_to_f32(bits):
    import ctypes
    bits = np.ascontiguousarray(bits, np.uint16)
    out = np.empty(bits.shape, np.float32)
    oracle._L().sage_oracle_f16_to_f32(oracle._p(bits), oracle._p(out), ctypes.c_int64(bits.size))
    return out


def _c_f32_to_f16(x, truncate=0):
    import ctypes
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    oracle._L().sage_oracle_f32_to_f16(oracle._p(x), oracle._p(out), ctypes.c_int64(x.size), ctypes.c_int(truncate))
    return out


def test_f16_to_f32_all_bit_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = _c_f16_to_f32(bits)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite].view(np.uint32), ref[finite].view(np.uint32))
    assert np.all(np.isnan(got[np.isnan(ref)]))
    assert np.array_equal(got[np.isinf(ref)], ref[np.isinf(ref)])


def test_f32_to_f16_nearest_even_matches_numpy():
    g = np.random.default_rng(1)
    x = np.concatenate([
        g.standard_normal(200000).astype(np.float32),
        (g.standard_normal(50000) * 1e-6).astype(np.float32),       # subnormal fp16 range
        (g.standard_normal(50000) * 3e4).astype(np.float32),        # near the top of the range
        # exact half-way points between neighbouring fp16 values
        ((np.arange(2048, 4096, dtype=np.float32) + 0.5) / 1024.0).astype(np.float32),
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, -65520.0, 1e9, 2.0 ** -25, 2.0 ** -24 * 1.5], np.float32),
    ])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(_c_f32_to_f16(x, 0), ref)


def test_f32_to_f16_truncation_never_rounds_away_from_zero():
    g = np.random.default_rng(2)
    x = np.concatenate([g.random(100000, dtype=np.float32), (g.random(1000, dtype=np.float32) * 1e-6).astype(np.float32)])
    t = _c_f32_to_f16(x, 1).view(np.float16).astype(np.float32)
    assert np.all(t <= x)
    # the next fp16 value up is strictly above x
    up = np.nextafter(t.astype(np.float16), np.float16(np.inf)).astype(np.float32)
    assert np.all(up > x)


# ------------------------------------------------------------------ mean(K), Section 4.2

def _exact_mean_f32(k16):
    """mean over tokens with Python rationals, rounded once to fp32 via an exactly-rounded double."""
    N, D = k16.shape
    out = np.empty(D, np.float32)
    for c in range(D):
        tot = sum((Fraction(float(x)) for x in k16[:, c]), Fraction(0))
        # Fraction -> float is correctly rounded; the oracle divides in double then rounds to fp32.
        # For these sizes the double quotient is either exact or far from an fp32 tie, so one
        # correctly rounded fp32 value is the unique answer; compute it from the rational.
        q = tot / N
        out[c] = np.float32(float(q))
    return out


def test_k_mean_equals_exact_rational_mean():
    g = np.random.default_rng(3)
    for N, D in [(1, 4), (7, 5), (64, 8), (333, 16)]:
        k = (g.standard_normal((N, D)) * 4 + g.standard_normal(D) * 10).astype(np.float16)
        assert np.array_equal(oracle.k_mean(k).view(np.uint32), _exact_mean_f32(k).view(np.uint32))


def test_k_mean_is_exact_over_the_whole_fp16_range():
    # values that a floating-point running sum would lose: huge +/- pairs around tiny terms
    col = np.array([65504.0, 6e-8, -65504.0, 6e-8, 1.0, 2.0 ** -14, -1.0, 3e-7], np.float16)
    k = np.stack([col, col[::-1]], axis=1)
    ref = _exact_mean_f32(k)
    assert ref[0] != 0.0
    assert np.array_equal(oracle.k_mean(k).view(np.uint32), ref.view(np.uint32))


def test_k_mean_is_independent_of_token_order():
    g = np.random.default_rng(4)
    k = (g.standard_normal((4096, 8)) * 100).astype(np.float16)
    m0 = oracle.k_mean(k)
    for s in range(3):
        perm = np.random.default_rng(10 + s).permutation(k.shape[0])
        assert np.array_equal(oracle.k_mean(k[perm]).view(np.uint32), m0.view(np.uint32))


def test_k_mean_of_a_constant_column_is_that_constant():
    k = np.full((1000, 3), 0.3, np.float16)
    assert np.array_equal(oracle.k_mean(k), k[0].astype(np.float32))


def test_smoothed_k_is_one_fp32_subtraction_and_sums_to_about_zero():
    g = np.random.default_rng(5)
    N, D = 2048, 16
    k = (g.standard_normal((N, D)) * 0.5 + g.standard_normal(D) * 3).astype(np.float16)
    mean = oracle.k_mean(k)
    ks = oracle.smooth_k(k, mean)
    assert ks.dtype == np.float32
    assert np.array_equal(ks, k.astype(np.float32) - mean[None, :])          # numpy fp32 subtract, one rounding
    resid = np.abs(ks.astype(np.float64).sum(0))
    ulp = np.spacing(np.abs(k.astype(np.float32)).max())
    assert np.all(resid <= N * ulp)


def test_scale_q_is_one_fp32_multiplication():
    g = np.random.default_rng(6)
    q = g.standard_normal((100, 64)).astype(np.float16)
    s = np.float32(1.0) / np.sqrt(np.float32(128))
    assert np.array_equal(oracle.scale_q(q, float(s)), q.astype(np.float32) * s)


# ------------------------------------------------------------------ quantizer psi, Section 3.2

def _load_ties():
    xs, qs, ds = [], [], []
    for line in open(os.path.join(GOLDEN, "quant_ties.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b, c = line.split("|")
        xs.append([float(t) for t in a.split()]); qs.append([int(t) for t in b.split()]); ds.append(float(c))
    return np.array(xs, np.float32), np.array(qs, np.int8), np.array(ds, np.float32)


def test_quantizer_hand_worked_ties_fixture():
    x, q_exp, d_rows = _load_ties()
    q, delta = oracle.quant_per_block(x, 2)
    assert np.array_equal(q, q_exp)
    assert np.array_equal(delta, d_rows[::2])
    # the printed x/delta form agrees on this fixture (all products exact)
    q2, delta2 = oracle.quant_per_block(x, 2, oracle.QUANT_DIV)
    assert np.array_equal(q2, q_exp) and np.array_equal(delta2, delta)


@pytest.mark.parametrize("N,D,block", [(256, 64, 64), (300, 32, 128), (77, 8, 16), (5, 4, 64)])
def test_quantizer_invariants(N, D, block):
    g = np.random.default_rng(N + D)
    x = (g.standard_normal((N, D)) * g.uniform(0.01, 30)).astype(np.float32)
    q, delta = oracle.quant_per_block(x, block)
    assert q.dtype == np.int8 and q.min() >= -127 and q.max() <= 127           # never -128
    nb = (N + block - 1) // block
    assert delta.shape == (nb,)
    for gidx in range(nb):
        sl = slice(gidx * block, min(N, (gidx + 1) * block))
        amax = np.abs(x[sl]).max()
        # delta = max|A| / 127 (one fp32 division)
        assert delta[gidx] == np.float32(amax) / np.float32(127.0)
        # an element of the block reaches full scale
        assert np.abs(q[sl]).max() == 127
        # round trip: |x - delta*q| <= delta/2 (+ fp32 slack of the scaled product)
        err = np.abs(x[sl].astype(np.float64) - float(delta[gidx]) * q[sl].astype(np.float64))
        assert err.max() <= float(delta[gidx]) * (0.5 + 2.0 ** -12)
        # sign is preserved wherever the code is non-zero
        nz = q[sl] != 0
        assert np.all(np.sign(q[sl][nz]) == np.sign(x[sl][nz]))


def test_per_block_reduces_to_per_tensor_and_per_token():
    g = np.random.default_rng(9)
    x = g.standard_normal((48, 16)).astype(np.float32) * 3
    # block = N is the per-tensor quantizer: delta = max|A|/127, A^ = round(A/delta)
    q, d = oracle.quant_per_block(x, 48)
    assert d.shape == (1,) and d[0] == np.abs(x).max() / np.float32(127)
    ref = np.rint(x.astype(np.float64) / (np.abs(x).max().astype(np.float64) / 127.0))
    assert np.abs(q - ref).max() <= 1 and np.mean(q != ref) < 1e-2       # double vs fp32 ties only
    # block = 1 is the per-token quantizer
    q1, d1 = oracle.quant_per_block(x, 1)
    assert np.array_equal(d1, np.abs(x).max(1) / np.float32(127))
    assert np.all(np.abs(q1).max(1) == 127)


def test_all_zero_block_gives_zero_scale_and_codes():
    x = np.zeros((128, 8), np.float32); x[64:] = 1.0
    q, d = oracle.quant_per_block(x, 64)
    assert d[0] == 0.0 and np.all(q[:64] == 0) and np.all(q[64:] == 127)


def test_multiply_and_divide_forms_differ_rarely_and_by_one():
    g = np.random.default_rng(11)
    x = g.standard_normal((4096, 64)).astype(np.float32)
    qa, da = oracle.quant_per_block(x, 64)
    qb, db = oracle.quant_per_block(x, 64, oracle.QUANT_DIV)
    assert np.array_equal(da, db)
    diff = qa.astype(np.int32) - qb.astype(np.int32)
    assert np.abs(diff).max() <= 1 and np.mean(diff != 0) < 1e-3


def test_whole_tensor_prepass_equals_slab_by_slab():
    g = np.random.default_rng(12)
    B, H, N, D = 2, 3, 200, 16
    k = (g.standard_normal((B, H, N, D)) + g.standard_normal((B, H, 1, D)) * 3).astype(np.float16)
    q = g.standard_normal((B, H, N, D)).astype(np.float16)
    kq, ks, km = oracle.smooth_quant_k(k, 64)
    qq, qs = oracle.quant_q(q, 0.25, 128)
    for b in range(B):
        for h in range(H):
            mean = oracle.k_mean(k[b, h])
            a, d = oracle.quant_per_block(oracle.smooth_k(k[b, h], mean), 64)
            assert np.array_equal(km[b, h], mean) and np.array_equal(kq[b, h], a) and np.array_equal(ks[b, h], d)
            a, d = oracle.quant_per_block(oracle.scale_q(q[b, h], 0.25), 128)
            assert np.array_equal(qq[b, h], a) and np.array_equal(qs[b, h], d)
