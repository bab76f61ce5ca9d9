"""Pins for the oracle's RoPE producer (the operator Section 4.6 fuses the quantizer into):
a hand-worked example, special angles, an independent complex-number formulation in numpy fp64,
and the property that defines a rotary embedding (scores depend on relative position only)."""
import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tables(N, D, base=10000.0, offset=0):
    """Angles t * base^(-2c/D), the usual choice; cos and sin in fp32."""
    t = np.arange(offset, offset + N, dtype=np.float64)[:, None]
    w = base ** (-2.0 * np.arange(D // 2, dtype=np.float64) / D)[None, :]
    return np.cos(t * w).astype(np.float32), np.sin(t * w).astype(np.float32)


def test_hand_worked_example():
    rows = {}
    for line in open(os.path.join(GOLDEN, "rope_worked.txt")):
        if line.strip() and not line.startswith("#"):
            name, *vals = line.split()
            rows[name] = np.array([float(v) for v in vals])
    y = oracle.rope(rows["x"].astype(np.float16)[None], rows["cos"].astype(np.float32)[None], rows["sin"].astype(np.float32)[None])
    assert np.array_equal(y[0].astype(np.float64), rows["y"])


def test_zero_angle_is_the_identity_and_a_quarter_turn_swaps_the_halves():
    g = np.random.default_rng(1)
    x = g.standard_normal((3, 50, 16)).astype(np.float16)
    one, zero = np.ones((50, 8), np.float32), np.zeros((50, 8), np.float32)
    assert np.array_equal(oracle.rope(x, one, zero).view(np.uint16), x.view(np.uint16))
    q = oracle.rope(x, zero, one)
    assert np.array_equal(q[..., :8], -x[..., 8:]) and np.array_equal(q[..., 8:], x[..., :8])


def test_matches_complex_multiplication_in_fp64_to_half_an_fp16_ulp():
    g = np.random.default_rng(2)
    N, D = 300, 64
    x = (g.standard_normal((N, D)) * 3).astype(np.float16)
    cos, sin = tables(N, D)
    z = (x[:, :D // 2].astype(np.float64) + 1j * x[:, D // 2:].astype(np.float64)) * (cos.astype(np.float64) + 1j * sin.astype(np.float64))
    ref = np.concatenate([z.real, z.imag], axis=1)
    y = oracle.rope(x, cos, sin).astype(np.float64)
    ulp = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -14))) - 10), 2.0 ** -24)
    assert np.all(np.abs(y - ref) <= 0.5 * ulp * (1 + 1e-3) + 4 * 2.0 ** -24 * np.abs(x.astype(np.float64)).max())
    # pair norms survive the rotation up to the output rounding
    n_in = np.hypot(x[:, :D // 2].astype(np.float64), x[:, D // 2:].astype(np.float64))
    n_out = np.hypot(y[:, :D // 2], y[:, D // 2:])
    assert np.abs(n_out - n_in).max() <= 2.0 ** -10 * n_in.max()


def test_scores_depend_on_the_relative_position_only():
    g = np.random.default_rng(3)
    N, D = 40, 32
    q = g.standard_normal((N, D)).astype(np.float16); k = g.standard_normal((N, D)).astype(np.float16)
    c0, s0 = tables(N, D); c1, s1 = tables(N, D, offset=1000)
    a = oracle.rope(q, c0, s0).astype(np.float64) @ oracle.rope(k, c0, s0).astype(np.float64).T
    b = oracle.rope(q, c1, s1).astype(np.float64) @ oracle.rope(k, c1, s1).astype(np.float64).T
    assert np.abs(a - b).max() <= 0.05 and np.abs(a).max() > 5.0          # fp16 rounding of the rotated vectors only
    plain = q.astype(np.float64) @ k.astype(np.float64).T
    assert np.abs(np.diag(a) - np.diag(plain)).max() <= 0.05              # equal positions: no rotation left
    assert np.abs(a - plain).max() > 1.0                                   # ... and it is not a no-op elsewhere


def test_leading_dimensions_share_the_tables():
    g = np.random.default_rng(4)
    x = g.standard_normal((2, 3, 20, 8)).astype(np.float16)
    cos, sin = tables(20, 8)
    y = oracle.rope(x, cos, sin)
    for b in range(2):
        for h in range(3):
            assert np.array_equal(y[b, h].view(np.uint16), oracle.rope(x[b, h], cos, sin).view(np.uint16))
