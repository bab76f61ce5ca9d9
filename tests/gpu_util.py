"""Helpers shared by the GPU parity tests: run the library on seeded inputs, run the oracle on the same."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2410_02367_amd as sage

ABS_TOL = 2e-3        # max |O_gpu - O_oracle| (project target for the fp16 output)
COS_TOL = 0.9999      # cosine similarity of the flattened outputs


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32 if a.dtype == np.float32 else np.uint16)


def with_token_outliers(w, gain=12.0, frac=0.03):
    """The workload's tensors with a few Q and K tokens scaled up.  Their blocks get large scales,
    the other tokens of those blocks small integer codes: one unit of an integer score is then a
    large step of the softmax argument, which any shortcut in the dequantization must survive."""
    import sage_inputs as si
    q, k, v = si.full(w)
    g = np.random.default_rng(w.seed + 1000)
    q = q.copy(); k = k.copy()
    for x in (q, k):
        hit = g.random(x.shape[:3]) < frac
        x[hit] = (x[hit].astype(np.float32) * gain).astype(np.float16)
    return q, k, v


def gpu_prepass(q, k, sm_scale, block_q, block_k):
    qd, kd = to_dev(q), to_dev(k)
    k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(kd, block_k)
    q_i8, q_scale = sage.sage_quant_q(qd, sm_scale, block_q)
    torch.cuda.synchronize()
    return q_i8, q_scale, k_i8, k_scale, k_mean


def assert_prepass_bit_exact(q, k, sm_scale, block_q, block_k):
    """Every INT8 code, scale and mean must equal the oracle's, bit for bit.  Returns device tensors."""
    q_i8, q_scale, k_i8, k_scale, k_mean = gpu_prepass(q, k, sm_scale, block_q, block_k)
    kq, ks, km = oracle.smooth_quant_k(k, block_k)
    qq, qs = oracle.quant_q(q, sm_scale, block_q)
    assert np.array_equal(bits(k_mean.cpu().numpy()), bits(km)), "k_mean differs"
    assert np.array_equal(bits(k_scale.cpu().numpy()), bits(ks)), "k_scale differs"
    assert np.array_equal(k_i8.cpu().numpy(), kq), "k_i8 differs"
    assert np.array_equal(bits(q_scale.cpu().numpy()), bits(qs)), "q_scale differs"
    assert np.array_equal(q_i8.cpu().numpy(), qq), "q_i8 differs"
    return (q_i8, q_scale, k_i8, k_scale, k_mean), (qq, qs, kq, ks, km)


def assert_output_close(o_gpu: np.ndarray, o_ref: np.ndarray, what=""):
    a = o_gpu.astype(np.float64); b = o_ref.astype(np.float64)
    assert np.all(np.isfinite(a)), f"{what}: non-finite output"
    err = np.abs(a - b).max()
    cos = float((a * b).sum() / (np.sqrt((a * a).sum()) * np.sqrt((b * b).sum())))
    assert err <= ABS_TOL, f"{what}: max abs err {err:.3e} > {ABS_TOL}"
    assert cos >= COS_TOL, f"{what}: cosine {cos:.7f} < {COS_TOL}"
    return err, cos
