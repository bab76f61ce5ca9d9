"""Seeded synthetic inputs shaped like the paper's workloads (Table of real-shape speeds;
Section 4.2's description of K as a large per-channel bias shared by all tokens plus a small
token-wise signal).  This module holds no arithmetic of the method: it only draws tensors.
Tests, bench.py and smoke() feed the SAME arrays to the CPU oracle and to the GPU library.

Every (config, batch, head) slab has its own PCG64 stream, so a single slab of a large
configuration can be generated without the rest.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20241002


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    D: int
    causal: bool
    block_q: int
    block_k: int
    k_noise: float      # std of the token-wise part of K
    k_bias: float       # std of the per-(b,h,channel) bias added to every token of K
    outlier_frac: float  # fraction of channels multiplied by outlier_gain (at least one if > 0)
    outlier_gain: float
    seed: int

    @property
    def sm_scale(self) -> float:
        return float(np.float32(1.0) / np.sqrt(np.float32(self.D)))

    @property
    def ops(self) -> float:
        """Counted operations 4*B*H*N^2*D, halved when causal."""
        full = 4.0 * self.B * self.H * float(self.N) ** 2 * self.D
        return full / 2 if self.causal else full


WORKLOADS = {
    # small case the oracle finishes in seconds
    "cfg1_tiny": Workload("cfg1_tiny", 1, 2, 256, 64, False, 64, 64, 0.5, 3.0, 0.0, 1.0, BASE_SEED + 1),
    # diffusion-style image attention
    "cfg2_image": Workload("cfg2_image", 4, 32, 4096, 128, False, 128, 64, 0.5, 3.0, 0.0, 1.0, BASE_SEED + 2),
    # LLM prefill, the headline configuration
    "cfg3_prefill16k": Workload("cfg3_prefill16k", 1, 32, 16384, 128, True, 128, 64, 1.0, 4.0, 0.01, 8.0, BASE_SEED + 3),
    # video generation, N not a multiple of either block size
    "cfg4_video": Workload("cfg4_video", 2, 30, 17776, 64, False, 128, 64, 0.5, 3.0, 0.0, 1.0, BASE_SEED + 4),
    # long-context prefill
    "cfg5_prefill128k": Workload("cfg5_prefill128k", 1, 8, 131072, 128, True, 128, 64, 1.0, 4.0, 0.0, 1.0, BASE_SEED + 5),
    # the remaining shapes of the paper's real-shape speed table (short and mid-length sequences)
    "shape_llm_1536": Workload("shape_llm_1536", 4, 32, 1536, 128, True, 128, 64, 1.0, 4.0, 0.0, 1.0, BASE_SEED + 6),
    "shape_image_7285": Workload("shape_image_7285", 2, 32, 7285, 64, False, 128, 64, 0.5, 3.0, 0.0, 1.0, BASE_SEED + 7),
    "shape_image_1105": Workload("shape_image_1105", 4, 24, 1105, 64, False, 128, 64, 0.5, 3.0, 0.0, 1.0, BASE_SEED + 8),
    "shape_vit_197": Workload("shape_vit_197", 12, 64, 197, 64, False, 128, 64, 0.5, 3.0, 0.0, 1.0, BASE_SEED + 9),
}


def custom(name, B, H, N, D, causal, block_q=128, block_k=64, k_noise=0.5, k_bias=3.0,
           outlier_frac=0.0, outlier_gain=1.0, seed=BASE_SEED + 100) -> Workload:
    return Workload(name, B, H, N, D, bool(causal), block_q, block_k, k_noise, k_bias,
                    outlier_frac, outlier_gain, seed)


def _rng(w: Workload, b: int, h: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([w.seed, b, h])))


def slab(w: Workload, b: int, h: int):
    """(Q, K, V) of one (batch, head): fp16 arrays [N, D].  Draw order: Q, V, K noise, bias, outliers."""
    g = _rng(w, b, h)
    q = g.standard_normal((w.N, w.D), dtype=np.float32)
    v = g.standard_normal((w.N, w.D), dtype=np.float32)
    k = g.standard_normal((w.N, w.D), dtype=np.float32)
    k *= np.float32(w.k_noise)
    bias = (g.standard_normal(w.D, dtype=np.float32) * np.float32(w.k_bias)).astype(np.float32)
    k += bias[None, :]
    if w.outlier_frac > 0:
        n_out = max(1, int(round(w.outlier_frac * w.D)))
        ch = g.choice(w.D, size=n_out, replace=False)
        k[:, ch] *= np.float32(w.outlier_gain)
    return q.astype(np.float16), k.astype(np.float16), v.astype(np.float16)


def full(w: Workload):
    """(Q, K, V) as fp16 arrays [B, H, N, D]."""
    q = np.empty((w.B, w.H, w.N, w.D), np.float16)
    k = np.empty_like(q)
    v = np.empty_like(q)
    for b in range(w.B):
        for h in range(w.H):
            q[b, h], k[b, h], v[b, h] = slab(w, b, h)
    return q, k, v
