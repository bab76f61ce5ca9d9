"""CPU oracle for the SageAttention forward pass -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end to ``sage_oracle.c`` (plain C written from the paper's Sections 3.1,
3.2, 4.1, 4.2, 4.4, 4.6 and Algorithm 1).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the GPU library never does, and the
two share no code.  All arrays are host numpy arrays; fp16 tensors are ``np.float16``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sage_oracle.c")
_LIB = os.path.join(_HERE, "libsage_oracle.so")

P_TRUNCATE = 1   # P~ -> fp16 by truncation instead of round-to-nearest-even
ACC_FP16 = 2     # emulate the fp16 accumulator Algorithm 1 names for P~V
QUANT_DIV = 4    # quantize as x / delta (the formula as printed) instead of x * fl32(127/amax)
L_FROM_P16 = 8   # accumulate the row sum l from the fp16-rounded P~


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, no fast-math) and return the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.sage_oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _f16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


def num_threads() -> int:
    return int(_L().sage_oracle_num_threads())


def nblocks(N: int, block: int) -> int:
    return (N + block - 1) // block


# ---------------------------------------------------------------- pre-pass pieces (one slab [N, D])

def k_mean(k: np.ndarray) -> np.ndarray:
    """mean(K) over tokens of one slab, exact sum then one fp32 rounding (Section 4.2)."""
    k = _f16(k); N, D = k.shape
    out = np.empty(D, np.float32)
    _L().sage_oracle_k_mean(_p(k), ctypes.c_int(N), ctypes.c_int(D), _p(out))
    return out


def smooth_k(k: np.ndarray, mean: np.ndarray) -> np.ndarray:
    """gamma(K) = K - mean(K) in fp32 (Section 4.2)."""
    k = _f16(k); N, D = k.shape
    mean = np.ascontiguousarray(mean, np.float32)
    out = np.empty((N, D), np.float32)
    _L().sage_oracle_smooth_k(_p(k), _p(mean), ctypes.c_int(N), ctypes.c_int(D), _p(out))
    return out


def scale_q(q: np.ndarray, sm_scale: float) -> np.ndarray:
    """Q * sm_scale in fp32 (Section 4.6)."""
    q = _f16(q); N, D = q.shape
    out = np.empty((N, D), np.float32)
    _L().sage_oracle_scale_q(_p(q), ctypes.c_float(sm_scale), ctypes.c_int(N), ctypes.c_int(D), _p(out))
    return out


def rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate-half RoPE of fp16 x [..., N, D] with fp32 tables cos, sin [N, D/2] -> fp16 (Section 4.6's producer)."""
    x = _f16(x); N, D = x.shape[-2:]
    cos = np.ascontiguousarray(cos, np.float32); sin = np.ascontiguousarray(sin, np.float32)
    assert D % 2 == 0 and cos.shape == (N, D // 2) and sin.shape == (N, D // 2)
    y = np.empty_like(x)
    xs, ys = x.reshape(-1, N, D), y.reshape(-1, N, D)
    for i in range(xs.shape[0]):
        _L().sage_oracle_rope(_p(xs[i]), _p(cos), _p(sin), ctypes.c_int(N), ctypes.c_int(D), _p(ys[i]))
    return y


def quant_per_block(x: np.ndarray, block: int, flags: int = 0):
    """Per-block INT8 quantizer psi of Section 3.2 on an fp32 [N, D] matrix -> (x_i8, delta)."""
    x = np.ascontiguousarray(x, np.float32); N, D = x.shape
    xq = np.empty((N, D), np.int8)
    delta = np.empty(nblocks(N, block), np.float32)
    _L().sage_oracle_quant_per_block(_p(x), ctypes.c_int(N), ctypes.c_int(D), ctypes.c_int(block),
                                     ctypes.c_uint(flags), _p(xq), _p(delta))
    return xq, delta


# ---------------------------------------------------------------- pre-pass on [B, H, N, D]

def smooth_quant_k(k: np.ndarray, block_k: int, flags: int = 0):
    """phi_K = psi_K o gamma on every (batch, head) slab -> (k_i8, k_scale, k_mean)."""
    k = _f16(k); B, H, N, D = k.shape
    kq = np.empty((B, H, N, D), np.int8)
    ks = np.empty((B, H, nblocks(N, block_k)), np.float32)
    km = np.empty((B, H, D), np.float32)
    _L().sage_oracle_smooth_quant_k(_p(k), *map(ctypes.c_int, (B, H, N, D, block_k)),
                                    ctypes.c_uint(flags), _p(kq), _p(ks), _p(km))
    return kq, ks, km


def quant_q(q: np.ndarray, sm_scale: float, block_q: int, flags: int = 0):
    """psi_Q(Q * sm_scale) on every slab -> (q_i8, q_scale)."""
    q = _f16(q); B, H, N, D = q.shape
    qq = np.empty((B, H, N, D), np.int8)
    qs = np.empty((B, H, nblocks(N, block_q)), np.float32)
    _L().sage_oracle_quant_q(_p(q), *map(ctypes.c_int, (B, H, N, D)), ctypes.c_float(sm_scale),
                             ctypes.c_int(block_q), ctypes.c_uint(flags), _p(qq), _p(qs))
    return qq, qs


# ---------------------------------------------------------------- attention

def qk_i32(qq: np.ndarray, kq: np.ndarray, row0: int = 0, nrows: int | None = None) -> np.ndarray:
    """Raw int32 scores Q^ K^^T of one slab for query rows [row0, row0+nrows)."""
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    N, D = kq.shape
    nrows = N - row0 if nrows is None else nrows
    assert 0 <= row0 and row0 + nrows <= qq.shape[0]
    s = np.empty((nrows, N), np.int32)
    _L().sage_oracle_qk_i32(_p(qq), _p(kq), *map(ctypes.c_int, (N, D, row0, nrows)), _p(s))
    return s


def attn_l2(qq, q_scale, kq, k_scale, v, causal: bool, block_q: int, block_k: int, flags: int = 0,
            gran_q: int | None = None, gran_k: int | None = None):
    """Algorithm 1 on whole [B, H, N, D] tensors -> fp16 output.

    gran_q / gran_k: tokens per scale of Q^ / K^ (default: the loop's block sizes, i.e. SAGEAttn-B;
    1 = the per-token quantizer of Section 3.2, i.e. SAGEAttn-T)."""
    gran_q = block_q if gran_q is None else gran_q
    gran_k = block_k if gran_k is None else gran_k
    v = _f16(v); B, H, N, D = v.shape
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    q_scale = np.ascontiguousarray(q_scale, np.float32); k_scale = np.ascontiguousarray(k_scale, np.float32)
    assert qq.shape == (B, H, N, D) and kq.shape == (B, H, N, D)
    assert q_scale.shape == (B, H, nblocks(N, gran_q)) and k_scale.shape == (B, H, nblocks(N, gran_k))
    o = np.zeros((B, H, N, D), np.float16)
    _L().sage_oracle_attn_l2_g(_p(qq), _p(q_scale), _p(kq), _p(k_scale), _p(v),
                               *map(ctypes.c_int, (B, H, N, D, int(causal), block_q, block_k, gran_q, gran_k)),
                               ctypes.c_uint(flags), _p(o))
    return o


def attn_l2_cross(qq, q_scale, kq, k_scale, v, causal: bool, block_q: int, block_k: int, flags: int = 0,
                  gran_q: int | None = None, gran_k: int | None = None):
    """Algorithm 1 with Nq queries against Nk keys: Q^ [B, H, Nq, D], K^ and V [B, H, Nk, D] -> fp16
    [B, H, Nq, D].  The causal mask is aligned at the end (query t is token t + Nk - Nq); it needs Nq <= Nk."""
    gran_q = block_q if gran_q is None else gran_q
    gran_k = block_k if gran_k is None else gran_k
    v = _f16(v); B, H, Nk, D = v.shape
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    Nq = qq.shape[2]
    q_scale = np.ascontiguousarray(q_scale, np.float32); k_scale = np.ascontiguousarray(k_scale, np.float32)
    assert qq.shape == (B, H, Nq, D) and kq.shape == (B, H, Nk, D) and (not causal or Nq <= Nk)
    assert q_scale.shape == (B, H, nblocks(Nq, gran_q)) and k_scale.shape == (B, H, nblocks(Nk, gran_k))
    o = np.zeros((B, H, Nq, D), np.float16)
    _L().sage_oracle_attn_l2_cross_g(_p(qq), _p(q_scale), _p(kq), _p(k_scale), _p(v),
                                     *map(ctypes.c_int, (B, H, Nq, Nk, D, int(causal), block_q, block_k, gran_q, gran_k)),
                                     ctypes.c_uint(flags), _p(o))
    return o


def attn_l2_slab(qq, q_scale, kq, k_scale, v, causal: bool, block_q: int, block_k: int,
                 q_blocks=None, flags: int = 0, gran_q: int | None = None, gran_k: int | None = None):
    """Algorithm 1 on one slab [N, D] for the listed Q blocks (all if None).

    Returns an fp16 [N, D] array; rows of blocks that were not requested are zero.
    gran_q / gran_k as in attn_l2."""
    gran_q = block_q if gran_q is None else gran_q
    gran_k = block_k if gran_k is None else gran_k
    v = _f16(v); N, D = v.shape
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    q_scale = np.ascontiguousarray(q_scale, np.float32); k_scale = np.ascontiguousarray(k_scale, np.float32)
    assert q_scale.shape == (nblocks(N, gran_q),) and k_scale.shape == (nblocks(N, gran_k),)
    o = np.zeros((N, D), np.float16)
    if q_blocks is None:
        blocks, nb = None, -1
    else:
        blocks = np.ascontiguousarray(q_blocks, np.int32); nb = len(blocks)
        assert nb == 0 or (blocks.min() >= 0 and blocks.max() < nblocks(N, block_q))
    _L().sage_oracle_attn_l2_slab_g(_p(qq), _p(q_scale), _p(kq), _p(k_scale), _p(v),
                                    *map(ctypes.c_int, (N, D, int(causal), block_q, block_k, gran_q, gran_k)),
                                    ctypes.c_uint(flags),
                                  _p(blocks) if blocks is not None else None, ctypes.c_int(nb), _p(o))
    return o


def quant_v(v: np.ndarray):
    """psi_V of Section 4.3: per-channel INT8 quantizer of V [..., N, D] (one scale per channel of every
    (batch, head) slab, over all tokens) -> (V^ int8 [..., N, D], delta_V float32 [..., D])."""
    v = _f16(v); N, D = v.shape[-2:]
    lead = v.shape[:-2]; S = int(np.prod(lead)) if lead else 1
    vq = np.zeros(v.shape, np.int8); sc = np.zeros(lead + (D,), np.float32)
    _L().sage_oracle_quant_v(_p(v), ctypes.c_int(1), ctypes.c_int(S), ctypes.c_int(N), ctypes.c_int(D),
                             _p(vq), _p(sc))
    return vq, sc


def attn_pv8(qq, q_scale, kq, k_scale, vq, v_scale, causal: bool, block_q: int, block_k: int,
             gran_q: int | None = None, gran_k: int | None = None, return_l: bool = False):
    """The kernels with an INT8 second product (Section 4.3; SAGEAttn-vB, or -vT with gran 1) on whole
    [B, H, N, D] tensors -> fp16 output (and, if asked, the final row sums l [B, H, N])."""
    gran_q = block_q if gran_q is None else gran_q
    gran_k = block_k if gran_k is None else gran_k
    vq = np.ascontiguousarray(vq, np.int8); B, H, N, D = vq.shape
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    q_scale = np.ascontiguousarray(q_scale, np.float32); k_scale = np.ascontiguousarray(k_scale, np.float32)
    v_scale = np.ascontiguousarray(v_scale, np.float32)
    assert qq.shape == (B, H, N, D) and kq.shape == (B, H, N, D) and v_scale.shape == (B, H, D)
    assert q_scale.shape == (B, H, nblocks(N, gran_q)) and k_scale.shape == (B, H, nblocks(N, gran_k))
    o = np.zeros((B, H, N, D), np.float16)
    lsum = np.zeros((B, H, N), np.float32)
    _L().sage_oracle_attn_pv8_g(_p(qq), _p(q_scale), _p(kq), _p(k_scale), _p(vq), _p(v_scale),
                                *map(ctypes.c_int, (B, H, N, D, int(causal), block_q, block_k, gran_q, gran_k)),
                                _p(o), _p(lsum))
    return (o, lsum) if return_l else o


def attn_pv8_cross(qq, q_scale, kq, k_scale, vq, v_scale, causal: bool, block_q: int, block_k: int,
                   gran_q: int | None = None, gran_k: int | None = None, return_l: bool = False,
                   return_m: bool = False):
    """attn_pv8 with Nq queries (Q^ [B, H, Nq, D]) against Nk keys (K^, V^ [B, H, Nk, D]); end-aligned causal mask.
    return_m: also the final row maxima m of Algorithm 1 [B, H, Nq] (implies return_l)."""
    gran_q = block_q if gran_q is None else gran_q
    gran_k = block_k if gran_k is None else gran_k
    vq = np.ascontiguousarray(vq, np.int8); B, H, Nk, D = vq.shape
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    Nq = qq.shape[2]
    q_scale = np.ascontiguousarray(q_scale, np.float32); k_scale = np.ascontiguousarray(k_scale, np.float32)
    v_scale = np.ascontiguousarray(v_scale, np.float32)
    assert qq.shape == (B, H, Nq, D) and kq.shape == (B, H, Nk, D) and v_scale.shape == (B, H, D)
    assert q_scale.shape == (B, H, nblocks(Nq, gran_q)) and k_scale.shape == (B, H, nblocks(Nk, gran_k))
    assert not causal or Nq <= Nk
    o = np.zeros((B, H, Nq, D), np.float16)
    lsum = np.zeros((B, H, Nq), np.float32)
    mrow = np.zeros((B, H, Nq), np.float32)
    _L().sage_oracle_attn_pv8_cross_g(_p(qq), _p(q_scale), _p(kq), _p(k_scale), _p(vq), _p(v_scale),
                                      *map(ctypes.c_int, (B, H, Nq, Nk, D, int(causal), block_q, block_k, gran_q, gran_k)),
                                      _p(o), _p(lsum), _p(mrow))
    if return_m:
        return o, lsum, mrow
    return (o, lsum) if return_l else o


def attn_pv8_cross_split(qq, q_scale, kq, k_scale, vq, v_scale, causal: bool, block_q: int, block_k: int,
                         starts, gran_q: int | None = None, gran_k: int | None = None, return_l: bool = False):
    """The INT8-second-product kernels with the keys of a slab cut into chunks (not in the paper: the
    decode-shape variant of the library).  Chunk s holds keys starts[s] .. starts[s+1]-1 (the last one
    up to Nk); Algorithm 1 with the second product of Section 4.3 runs on each chunk as if it were the
    whole key set -- own running maximum, hence own codes of P~ -- and leaves O_s (fp16), m_s, l_s;
    the partial results are merged by their shares of the softmax denominator,
        O = sum_s w_s O_s / sum_s w_s,   w_s = l_s exp(m_s - max_s m_s)      (fp64, rounded to fp16).
    starts must be multiples of gran_k (and of block_k), increasing from 0, and with a causal mask the
    last start must not exceed Nk - Nq: then all chunks but the last are fully visible to every query
    and the last carries the end-aligned mask.  return_l: also L = sum_s w_s, the denominator relative
    to the global maximum [B, H, Nq]."""
    gran_q = block_q if gran_q is None else gran_q
    gran_k = block_k if gran_k is None else gran_k
    Nk, Nq = kq.shape[2], qq.shape[2]
    starts = [int(x) for x in starts]
    assert starts[0] == 0 and all(a < b for a, b in zip(starts, starts[1:])) and starts[-1] < Nk
    assert all(x % gran_k == 0 and x % block_k == 0 for x in starts)
    assert not causal or starts[-1] <= Nk - Nq
    ends = starts[1:] + [Nk]
    parts, ms, ls = [], [], []
    for s, (a, b) in enumerate(zip(starts, ends)):
        o_s, l_s, m_s = attn_pv8_cross(qq, q_scale, kq[:, :, a:b], k_scale[:, :, a // gran_k:nblocks(b, gran_k)],
                                       vq[:, :, a:b], v_scale, causal and s == len(starts) - 1, block_q, block_k,
                                       gran_q, gran_k, return_m=True)
        parts.append(o_s.astype(np.float64)); ms.append(m_s.astype(np.float64)); ls.append(l_s.astype(np.float64))
    top = np.max(np.stack(ms), axis=0)
    w = [l_s * np.exp(m_s - top) for l_s, m_s in zip(ls, ms)]
    total = np.sum(np.stack(w), axis=0)
    o = sum(w_s[..., None] * o_s for w_s, o_s in zip(w, parts)) / total[..., None]
    o = o.astype(np.float16)
    return (o, total.astype(np.float32)) if return_l else o


def attn_pv8_slab(qq, q_scale, kq, k_scale, vq, v_scale, causal: bool, block_q: int, block_k: int,
                  q_blocks=None, gran_q: int | None = None, gran_k: int | None = None, return_l: bool = False):
    """attn_pv8 on one slab [N, D] for the listed Q blocks (all if None); other rows stay zero."""
    gran_q = block_q if gran_q is None else gran_q
    gran_k = block_k if gran_k is None else gran_k
    vq = np.ascontiguousarray(vq, np.int8); N, D = vq.shape
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    q_scale = np.ascontiguousarray(q_scale, np.float32); k_scale = np.ascontiguousarray(k_scale, np.float32)
    v_scale = np.ascontiguousarray(v_scale, np.float32)
    assert q_scale.shape == (nblocks(N, gran_q),) and k_scale.shape == (nblocks(N, gran_k),)
    assert v_scale.shape == (D,)
    o = np.zeros((N, D), np.float16); lsum = np.zeros((N,), np.float32)
    if q_blocks is None:
        blocks, nb = None, -1
    else:
        blocks = np.ascontiguousarray(q_blocks, np.int32); nb = len(blocks)
        assert nb == 0 or (blocks.min() >= 0 and blocks.max() < nblocks(N, block_q))
    _L().sage_oracle_attn_pv8_slab_g(_p(qq), _p(q_scale), _p(kq), _p(k_scale), _p(vq), _p(v_scale),
                                     *map(ctypes.c_int, (N, D, int(causal), block_q, block_k, gran_q, gran_k)),
                                     _p(blocks) if blocks is not None else None, ctypes.c_int(nb),
                                     _p(o), _p(lsum))
    return (o, lsum) if return_l else o


def attn_l1_slab(qq, q_scale, kq, k_scale, v, causal: bool, block_q: int, block_k: int,
                 row0: int = 0, nrows: int | None = None) -> np.ndarray:
    """Quantized scores, exact fp64 softmax and P V (Section 4.1 with P, V unquantized).

    block_q / block_k are the tokens per scale (1 = per-token quantizer); there is no block loop."""
    v = _f16(v); N, D = v.shape
    qq = np.ascontiguousarray(qq, np.int8); kq = np.ascontiguousarray(kq, np.int8)
    q_scale = np.ascontiguousarray(q_scale, np.float32); k_scale = np.ascontiguousarray(k_scale, np.float32)
    nrows = N - row0 if nrows is None else nrows
    assert 0 <= row0 and row0 + nrows <= N
    o = np.empty((nrows, D), np.float64)
    _L().sage_oracle_attn_l1_slab(_p(qq), _p(q_scale), _p(kq), _p(k_scale), _p(v),
                                  *map(ctypes.c_int, (N, D, int(causal), block_q, block_k, row0, nrows)),
                                  _p(o))
    return o


def attn_l0_slab(q, k, v, causal: bool, sm_scale: float, row0: int = 0, nrows: int | None = None) -> np.ndarray:
    """Exact attention of Section 3.1 in fp64 on the given values (any float arrays [N, D])."""
    q = np.ascontiguousarray(q, np.float32); k = np.ascontiguousarray(k, np.float32)
    v = np.ascontiguousarray(v, np.float32)
    N, D = k.shape
    nrows = N - row0 if nrows is None else nrows
    assert 0 <= row0 and row0 + nrows <= N
    o = np.empty((nrows, D), np.float64)
    _L().sage_oracle_attn_l0_slab(_p(q), _p(k), _p(v), *map(ctypes.c_int, (N, D, int(causal))),
                                  ctypes.c_double(sm_scale), ctypes.c_int(row0), ctypes.c_int(nrows), _p(o))
    return o


# ---------------------------------------------------------------- Section 4.3 accuracy metrics

def accuracy_metrics(o_ref: np.ndarray, o_test: np.ndarray) -> dict:
    """Cosine similarity, relative L1 and RMSE over the flattened outputs."""
    a = np.asarray(o_ref, np.float64).ravel(); b = np.asarray(o_test, np.float64).ravel()
    cos = float(np.dot(a, b) / (np.sqrt(np.dot(a, a)) * np.sqrt(np.dot(b, b))))
    rel_l1 = float(np.abs(a - b).sum() / np.abs(a).sum())
    rmse = float(np.sqrt(np.mean((a - b) ** 2)))
    return {"cos": cos, "rel_l1": rel_l1, "rmse": rmse, "max_abs": float(np.abs(a - b).max())}
