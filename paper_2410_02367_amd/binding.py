"""ctypes binding of libsage.so (declared in include/sage.h).  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsage.so")
_lib = None

EXPORTS = ("sage_status_string", "sage_source_hash", "sage_default_sm_scale", "sage_quant_q", "sage_smooth_quant_k_workspace",
           "sage_smooth_quant_k", "sage_quant_qk", "sage_smooth_quant_k_noalloc", "sage_rope_quant_q", "sage_rope_smooth_quant_k",
           "sage_attn_fwd", "sage_attn_qk_i32_debug", "sage_attn_clock_debug",
           "sage_quant_v_workspace", "sage_quant_v_pitch", "sage_quant_v", "sage_attn_pv_int8_fwd",
           "sage_attn_cross_fwd", "sage_attn_pv_int8_cross_fwd",
           "sage_attn_split_count", "sage_attn_split_workspace", "sage_attn_cross_split_fwd",
           "sage_attn_pv_int8_cross_split_fwd", "sage_microbench")


class SageError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {sage_status_string(status)} (status {status})")


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load the built library.  A library that is missing, or that was built from other sources than
    the ones beside it (its embedded source hash says so), is rebuilt first where the compiler
    exists; elsewhere that is an error -- kernels are never run from a stale binary, and there is no
    other code path to fall back to."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build
    if _build.is_stale():
        if not _build.have_compiler():
            raise RuntimeError(f"{_LIB_PATH} is missing or was not built from the present sources "
                               f"(embedded hash {_build.built_hash()}, sources {_build.source_hash()}), "
                               "and there is no hipcc to rebuild it")
        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    lib.sage_source_hash.restype = ctypes.c_char_p
    lib.sage_source_hash.argtypes = []
    if lib.sage_source_hash().decode() != _build.source_hash():
        raise RuntimeError(f"{_LIB_PATH}: the loaded library reports another source hash than the file holds")
    c_int, c_float, c_void_p, c_size_t = ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    lib.sage_status_string.restype = ctypes.c_char_p
    lib.sage_status_string.argtypes = [c_int]
    lib.sage_default_sm_scale.restype = c_float
    lib.sage_default_sm_scale.argtypes = [c_int]
    lib.sage_quant_q.restype = c_int
    lib.sage_quant_q.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_float, c_int, c_void_p]
    lib.sage_smooth_quant_k_workspace.restype = c_size_t
    lib.sage_smooth_quant_k_workspace.argtypes = [c_int, c_int, c_int, c_int]
    lib.sage_smooth_quant_k.restype = c_int
    lib.sage_smooth_quant_k.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                        c_int, c_int, c_int, c_int, c_int, c_void_p]
    lib.sage_quant_qk.restype = c_int
    lib.sage_quant_qk.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t,
                                  c_int, c_int, c_int, c_int, c_int, c_float, c_int, c_int, c_void_p]
    lib.sage_smooth_quant_k_noalloc.restype = c_int
    lib.sage_smooth_quant_k_noalloc.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p]
    lib.sage_rope_quant_q.restype = c_int
    lib.sage_rope_quant_q.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                      c_int, c_int, c_int, c_int, c_float, c_int, c_void_p]
    lib.sage_rope_smooth_quant_k.restype = c_int
    lib.sage_rope_smooth_quant_k.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                             c_size_t, c_int, c_int, c_int, c_int, c_int, c_void_p]
    lib.sage_attn_fwd.restype = c_int
    lib.sage_attn_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                  c_int, c_int, c_int, c_int, c_int, c_float, c_int, c_int, c_void_p]
    lib.sage_attn_qk_i32_debug.restype = c_int
    lib.sage_attn_qk_i32_debug.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p]
    lib.sage_attn_clock_debug.restype = c_int
    lib.sage_attn_clock_debug.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                          c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p]
    lib.sage_attn_cross_fwd.restype = c_int
    lib.sage_attn_cross_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                        c_int, c_int, c_int, c_int, c_int, c_int, c_float, c_int, c_int, c_void_p]
    lib.sage_attn_split_count.restype = c_int
    lib.sage_attn_split_count.argtypes = [c_int] * 6
    lib.sage_attn_split_workspace.restype = c_size_t
    lib.sage_attn_split_workspace.argtypes = [c_int] * 7
    lib.sage_attn_cross_split_fwd.restype = c_int
    lib.sage_attn_cross_split_fwd.argtypes = [c_void_p] * 7 + [c_size_t] + [c_int] * 6 + [c_float, c_int, c_int, c_int, c_void_p]
    lib.sage_attn_pv_int8_cross_split_fwd.restype = c_int
    lib.sage_attn_pv_int8_cross_split_fwd.argtypes = [c_void_p] * 8 + [c_size_t] + [c_int] * 6 + [c_float, c_int, c_int, c_int, c_void_p]
    lib.sage_attn_pv_int8_cross_fwd.restype = c_int
    lib.sage_attn_pv_int8_cross_fwd.argtypes = [c_void_p] * 7 + [c_int] * 6 + [c_float, c_int, c_int, c_void_p]
    lib.sage_quant_v_workspace.restype = c_size_t
    lib.sage_quant_v_workspace.argtypes = [c_int, c_int, c_int, c_int]
    lib.sage_quant_v_pitch.restype = c_int
    lib.sage_quant_v_pitch.argtypes = [c_int]
    lib.sage_quant_v.restype = c_int
    lib.sage_quant_v.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_int, c_int, c_int, c_int, c_void_p]
    lib.sage_attn_pv_int8_fwd.restype = c_int
    lib.sage_attn_pv_int8_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                          c_int, c_int, c_int, c_int, c_int, c_float, c_int, c_int, c_void_p]
    lib.sage_microbench.restype = c_int
    lib.sage_microbench.argtypes = [c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p]
    _lib = lib
    return lib


def sage_status_string(status: int) -> str:
    return load().sage_status_string(int(status)).decode()


def sage_source_hash() -> str:
    """The hash of the sources the loaded library was built from."""
    return load().sage_source_hash().decode()


def sage_default_sm_scale(D: int) -> float:
    """1 / sqrt(D) as the fp32 value the library uses when the caller names no softmax scale."""
    return float(load().sage_default_sm_scale(int(D)))


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} tensor in device memory")
    return t.data_ptr()


def _nblk(N: int, block: int) -> int:
    return (N + block - 1) // block


def _rope_tables(cos, sin, N: int, D: int):
    for name, t in (("rope_cos", cos), ("rope_sin", sin)):
        if tuple(t.shape) != (N, D // 2):
            raise ValueError(f"{name}: expected shape ({N}, {D // 2}), got {tuple(t.shape)}")
    return _dev(cos, torch.float32, "rope_cos"), _dev(sin, torch.float32, "rope_sin")


def sage_rope_quant_q(q: torch.Tensor, rope_cos, rope_sin, sm_scale: float, block_q: int = 128,
                      q_i8=None, q_scale=None, stream=None):
    """sage_quant_q on RoPE(Q), the rotation applied on the fly (tables [N, D/2] fp32)."""
    B, H, N, D = q.shape
    pc, ps = _rope_tables(rope_cos, rope_sin, N, D)
    if q_i8 is None:
        q_i8 = torch.empty((B, H, N, D), dtype=torch.int8, device=q.device)
    if q_scale is None:
        q_scale = torch.empty((B, H, _nblk(N, block_q)), dtype=torch.float32, device=q.device)
    st = load().sage_rope_quant_q(_dev(q, torch.float16, "q"), pc, ps, _dev(q_i8, torch.int8, "q_i8"),
                                  _dev(q_scale, torch.float32, "q_scale"), B, H, N, D, float(sm_scale),
                                  int(block_q), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_rope_quant_q")
    return q_i8, q_scale


def sage_rope_smooth_quant_k(k: torch.Tensor, rope_cos, rope_sin, block_k: int = 64, k_i8=None, k_scale=None,
                             k_mean=None, workspace=None, stream=None):
    """sage_smooth_quant_k on RoPE(K), the rotation applied on the fly (tables [N, D/2] fp32)."""
    B, H, N, D = k.shape
    pc, ps = _rope_tables(rope_cos, rope_sin, N, D)
    if k_i8 is None:
        k_i8 = torch.empty((B, H, N, D), dtype=torch.int8, device=k.device)
    if k_scale is None:
        k_scale = torch.empty((B, H, _nblk(N, block_k)), dtype=torch.float32, device=k.device)
    if k_mean is None:
        k_mean = torch.empty((B, H, D), dtype=torch.float32, device=k.device)
    need = sage_smooth_quant_k_workspace(B, H, N, D)
    if workspace is None:
        workspace = torch.empty((max(need, 8) + 7) // 8, dtype=torch.int64, device=k.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    st = load().sage_rope_smooth_quant_k(_dev(k, torch.float16, "k"), pc, ps, _dev(k_i8, torch.int8, "k_i8"),
                                         _dev(k_scale, torch.float32, "k_scale"),
                                         _dev(k_mean, torch.float32, "k_mean"), workspace.data_ptr(), ws_bytes,
                                         B, H, N, D, int(block_k), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_rope_smooth_quant_k")
    return k_i8, k_scale, k_mean


def sage_quant_q(q: torch.Tensor, sm_scale: float, block_q: int = 128, q_i8=None, q_scale=None, stream=None):
    """psi_Q(Q * sm_scale) -> (q_i8 [B,H,N,D] int8, q_scale [B,H,ceil(N/block_q)] fp32); block_q = 1: per token."""
    B, H, N, D = q.shape
    if q_i8 is None:
        q_i8 = torch.empty((B, H, N, D), dtype=torch.int8, device=q.device)
    if q_scale is None:
        q_scale = torch.empty((B, H, _nblk(N, block_q)), dtype=torch.float32, device=q.device)
    st = load().sage_quant_q(_dev(q, torch.float16, "q"), _dev(q_i8, torch.int8, "q_i8"),
                             _dev(q_scale, torch.float32, "q_scale"), B, H, N, D, float(sm_scale),
                             int(block_q), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_quant_q")
    return q_i8, q_scale


def sage_smooth_quant_k_workspace(B: int, H: int, N: int, D: int) -> int:
    return int(load().sage_smooth_quant_k_workspace(B, H, N, D))


def sage_smooth_quant_k(k: torch.Tensor, block_k: int = 64, k_i8=None, k_scale=None, k_mean=None,
                        workspace=None, stream=None):
    """phi_K(K) -> (k_i8 int8, k_scale [B,H,ceil(N/block_k)] fp32, k_mean [B,H,D] fp32); block_k = 1: per token."""
    B, H, N, D = k.shape
    if k_i8 is None:
        k_i8 = torch.empty((B, H, N, D), dtype=torch.int8, device=k.device)
    if k_scale is None:
        k_scale = torch.empty((B, H, _nblk(N, block_k)), dtype=torch.float32, device=k.device)
    if k_mean is None:
        k_mean = torch.empty((B, H, D), dtype=torch.float32, device=k.device)
    need = sage_smooth_quant_k_workspace(B, H, N, D)
    if workspace is None:
        workspace = torch.empty((max(need, 8) + 7) // 8, dtype=torch.int64, device=k.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    st = load().sage_smooth_quant_k(_dev(k, torch.float16, "k"), _dev(k_i8, torch.int8, "k_i8"),
                                    _dev(k_scale, torch.float32, "k_scale"), _dev(k_mean, torch.float32, "k_mean"),
                                    workspace.data_ptr(), ws_bytes, B, H, N, D, int(block_k), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_smooth_quant_k")
    return k_i8, k_scale, k_mean


def sage_quant_qk(q: torch.Tensor, k: torch.Tensor, sm_scale: float, block_q: int = 128, block_k: int = 64,
                  q_i8=None, q_scale=None, k_i8=None, k_scale=None, k_mean=None, workspace=None, stream=None):
    """sage_quant_q(q) and sage_smooth_quant_k(k) in one launch less -> (q_i8, q_scale, k_i8, k_scale, k_mean)."""
    B, H, Nq, D = q.shape
    Nkv = k.shape[2]
    if k.shape[0] != B or k.shape[1] != H or k.shape[3] != D:
        raise ValueError("sage_quant_qk: q and k differ in batch, heads or head dimension")
    dev = q.device
    if q_i8 is None:
        q_i8 = torch.empty((B, H, Nq, D), dtype=torch.int8, device=dev)
    if q_scale is None:
        q_scale = torch.empty((B, H, _nblk(Nq, block_q)), dtype=torch.float32, device=dev)
    if k_i8 is None:
        k_i8 = torch.empty((B, H, Nkv, D), dtype=torch.int8, device=dev)
    if k_scale is None:
        k_scale = torch.empty((B, H, _nblk(Nkv, block_k)), dtype=torch.float32, device=dev)
    if k_mean is None:
        k_mean = torch.empty((B, H, D), dtype=torch.float32, device=dev)
    need = sage_smooth_quant_k_workspace(B, H, Nkv, D)
    if workspace is None:
        workspace = torch.empty((max(need, 8) + 7) // 8, dtype=torch.int64, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size()
    st = load().sage_quant_qk(_dev(q, torch.float16, "q"), _dev(k, torch.float16, "k"), _dev(q_i8, torch.int8, "q_i8"),
                              _dev(q_scale, torch.float32, "q_scale"), _dev(k_i8, torch.int8, "k_i8"),
                              _dev(k_scale, torch.float32, "k_scale"), _dev(k_mean, torch.float32, "k_mean"),
                              workspace.data_ptr(), ws_bytes, B, H, Nq, Nkv, D, float(sm_scale), int(block_q), int(block_k),
                              _stream(stream))
    if st != 0:
        raise SageError(st, "sage_quant_qk")
    return q_i8, q_scale, k_i8, k_scale, k_mean


NOALLOC_SCRATCH_BYTES = 4 << 20     # SAGE_NOALLOC_SCRATCH_BYTES of include/sage.h


def sage_smooth_quant_k_noalloc(k: torch.Tensor, block_k: int = 64, k_i8=None, k_scale=None, k_mean=None, stream=None):
    """sage_smooth_quant_k without a workspace argument: the library call allocates nothing (its scratch is a
    static device array); pass k_i8 / k_scale / k_mean as well and neither does this wrapper."""
    B, H, N, D = k.shape
    if k_i8 is None:
        k_i8 = torch.empty((B, H, N, D), dtype=torch.int8, device=k.device)
    if k_scale is None:
        k_scale = torch.empty((B, H, _nblk(N, block_k)), dtype=torch.float32, device=k.device)
    if k_mean is None:
        k_mean = torch.empty((B, H, D), dtype=torch.float32, device=k.device)
    st = load().sage_smooth_quant_k_noalloc(_dev(k, torch.float16, "k"), _dev(k_i8, torch.int8, "k_i8"),
                                            _dev(k_scale, torch.float32, "k_scale"), _dev(k_mean, torch.float32, "k_mean"),
                                            B, H, N, D, int(block_k), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_smooth_quant_k_noalloc")
    return k_i8, k_scale, k_mean


def sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, v, causal: bool, sm_scale: float,
                  block_q: int = 128, block_k: int = 64, out=None, stream=None):
    """Algorithm 1's loop on pre-quantized Q^, K^ and fp16 V -> O [B,H,N,D] fp16.

    block_q / block_k are the tokens per scale the tensors were quantized with (1 = per token)."""
    B, H, N, D = v.shape
    if out is None:
        out = torch.empty((B, H, N, D), dtype=torch.float16, device=v.device)
    st = load().sage_attn_fwd(_dev(q_i8, torch.int8, "q_i8"), _dev(q_scale, torch.float32, "q_scale"),
                              _dev(k_i8, torch.int8, "k_i8"), _dev(k_scale, torch.float32, "k_scale"),
                              _dev(v, torch.float16, "v"), _dev(out, torch.float16, "out"),
                              B, H, N, D, int(bool(causal)), float(sm_scale), int(block_q), int(block_k),
                              _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_fwd")
    return out


def sage_attn_cross_fwd(q_i8, q_scale, k_i8, k_scale, v, causal: bool, sm_scale: float,
                        block_q: int = 128, block_k: int = 64, out=None, stream=None):
    """sage_attn_fwd with Nq queries (q_i8 [B,H,Nq,D]) against Nkv keys and values ([B,H,Nkv,D]) -> O [B,H,Nq,D];
    the causal mask is aligned at the end (needs Nq <= Nkv)."""
    B, H, Nkv, D = v.shape
    Nq = q_i8.shape[2]
    if tuple(q_i8.shape) != (B, H, Nq, D) or tuple(k_i8.shape) != (B, H, Nkv, D):
        raise TypeError("q_i8 / k_i8: shapes do not match v")
    if out is None:
        out = torch.empty((B, H, Nq, D), dtype=torch.float16, device=v.device)
    st = load().sage_attn_cross_fwd(_dev(q_i8, torch.int8, "q_i8"), _dev(q_scale, torch.float32, "q_scale"),
                                    _dev(k_i8, torch.int8, "k_i8"), _dev(k_scale, torch.float32, "k_scale"),
                                    _dev(v, torch.float16, "v"), _dev(out, torch.float16, "out"),
                                    B, H, Nq, Nkv, D, int(bool(causal)), float(sm_scale), int(block_q), int(block_k),
                                    _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_cross_fwd")
    return out


def sage_attn_split_count(B: int, H: int, Nq: int, Nkv: int, causal: bool, n_splits: int = 0) -> int:
    """Number of key chunks sage_attn_cross_split_fwd uses for a requested n_splits (0 = chosen from the shape)."""
    return int(load().sage_attn_split_count(B, H, Nq, Nkv, int(bool(causal)), int(n_splits)))


def sage_attn_split_workspace(B: int, H: int, Nq: int, Nkv: int, D: int, causal: bool, n_splits: int = 0) -> int:
    return int(load().sage_attn_split_workspace(B, H, Nq, Nkv, D, int(bool(causal)), int(n_splits)))


def sage_attn_cross_split_fwd(q_i8, q_scale, k_i8, k_scale, v, causal: bool, sm_scale: float,
                              block_q: int = 128, block_k: int = 64, n_splits: int = 0,
                              out=None, workspace=None, stream=None):
    """sage_attn_cross_fwd with the keys cut into n_splits chunks (0 = chosen from the shape) and a merge:
    for few queries against many keys.  workspace: uint8 device tensor of at least
    sage_attn_split_workspace(...) bytes (allocated here if not given)."""
    B, H, Nkv, D = v.shape
    Nq = q_i8.shape[2]
    if tuple(q_i8.shape) != (B, H, Nq, D) or tuple(k_i8.shape) != (B, H, Nkv, D):
        raise TypeError("q_i8 / k_i8: shapes do not match v")
    if out is None:
        out = torch.empty((B, H, Nq, D), dtype=torch.float16, device=v.device)
    need = sage_attn_split_workspace(B, H, Nq, Nkv, D, causal, n_splits)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=v.device)
    ws_ptr = _dev(workspace, torch.uint8, "workspace") if workspace is not None else 0
    ws_bytes = workspace.numel() if workspace is not None else 0
    st = load().sage_attn_cross_split_fwd(_dev(q_i8, torch.int8, "q_i8"), _dev(q_scale, torch.float32, "q_scale"),
                                          _dev(k_i8, torch.int8, "k_i8"), _dev(k_scale, torch.float32, "k_scale"),
                                          _dev(v, torch.float16, "v"), _dev(out, torch.float16, "out"),
                                          ws_ptr, ws_bytes, B, H, Nq, Nkv, D, int(bool(causal)), float(sm_scale),
                                          int(block_q), int(block_k), int(n_splits), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_cross_split_fwd")
    return out


def sage_attn_pv_int8_cross_split_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal: bool, sm_scale: float,
                                      block_q: int = 128, block_k: int = 64, n_splits: int = 0,
                                      out=None, workspace=None, stream=None):
    """sage_attn_pv_int8_cross_fwd with the keys cut into n_splits chunks (0 = chosen from the shape) and a merge.
    workspace: uint8 device tensor of at least sage_attn_split_workspace(...) bytes (allocated here if not given)."""
    B, H, Nkv, D = k_i8.shape
    Nq = q_i8.shape[2]
    if tuple(q_i8.shape) != (B, H, Nq, D) or tuple(v_i8t.shape) != (B, H, D, sage_quant_v_pitch(Nkv)):
        raise TypeError("q_i8 / v_i8t: shapes do not match k_i8")
    if out is None:
        out = torch.empty((B, H, Nq, D), dtype=torch.float16, device=k_i8.device)
    need = sage_attn_split_workspace(B, H, Nq, Nkv, D, causal, n_splits)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=k_i8.device)
    ws_ptr = _dev(workspace, torch.uint8, "workspace") if workspace is not None else 0
    ws_bytes = workspace.numel() if workspace is not None else 0
    st = load().sage_attn_pv_int8_cross_split_fwd(
        _dev(q_i8, torch.int8, "q_i8"), _dev(q_scale, torch.float32, "q_scale"),
        _dev(k_i8, torch.int8, "k_i8"), _dev(k_scale, torch.float32, "k_scale"),
        _dev(v_i8t, torch.int8, "v_i8t"), _dev(v_scale, torch.float32, "v_scale"), _dev(out, torch.float16, "out"),
        ws_ptr, ws_bytes, B, H, Nq, Nkv, D, int(bool(causal)), float(sm_scale), int(block_q), int(block_k), int(n_splits),
        _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_pv_int8_cross_split_fwd")
    return out


def sage_quant_v_workspace(B: int, H: int, N: int, D: int) -> int:
    return int(load().sage_quant_v_workspace(B, H, N, D))


def sage_quant_v_pitch(N: int) -> int:
    return int(load().sage_quant_v_pitch(N))


def sage_quant_v(v: torch.Tensor, v_i8t=None, v_scale=None, workspace=None, stream=None):
    """psi_V(V), per channel -> (v_i8t int8 [B,H,D,Np] (transposed, Np = sage_quant_v_pitch(N)), v_scale [B,H,D] fp32)."""
    B, H, N, D = v.shape
    Np = sage_quant_v_pitch(N)
    if v_i8t is None:
        v_i8t = torch.empty((B, H, D, Np), dtype=torch.int8, device=v.device)
    if v_scale is None:
        v_scale = torch.empty((B, H, D), dtype=torch.float32, device=v.device)
    need = sage_quant_v_workspace(B, H, N, D)
    if workspace is None:
        workspace = torch.empty((max(need, 4) + 3) // 4, dtype=torch.int32, device=v.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    if tuple(v_i8t.shape) != (B, H, D, Np):
        raise TypeError(f"v_i8t: expected shape {(B, H, D, Np)}")
    st = load().sage_quant_v(_dev(v, torch.float16, "v"), _dev(v_i8t, torch.int8, "v_i8t"),
                             _dev(v_scale, torch.float32, "v_scale"), workspace.data_ptr(), ws_bytes,
                             B, H, N, D, _stream(stream))
    if st != 0:
        raise SageError(st, "sage_quant_v")
    return v_i8t, v_scale


def sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal: bool, sm_scale: float,
                          block_q: int = 128, block_k: int = 64, out=None, stream=None):
    """Algorithm 1's loop with the INT8 second product of Section 4.3 (SAGEAttn-vB; block sizes 1: -vT)
    on pre-quantized Q^, K^ and V^^T -> O [B,H,N,D] fp16."""
    B, H, N, D = q_i8.shape
    if tuple(v_i8t.shape) != (B, H, D, sage_quant_v_pitch(N)):
        raise TypeError(f"v_i8t: expected shape {(B, H, D, sage_quant_v_pitch(N))}")
    if out is None:
        out = torch.empty((B, H, N, D), dtype=torch.float16, device=q_i8.device)
    st = load().sage_attn_pv_int8_fwd(_dev(q_i8, torch.int8, "q_i8"), _dev(q_scale, torch.float32, "q_scale"),
                                      _dev(k_i8, torch.int8, "k_i8"), _dev(k_scale, torch.float32, "k_scale"),
                                      _dev(v_i8t, torch.int8, "v_i8t"), _dev(v_scale, torch.float32, "v_scale"),
                                      _dev(out, torch.float16, "out"),
                                      B, H, N, D, int(bool(causal)), float(sm_scale), int(block_q), int(block_k),
                                      _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_pv_int8_fwd")
    return out


def sage_attn_pv_int8_cross_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal: bool, sm_scale: float,
                                block_q: int = 128, block_k: int = 64, out=None, stream=None):
    """sage_attn_pv_int8_fwd with Nq queries (q_i8 [B,H,Nq,D]) against Nkv keys (k_i8 [B,H,Nkv,D], v_i8t from
    sage_quant_v of the Nkv values) -> O [B,H,Nq,D]; end-aligned causal mask (needs Nq <= Nkv)."""
    B, H, Nq, D = q_i8.shape
    Nkv = k_i8.shape[2]
    if tuple(k_i8.shape) != (B, H, Nkv, D) or tuple(v_i8t.shape) != (B, H, D, sage_quant_v_pitch(Nkv)):
        raise TypeError("k_i8 / v_i8t: shapes do not match q_i8")
    if out is None:
        out = torch.empty((B, H, Nq, D), dtype=torch.float16, device=q_i8.device)
    st = load().sage_attn_pv_int8_cross_fwd(_dev(q_i8, torch.int8, "q_i8"), _dev(q_scale, torch.float32, "q_scale"),
                                            _dev(k_i8, torch.int8, "k_i8"), _dev(k_scale, torch.float32, "k_scale"),
                                            _dev(v_i8t, torch.int8, "v_i8t"), _dev(v_scale, torch.float32, "v_scale"),
                                            _dev(out, torch.float16, "out"),
                                            B, H, Nq, Nkv, D, int(bool(causal)), float(sm_scale), int(block_q), int(block_k),
                                            _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_pv_int8_cross_fwd")
    return out


def sage_attn_qk_i32_debug(q_i8, k_i8, s_i32=None, block_q: int = 128, block_k: int = 64, wg_rows: int = 0, stream=None):
    """Raw int32 scores Q^ K^^T [B,H,N,N] through the attention kernel's MFMA path (test hook);
    wg_rows = 128 / 256 names the workgroup shape, 0 leaves it to the launcher."""
    B, H, N, D = q_i8.shape
    if s_i32 is None:
        s_i32 = torch.empty((B, H, N, N), dtype=torch.int32, device=q_i8.device)
    st = load().sage_attn_qk_i32_debug(_dev(q_i8, torch.int8, "q_i8"), _dev(k_i8, torch.int8, "k_i8"),
                                       _dev(s_i32, torch.int32, "s_i32"), B, H, N, D, int(block_q), int(block_k),
                                       int(wg_rows), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_qk_i32_debug")
    return s_i32


def sage_attn_clock_debug(q_i8, q_scale, k_i8, k_scale, v, out=None, causal: bool = False, block_q: int = 128,
                          block_k: int = 64, stream=None):
    """sage_attn_fwd's kernel at D = 128 in its 256-row shape, built with counters (measurement hook) ->
    (out, clocks): clocks [B*H*ceil(N/256)*8, 4] int64, per wavefront shader-clock ticks, 100 MHz ticks, raises
    of the running maximum, key tiles visited."""
    B, H, N, D = q_i8.shape
    if out is None:
        out = torch.empty((B, H, N, D), dtype=torch.float16, device=q_i8.device)
    clocks = torch.zeros((B * H * ((N + 255) // 256) * 8, 4), dtype=torch.int64, device=q_i8.device)
    st = load().sage_attn_clock_debug(_dev(q_i8, torch.int8, "q_i8"), _dev(q_scale, torch.float32, "q_scale"),
                                      _dev(k_i8, torch.int8, "k_i8"), _dev(k_scale, torch.float32, "k_scale"),
                                      _dev(v, torch.float16, "v"), _dev(out, torch.float16, "out"),
                                      _dev(clocks, torch.int64, "clocks"), B, H, N, D, int(bool(causal)),
                                      int(block_q), int(block_k), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_attn_clock_debug")
    return out, clocks


def sage_microbench(kind: int, waves_per_simd: int, workgroups: int, iters: int, data, out=None, stream=None):
    """One launch of an instruction-stream probe (see include/sage.h) -> out [wavefronts, 4] uint64 as int64:
    shader-clock ticks, constant-rate ticks, checksum, 0.  data: 1024 int32 of random bits on the device."""
    waves = workgroups * 4 * waves_per_simd
    if out is None:
        out = torch.empty((waves, 4), dtype=torch.int64, device=data.device)
    if data.numel() < 1024 or out.numel() < 4 * waves:
        raise ValueError("sage_microbench: data needs 1024 words, out 4 per wavefront")
    st = load().sage_microbench(int(kind), int(waves_per_simd), int(workgroups), int(iters),
                                _dev(data, torch.int32, "data"), _dev(out, torch.int64, "out"), _stream(stream))
    if st != 0:
        raise SageError(st, "sage_microbench")
    return out


def sageattn(q, k, v, causal: bool = False, sm_scale: float | None = None, block_q: int = 128, block_k: int = 64,
             pv_int8: bool = False):
    """Convenience: the library calls in order (pre-pass on K, on Q and, with pv_int8, on V; attention).
    q [B,H,Nq,D] against k, v [B,H,Nkv,D]: equal lengths take the self-attention calls, different
    lengths the calls that may split the keys over workgroups (end-aligned causal mask)."""
    D = q.shape[-1]
    if sm_scale is None:
        sm_scale = sage_default_sm_scale(D)
    q_i8, q_scale, k_i8, k_scale, _ = sage_quant_qk(q, k, sm_scale, block_q, block_k)
    same = q.shape[2] == k.shape[2]
    if pv_int8:
        v_i8t, v_scale = sage_quant_v(v)
        if same:
            return sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal, sm_scale, block_q, block_k)
        return sage_attn_pv_int8_cross_split_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal, sm_scale, block_q, block_k)
    if same:
        return sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, v, causal, sm_scale, block_q, block_k)
    return sage_attn_cross_split_fwd(q_i8, q_scale, k_i8, k_scale, v, causal, sm_scale, block_q, block_k)
