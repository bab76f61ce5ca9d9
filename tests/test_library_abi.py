"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
and validates arguments on the host (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2410_02367_amd import binding
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sage_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"sage_quant_q", "sage_smooth_quant_k", "sage_attn_fwd"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None


def test_binding_covers_the_header():
    from paper_2410_02367_amd import binding
    assert sorted(binding.EXPORTS) == declared_symbols()
    import paper_2410_02367_amd as pkg
    for n in binding.EXPORTS:
        assert callable(getattr(pkg, n))


def test_status_strings(lib):
    assert lib.sage_status_string(0) == b"SAGE_OK"
    for code in range(1, 8):
        assert lib.sage_status_string(code).startswith(b"SAGE_ERR_")
    assert lib.sage_status_string(99) == b"SAGE_ERR_UNKNOWN"


def test_workspace_query(lib):
    """Partial column sums: [B*H, chunks, D] 64-bit words, chunks of whole 256-row batches (at least 512
    rows), about 512 chunks over all slabs and never more than 64 per slab; none for short sequences."""
    assert lib.sage_smooth_quant_k_workspace(1, 2, 256, 64) == 0
    assert lib.sage_smooth_quant_k_workspace(1, 2, 512, 64) == 0
    assert lib.sage_smooth_quant_k_workspace(1, 2, 513, 64) == 2 * 2 * 64 * 8
    assert lib.sage_smooth_quant_k_workspace(1, 32, 16384, 128) == 16 * 32 * 128 * 8
    assert lib.sage_smooth_quant_k_workspace(1, 8, 131072, 128) == 64 * 8 * 128 * 8
    assert lib.sage_smooth_quant_k_workspace(4, 32, 4096, 128) == 4 * 128 * 128 * 8
    assert lib.sage_smooth_quant_k_workspace(1, 1, 1 << 23, 128) == 64 * 128 * 8
    assert lib.sage_smooth_quant_k_workspace(0, 8, 10, 128) == 0
    for B, H, N, D in ((2, 30, 17776, 64), (1, 1, 100000, 64), (3, 7, 5000, 128), (1, 1, 513, 128)):
        chunks = lib.sage_smooth_quant_k_workspace(B, H, N, D) // (B * H * D * 8)
        assert 1 <= chunks <= 64 and lib.sage_smooth_quant_k_workspace(B, H, N, D) == chunks * B * H * D * 8


def test_host_validation_rejects_bad_arguments_before_any_launch(lib):
    f = ctypes.c_float
    good = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    # NULL pointers
    assert lib.sage_quant_q(None, good, good, 1, 1, 64, 64, f(0.125), 64, None) == 1
    assert lib.sage_attn_fwd(good, good, good, good, None, good, 1, 1, 64, 64, 0, f(0.125), 128, 64, None) == 1
    assert lib.sage_smooth_quant_k(good, good, good, good, None, 0, 1, 1, 1024, 64, 64, None) == 1
    # shapes
    assert lib.sage_quant_q(good, good, good, 0, 1, 64, 64, f(0.125), 64, None) == 2
    assert lib.sage_quant_q(good, good, good, 1, 1, (1 << 23) + 1, 64, f(0.125), 64, None) == 2
    assert lib.sage_quant_q(good, good, good, 1, 1, 64, 96, f(0.125), 64, None) == 3
    assert lib.sage_quant_q(good, good, good, 1, 1, 64, 64, f(0.125), 48, None) == 3
    assert lib.sage_attn_fwd(good, good, good, good, good, good, 1, 1, 64, 64, 0, f(0.125), 128, 32, None) == 3
    # values
    assert lib.sage_quant_q(good, good, good, 1, 1, 64, 64, f(float("inf")), 64, None) == 7
    assert lib.sage_attn_fwd(good, good, good, good, good, good, 1, 1, 64, 64, 0, f(-1.0), 128, 64, None) == 7
    # workspace, alignment
    assert lib.sage_smooth_quant_k(good, good, good, good, good, 8, 1, 1, 1024, 64, 64, None) == 4
    assert lib.sage_quant_q(odd, good, good, 1, 1, 64, 64, f(0.125), 64, None) == 5
    assert lib.sage_attn_qk_i32_debug(good, odd, good, 1, 1, 64, 64, 128, 64, 0, None) == 5
    assert lib.sage_attn_qk_i32_debug(good, good, good, 1, 1, 64, 64, 128, 32, 0, None) == 3
    assert lib.sage_attn_qk_i32_debug(good, good, good, 1, 1, 64, 64, 128, 64, 64, None) == 3
    # the attention kernel's measurement build: D = 128 with one scale per key block only
    assert lib.sage_attn_clock_debug(good, good, good, good, good, good, None, 1, 1, 64, 128, 0, 128, 64, None) == 1
    assert lib.sage_attn_clock_debug(good, good, good, good, good, good, good, 1, 1, 64, 64, 0, 128, 64, None) == 3
    assert lib.sage_attn_clock_debug(good, good, good, good, good, good, good, 1, 1, 64, 128, 0, 1, 1, None) == 3
    assert lib.sage_attn_clock_debug(good, good, good, good, good, good, good, 0, 1, 64, 128, 0, 128, 64, None) == 2
    assert lib.sage_attn_clock_debug(good, good, good, good, good, good, odd, 1, 1, 64, 128, 0, 128, 64, None) == 5
    # both pre-passes in one call: the checks of either side
    sz = ctypes.c_size_t
    assert lib.sage_quant_qk(good, None, good, good, good, good, good, good, sz(1 << 20), 1, 1, 64, 64, 64, f(0.125), 64, 64, None) == 1
    assert lib.sage_quant_qk(good, good, good, good, good, good, good, good, sz(8), 1, 1, 64, 1024, 64, f(0.125), 64, 64, None) == 4
    assert lib.sage_quant_qk(good, good, good, good, good, good, good, good, sz(1 << 20), 1, 1, 0, 64, 64, f(0.125), 64, 64, None) == 2
    assert lib.sage_quant_qk(good, good, good, good, good, good, good, good, sz(1 << 20), 1, 1, 64, 64, 64, f(0.125), 48, 64, None) == 3
    assert lib.sage_quant_qk(good, good, good, good, good, good, good, good, sz(1 << 20), 1, 1, 64, 64, 64, f(0.125), 64, 48, None) == 3
    assert lib.sage_quant_qk(good, good, good, good, good, good, good, good, sz(1 << 20), 1, 1, 64, 64, 64, f(0.0), 64, 64, None) == 7
    assert lib.sage_quant_qk(good, odd, good, good, good, good, good, good, sz(1 << 20), 1, 1, 64, 64, 64, f(0.125), 64, 64, None) == 5
    # more (batch, head) slabs than the documented limit
    assert lib.sage_quant_q(good, good, good, 256, 256, 64, 64, f(0.125), 64, None) == 2
    # the fused-RoPE calls: tables required and 16-byte aligned, everything else as the unfused calls
    assert lib.sage_rope_quant_q(good, None, good, good, good, 1, 1, 64, 64, f(0.125), 64, None) == 1
    assert lib.sage_rope_quant_q(good, good, odd, good, good, 1, 1, 64, 64, f(0.125), 64, None) == 5
    assert lib.sage_rope_quant_q(good, good, good, good, good, 1, 1, 64, 64, f(0.125), 48, None) == 3
    assert lib.sage_rope_smooth_quant_k(good, good, None, good, good, good, good, 1 << 20, 1, 1, 64, 64, 64, None) == 1
    assert lib.sage_rope_smooth_quant_k(good, good, good, good, good, good, good, 8, 1, 1, 1024, 64, 64, None) == 4
    assert lib.sage_rope_smooth_quant_k(good, odd, good, good, good, good, good, 1 << 20, 1, 1, 64, 64, 64, None) == 5


def test_int8_second_product_calls_validate_like_the_others(lib):
    f = ctypes.c_float
    good = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    assert lib.sage_quant_v_workspace(1, 2, 256, 64) == 2 * 64 * 4
    assert lib.sage_quant_v_workspace(1, 0, 256, 64) == 0
    assert [lib.sage_quant_v_pitch(n) for n in (0, 1, 64, 65, 17776)] == [0, 64, 64, 128, 17792]
    assert lib.sage_quant_v(None, good, good, good, 1 << 20, 1, 1, 64, 64, None) == 1
    assert lib.sage_quant_v(good, good, good, good, 1 << 20, 1, 1, 0, 64, None) == 2
    assert lib.sage_quant_v(good, good, good, good, 1 << 20, 1, 1, 64, 96, None) == 3
    assert lib.sage_quant_v(good, good, good, good, 8, 1, 1, 64, 64, None) == 4
    assert lib.sage_quant_v(good, odd, good, good, 1 << 20, 1, 1, 64, 64, None) == 5
    args = (1, 1, 64, 64, 0)
    assert lib.sage_attn_pv_int8_fwd(good, good, good, good, None, good, good, *args, f(0.125), 128, 64, None) == 1
    assert lib.sage_attn_pv_int8_fwd(good, good, good, good, good, good, good, 1, 1, 64, 96, 0, f(0.125), 128, 64, None) == 3
    assert lib.sage_attn_pv_int8_fwd(good, good, good, good, good, good, good, *args, f(0.125), 128, 32, None) == 3
    assert lib.sage_attn_pv_int8_fwd(good, good, good, good, good, good, good, *args, f(float("nan")), 128, 64, None) == 7
    assert lib.sage_attn_pv_int8_fwd(good, good, good, good, good, odd, good, *args, f(0.125), 128, 64, None) == 5


def test_cross_attention_call_validates_both_lengths(lib):
    f = ctypes.c_float
    good = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    assert lib.sage_attn_cross_fwd(good, good, good, good, good, None, 1, 1, 64, 64, 64, 0, f(0.125), 128, 64, None) == 1
    assert lib.sage_attn_cross_fwd(good, good, good, good, good, good, 1, 1, 0, 64, 64, 0, f(0.125), 128, 64, None) == 2
    assert lib.sage_attn_cross_fwd(good, good, good, good, good, good, 1, 1, 64, (1 << 23) + 1, 64, 0, f(0.125), 128, 64, None) == 2
    assert lib.sage_attn_cross_fwd(good, good, good, good, good, good, 1, 1, 65, 64, 64, 1, f(0.125), 128, 64, None) == 3
    assert lib.sage_attn_cross_fwd(good, good, good, good, good, good, 1, 1, 64, 64, 64, 0, f(0.125), 128, 32, None) == 3
    assert lib.sage_attn_cross_fwd(good, good, good, good, good, good, 1, 1, 64, 64, 64, 0, f(0.0), 128, 64, None) == 7
    assert lib.sage_attn_cross_fwd(good, good, odd, good, good, good, 1, 1, 64, 64, 64, 0, f(0.125), 128, 64, None) == 5
    args = (good,) * 7
    assert lib.sage_attn_pv_int8_cross_fwd(*args, 1, 1, 65, 64, 64, 1, f(0.125), 128, 64, None) == 3
    assert lib.sage_attn_pv_int8_cross_fwd(*args, 1, 1, 64, 0, 64, 0, f(0.125), 128, 64, None) == 2
    assert lib.sage_attn_pv_int8_cross_fwd(good, good, good, good, None, good, good, 1, 1, 64, 64, 64, 0, f(0.125), 128, 64, None) == 1


def test_split_call_validates_and_its_chunk_plan_keeps_its_promises(lib):
    """Host logic of sage_attn_cross_split_fwd: argument checks, and the chunk plan -- never more chunks
    than requested (64 when it chooses), never an empty chunk and, with a causal mask, never a chunk
    that some query row cannot see (the last chunk starts at or before key Nkv - Nq)."""
    import numpy as np
    f = ctypes.c_float
    good = ctypes.c_void_p(0x1000)
    sz = ctypes.c_size_t
    head = (good,) * 6
    assert lib.sage_attn_cross_split_fwd(*head, None, sz(0), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, 4, None) == 1
    assert lib.sage_attn_cross_split_fwd(*head, good, sz(64), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, 4, None) == 4
    assert lib.sage_attn_cross_split_fwd(*head, good, sz(1 << 30), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, -1, None) == 7
    assert lib.sage_attn_cross_split_fwd(*head, good, sz(1 << 30), 1, 1, 4097, 4096, 64, 1, f(0.125), 128, 64, 4, None) == 3
    assert lib.sage_attn_cross_split_fwd(*head, ctypes.c_void_p(0x1004), sz(1 << 30), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, 4, None) == 5
    head8 = (good,) * 7
    assert lib.sage_attn_pv_int8_cross_split_fwd(*head8, None, sz(0), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, 4, None) == 1
    assert lib.sage_attn_pv_int8_cross_split_fwd(*head8, good, sz(64), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, 4, None) == 4
    assert lib.sage_attn_pv_int8_cross_split_fwd(*head8, good, sz(1 << 30), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, -1, None) == 7
    assert lib.sage_attn_pv_int8_cross_split_fwd(*head8, good, sz(1 << 30), 1, 1, 4097, 4096, 64, 1, f(0.125), 128, 64, 4, None) == 3
    # 65535 slabs x 32768 chunks of 128 keys: more (slab, chunk) pairs than the kernels count
    assert lib.sage_attn_cross_split_fwd(*head, good, sz(1 << 62), 255, 257, 1, 1 << 22, 64, 0, f(0.125), 128, 64, 1 << 15, None) == 2
    assert lib.sage_attn_split_count(1, 1, 4097, 4096, 1, 4) == 0
    assert lib.sage_attn_split_count(1, 1, 4, 4096, 1, 1) == 1 and lib.sage_attn_split_workspace(1, 1, 4, 4096, 64, 1, 1) == 0
    assert lib.sage_attn_split_workspace(2, 3, 4, 4096, 64, 1, 4) == 4 * 2 * 3 * 4 * (2 * 64 + 4)
    # a request far beyond the number of 128-key groups is the plan of that number (and must not
    # overflow the host arithmetic): 4096 keys are 32 groups
    for huge in (1 << 24, 1 << 25, (1 << 31) - 1):
        assert lib.sage_attn_split_count(1, 1, 4, 4096, 1, huge) == 32
        assert lib.sage_attn_split_count(1, 1, 4, 4096, 0, huge) == 32
        assert lib.sage_attn_split_workspace(1, 1, 4, 4096, 64, 1, huge) == 32 * 4 * (2 * 64 + 4)
        assert lib.sage_attn_cross_split_fwd(*head, good, sz(64), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, huge, None) == 4
        assert lib.sage_attn_pv_int8_cross_split_fwd(*head8, good, sz(64), 1, 1, 4, 4096, 64, 1, f(0.125), 128, 64, huge, None) == 4
        assert lib.sage_attn_split_count(1, 1, 1, 1, 0, huge) == 1
    g = np.random.default_rng(20241002)
    for _ in range(3000):
        Nkv = int(g.integers(1, 40000))
        causal = int(g.integers(0, 2))
        Nq = int(g.integers(1, Nkv + 1)) if causal else int(g.integers(1, 3000))
        req = int(g.integers(0, 70))
        B, H = int(g.integers(1, 4)), int(g.integers(1, 40))
        n = lib.sage_attn_split_count(B, H, Nq, Nkv, causal, req)
        assert 1 <= n <= (req if req > 0 else 64), (Nq, Nkv, causal, req, n)
        if n > 1 and req > 0:        # the chunk length follows from the requested count
            chunk = 128 * -(-Nkv // (128 * req))
            assert (n - 1) * chunk <= (Nkv - Nq if causal else Nkv - 1), (Nq, Nkv, causal, req, n)


def test_microbench_call_validates_its_arguments(lib):
    good = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    assert lib.sage_microbench(0, 1, 256, 10, None, good, None) == 1
    assert lib.sage_microbench(99, 1, 256, 10, good, good, None) == 3
    assert lib.sage_microbench(0, 3, 256, 10, good, good, None) == 3
    assert lib.sage_microbench(5, 1, 256, 10, good, good, None) == 3       # the split probe needs two wavefronts per SIMD
    assert lib.sage_microbench(0, 1, 0, 10, good, good, None) == 2
    assert lib.sage_microbench(0, 1, 256, 0, good, good, None) == 2
    assert lib.sage_microbench(0, 1, 256, 10, odd, good, None) == 5
    assert lib.sage_default_sm_scale(64) == 0.125 and lib.sage_default_sm_scale(0) == 0.0
    assert abs(lib.sage_default_sm_scale(128) - 128 ** -0.5) < 1e-8
