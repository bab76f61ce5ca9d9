"""sage_smooth_quant_k_noalloc (the pre-pass of K with the library's static scratch instead of a
caller-supplied workspace) against sage_smooth_quant_k, through the C ABI: the same kernels on another
scratch buffer, so every INT8 code, scale and mean must be the same bits.  Two calls in a row share the
buffer, the second on a smaller input (it must not see what the first left there); the first call is
also checked against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import bits, to_dev

pytestmark = pytest.mark.gpu


def both_calls(k, block_k):
    kd = to_dev(k)
    ref = sage.sage_smooth_quant_k(kd, block_k)
    # outputs pre-filled with a pattern the kernels must overwrite completely
    B, H, N, D = k.shape
    k_i8 = torch.full((B, H, N, D), 0x55, dtype=torch.int8, device="cuda")
    k_scale = torch.full((B, H, (N + block_k - 1) // block_k), float("nan"), dtype=torch.float32, device="cuda")
    k_mean = torch.full((B, H, D), float("nan"), dtype=torch.float32, device="cuda")
    got = sage.sage_smooth_quant_k_noalloc(kd, block_k, k_i8=k_i8, k_scale=k_scale, k_mean=k_mean)
    torch.cuda.synchronize()
    return ref, got


def assert_same_bits(ref, got, what):
    for name, a, b in zip(("k_i8", "k_scale", "k_mean"), ref, got):
        a, b = a.cpu().numpy(), b.cpu().numpy()
        same = np.array_equal(a, b) if a.dtype == np.int8 else np.array_equal(bits(a), bits(b))
        assert same, f"{what}: {name} differs between the two entry points"


def test_two_calls_in_a_row_the_second_smaller():
    # first: 3 slabs of 5000 tokens at D = 128 (several partial sums per slab, a ragged last chunk and block)
    w1 = si.custom("noalloc_first", 1, 3, 5000, 128, False, 128, 64, k_noise=1.0, k_bias=4.0, seed=si.BASE_SEED + 700)
    _, k1, _ = si.full(w1)
    print(f"[case] no-alloc K pre-pass, first call B1 H3 N5000 D128 block 64 "
          f"(workspace {sage.sage_smooth_quant_k_workspace(1, 3, 5000, 128)} bytes)", flush=True)
    ref1, got1 = both_calls(k1, 64)
    assert_same_bits(ref1, got1, "first call")
    kq, ks, km = oracle.smooth_quant_k(k1, 64)
    assert np.array_equal(got1[0].cpu().numpy(), kq)
    assert np.array_equal(bits(got1[1].cpu().numpy()), bits(ks)) and np.array_equal(bits(got1[2].cpu().numpy()), bits(km))
    # second: a smaller input, other head dimension and granularity, right after the first on the same scratch
    w2 = si.custom("noalloc_second", 2, 2, 1300, 64, False, 128, 64, k_noise=0.5, k_bias=3.0, seed=si.BASE_SEED + 701)
    _, k2, _ = si.full(w2)
    print("[case] no-alloc K pre-pass, second call B2 H2 N1300 D64 per-token scales", flush=True)
    ref2, got2 = both_calls(k2, 1)
    assert_same_bits(ref2, got2, "second call")
    kq, ks, km = oracle.smooth_quant_k(k2, 1)
    assert np.array_equal(got2[0].cpu().numpy(), kq)
    assert np.array_equal(bits(got2[1].cpu().numpy()), bits(ks)) and np.array_equal(bits(got2[2].cpu().numpy()), bits(km))
    # and a short sequence, which needs no scratch at all
    w3 = si.custom("noalloc_short", 1, 2, 300, 128, False, 128, 64, seed=si.BASE_SEED + 702)
    _, k3, _ = si.full(w3)
    ref3, got3 = both_calls(k3, 64)
    assert_same_bits(ref3, got3, "short sequence")


def test_shapes_beyond_the_static_scratch_are_refused_before_any_launch():
    # 65535 slabs x 2 partial sums x 128 channels x 8 bytes = 134 MB of partial sums: far beyond 4 MiB
    assert sage.sage_smooth_quant_k_workspace(255, 257, 1024, 128) > sage.NOALLOC_SCRATCH_BYTES
    lib = sage.load()
    good = 0x1000        # never dereferenced: the size check comes before any launch
    assert lib.sage_smooth_quant_k_noalloc(good, good, good, good, 255, 257, 1024, 128, 64, None) == 8
    assert sage.sage_status_string(8).startswith("SAGE_ERR_SCRATCH")
    # the headline and the long-context shapes fit
    for B, H, N, D in ((1, 32, 16384, 128), (1, 8, 131072, 128), (2, 30, 17776, 64), (4, 32, 4096, 128)):
        assert sage.sage_smooth_quant_k_workspace(B, H, N, D) <= sage.NOALLOC_SCRATCH_BYTES
