"""sage_attn_clock_debug: the attention kernel built with its two counters (a measurement hook).  Its output
must be sage_attn_fwd's kernel's, bit for bit -- the counters may not change what is computed -- and what it
reports must make sense: every wavefront of every workgroup leaves a row, visits the key tiles the mask leaves
it, and the two counters give a clock a gfx950 can hold."""
import numpy as np
import pytest
import torch

import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

# (name, B, H, N, causal, block_q, block_k)
CASES = [
    ("full_ragged", 1, 3, 2049, False, 128, 64),
    ("causal_ragged", 2, 2, 1000, True, 64, 128),
    ("causal_long", 1, 2, 4608, True, 128, 64),
]


@pytest.mark.parametrize("name,B,H,N,causal,bq,bk", CASES, ids=[c[0] for c in CASES])
def test_clock_debug_matches_the_plain_kernel(name, B, H, N, causal, bq, bk):
    print(f"[case] clock debug {name} B{B} H{H} N{N} causal={causal} scales {bq}x{bk}", flush=True)
    w = si.custom(name, B, H, N, 128, causal, seed=si.BASE_SEED + 1200 + len(name))
    q, k, v = si.full(w)
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(to_dev(k), bk)
    q_i8, q_scale = sage.sage_quant_q(to_dev(q), w.sm_scale, bq)
    vd = to_dev(v)
    o_plain = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, vd, causal, w.sm_scale, bq, bk)
    o_probe, clocks = sage.sage_attn_clock_debug(q_i8, q_scale, k_i8, k_scale, vd, causal=causal, block_q=bq, block_k=bk)
    torch.cuda.synchronize()
    a, b = o_plain.cpu().numpy().astype(np.float32), o_probe.cpu().numpy().astype(np.float32)
    # the plain call may have picked the 128-row workgroup shape: the same arithmetic per row, in the same order
    assert np.array_equal(a, b), f"{name}: outputs differ, max {np.abs(a - b).max()}"
    c = clocks.cpu().numpy()
    tiles_q = (N + 255) // 256
    assert c.shape == (B * H * tiles_q * 8, 4)
    assert (c[:, 0] > 0).all() and (c[:, 1] > 0).all(), "every wavefront leaves its counters"
    ghz = c[:, 0].sum() / c[:, 1].sum() * 0.1
    assert 0.3 < ghz < 2.6, f"{name}: implied clock {ghz:.2f} GHz"
    # key tiles per wavefront: all of them without mask; up to the wavefront's last row when causal
    per = c.reshape(B * H, tiles_q, 8, 4)
    all_tiles = (N + 63) // 64
    for rank in range(tiles_q):                       # workgroups are numbered from the last query tile
        qt = tiles_q - 1 - rank
        for wv in range(8):
            last_row = qt * 256 + wv * 32 + 31
            want = min(all_tiles, last_row // 64 + 1) if causal else all_tiles
            assert (per[:, rank, wv, 3] == want).all(), f"{name}: tile count of query tile {qt}, wavefront {wv}"
    assert (c[:, 2] >= 1).all() and (c[:, 2] <= c[:, 3]).all(), "a maximum is raised at least on the first tile"


def test_clock_debug_refuses_what_it_is_not_built_for():
    q = torch.zeros((1, 1, 256, 64), dtype=torch.int8, device="cuda")
    s = torch.ones((1, 1, 2), dtype=torch.float32, device="cuda")
    v = torch.zeros((1, 1, 256, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(sage.SageError):
        sage.sage_attn_clock_debug(q, s, q, s, v)               # D = 64
    q = torch.zeros((1, 1, 256, 128), dtype=torch.int8, device="cuda")
    s = torch.ones((1, 1, 256), dtype=torch.float32, device="cuda")
    v = torch.zeros((1, 1, 256, 128), dtype=torch.float16, device="cuda")
    with pytest.raises(sage.SageError):
        sage.sage_attn_clock_debug(q, s, q, s, v, block_q=1, block_k=1)     # one scale per key token
