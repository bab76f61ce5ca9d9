"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Pre-pass: every INT8 code, scale and mean of the whole tensor, bit-exact.
Attention: Q blocks sampled from several heads (first, last, diagonal-heavy, random); each block's
output depends only on K^, V and the scales, so the oracle computes exactly those rows.
Int32 scores: the dump of one head, compared on sampled rows."""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import assert_output_close, bits, to_dev

pytestmark = pytest.mark.gpu

CASES = [("cfg2_image", 2, 6), ("cfg3_prefill16k", 2, 6), ("cfg4_video", 2, 5), ("cfg5_prefill128k", 1, 4),
         ("shape_llm_1536", 2, 12), ("shape_image_7285", 2, 8), ("shape_image_1105", 2, 9), ("shape_vit_197", 2, 2)]


def sample_blocks(Tm, n, seed):
    g = np.random.default_rng(seed)
    picks = {0, Tm - 1, Tm // 2}
    while len(picks) < min(n, Tm):
        picks.add(int(g.integers(0, Tm)))
    return sorted(picks)


@pytest.mark.parametrize("name,n_heads,n_blocks", CASES, ids=[c[0] for c in CASES])
def test_full_size_parity(name, n_heads, n_blocks):
    w = si.WORKLOADS[name]
    t0 = time.time()
    print(f"[case] {name} B{w.B} H{w.H} N{w.N} D{w.D} causal={w.causal}", flush=True)
    q, k, v = si.full(w)
    print(f"  inputs generated {time.time() - t0:.1f}s", flush=True)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(kd, w.block_k)
    q_i8, q_scale = sage.sage_quant_q(qd, w.sm_scale, w.block_q)
    o = sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, vd, w.causal, w.sm_scale, w.block_q, w.block_k)
    torch.cuda.synchronize()
    print(f"  gpu done {time.time() - t0:.1f}s", flush=True)

    # ---- pre-pass, whole tensors
    kq, ks, km = oracle.smooth_quant_k(k, w.block_k)
    qq, qs = oracle.quant_q(q, w.sm_scale, w.block_q)
    print(f"  oracle pre-pass {time.time() - t0:.1f}s", flush=True)
    assert np.array_equal(bits(k_mean.cpu().numpy()), bits(km))
    assert np.array_equal(bits(k_scale.cpu().numpy()), bits(ks))
    assert np.array_equal(bits(q_scale.cpu().numpy()), bits(qs))
    assert np.array_equal(k_i8.cpu().numpy(), kq)
    assert np.array_equal(q_i8.cpu().numpy(), qq)

    # ---- attention on sampled Q blocks
    Tm = (w.N + w.block_q - 1) // w.block_q
    o_host = o.cpu().numpy()
    heads = [(0, 0), (w.B - 1, w.H - 1)][:n_heads]
    for hi, (b, h) in enumerate(heads):
        blocks = sample_blocks(Tm, n_blocks, 100 + hi)
        ref = oracle.attn_l2_slab(qq[b, h], qs[b, h], kq[b, h], ks[b, h], v[b, h], w.causal,
                                  w.block_q, w.block_k, q_blocks=blocks)
        rows = np.concatenate([np.arange(i * w.block_q, min(w.N, (i + 1) * w.block_q)) for i in blocks])
        err, cos = assert_output_close(o_host[b, h][rows], ref[rows], f"{name} head ({b},{h}) blocks {blocks}")
        print(f"  head ({b},{h}) blocks {blocks}: max_abs {err:.2e} cos {cos:.7f}  {time.time() - t0:.1f}s", flush=True)

    # ---- int32 scores of one head on sampled rows
    b, h = heads[-1]
    q1, k1 = q_i8[b:b + 1, h:h + 1].contiguous(), k_i8[b:b + 1, h:h + 1].contiguous()
    for wg_rows in (256, 128):       # both workgroup shapes of the attention kernel
        s_dev = sage.sage_attn_qk_i32_debug(q1, k1, block_q=w.block_q, block_k=w.block_k, wg_rows=wg_rows)
        torch.cuda.synchronize()
        for row0 in sorted({0, (w.N // 2) // 32 * 32, max(0, w.N - 40)}):
            nrows = min(40, w.N - row0)
            ref = oracle.qk_i32(qq[b, h], kq[b, h], row0, nrows)
            got = s_dev[0, 0, row0:row0 + nrows].cpu().numpy()
            assert np.array_equal(got, ref), f"int32 scores differ at rows {row0}.. (workgroup rows {wg_rows})"
        del s_dev
    print(f"  int32 dump ok {time.time() - t0:.1f}s", flush=True)
