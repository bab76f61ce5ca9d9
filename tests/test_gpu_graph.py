"""The library calls enqueue kernels only (no allocation, no memset, no synchronization), so a
caller may capture them into a HIP graph.  Every replay must reproduce the eager result bit for bit,
also after the inputs changed in place and with eager work between the replays."""
import numpy as np
import pytest
import torch

import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block_q,block_k,rope,pv8", [(128, 64, False, False), (1, 1, False, False), (128, 64, True, False),
                                                      (128, 64, False, True)])
def test_graph_replays_equal_eager_runs(block_q, block_k, rope, pv8):
    print(f"[case] graph capture blocks {block_q}x{block_k} rope={rope} int8_pv={pv8}", flush=True)
    w = si.custom("graph", 2, 3, 457, 128, True, 128, 64, seed=si.BASE_SEED + 80)
    B, H, N, D = w.B, w.H, w.N, w.D
    inputs = [si.full(si.custom("graph", B, H, N, D, True, 128, 64, seed=si.BASE_SEED + 80 + i)) for i in range(3)]
    qd, kd, vd = (torch.empty((B, H, N, D), dtype=torch.float16, device="cuda") for _ in range(3))
    nq, nk = (N + block_q - 1) // block_q, (N + block_k - 1) // block_k
    q_i8 = torch.empty((B, H, N, D), dtype=torch.int8, device="cuda"); k_i8 = torch.empty_like(q_i8)
    q_scale = torch.empty((B, H, nq), dtype=torch.float32, device="cuda")
    k_scale = torch.empty((B, H, nk), dtype=torch.float32, device="cuda")
    k_mean = torch.empty((B, H, D), dtype=torch.float32, device="cuda")
    ws = torch.empty(sage.sage_smooth_quant_k_workspace(B, H, N, D) // 8, dtype=torch.int64, device="cuda")
    out = torch.empty((B, H, N, D), dtype=torch.float16, device="cuda")
    v_i8t = torch.empty((B, H, D, sage.sage_quant_v_pitch(N)), dtype=torch.int8, device="cuda")
    v_scale = torch.empty((B, H, D), dtype=torch.float32, device="cuda")
    ws_v = torch.empty(sage.sage_quant_v_workspace(B, H, N, D) // 4, dtype=torch.int32, device="cuda")
    pos = torch.arange(N, dtype=torch.float64, device="cuda")[:, None]
    freq = 10000.0 ** (-2.0 * torch.arange(D // 2, dtype=torch.float64, device="cuda") / D)[None, :]
    cs, sn = torch.cos(pos * freq).float().contiguous(), torch.sin(pos * freq).float().contiguous()

    def step():
        if rope:
            sage.sage_rope_smooth_quant_k(kd, cs, sn, block_k, k_i8, k_scale, k_mean, ws)
            sage.sage_rope_quant_q(qd, cs, sn, w.sm_scale, block_q, q_i8, q_scale)
        else:
            sage.sage_smooth_quant_k(kd, block_k, k_i8, k_scale, k_mean, ws)
            sage.sage_quant_q(qd, w.sm_scale, block_q, q_i8, q_scale)
        if pv8:
            sage.sage_quant_v(vd, v_i8t, v_scale, ws_v)
            sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, True, w.sm_scale, block_q, block_k, out)
        else:
            sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, vd, True, w.sm_scale, block_q, block_k, out)

    def set_inputs(i):
        q, k, v = inputs[i]
        qd.copy_(to_dev(q)); kd.copy_(to_dev(k)); vd.copy_(to_dev(v))

    eager = []
    for i in range(3):
        set_inputs(i)
        step()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in (k_i8, k_scale, k_mean, q_i8, q_scale, out, v_i8t, v_scale)])
    assert not torch.equal(eager[0][5], eager[1][5])

    set_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for i in (1, 2, 0, 1):
        set_inputs(i)
        for t in (k_i8, k_scale, k_mean, q_i8, q_scale, out, ws, v_i8t, v_scale, ws_v):
            t.fill_(1)                            # eager work between replays; stale outputs must not survive
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        outs = (k_i8, k_scale, k_mean, q_i8, q_scale, out) + ((v_i8t, v_scale) if pv8 else ())
        for got, want in zip(outs, eager[i]):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), f"replay with inputs {i} differs from the eager run"


def test_graph_replays_of_a_decode_step_with_the_keys_split():
    """A decode step -- quantize a few new queries, attend to all keys with the keys split over
    workgroups -- captured once and replayed with other queries; the workspace is dirtied between replays."""
    print("[case] graph capture of sage_quant_q + sage_attn_cross_split_fwd", flush=True)
    B, H, Nq, Nkv, D, chunks = 2, 3, 4, 2000, 128, 3
    wk = si.custom("graph_split_k", B, H, Nkv, D, False, seed=si.BASE_SEED + 90)
    _, k, v = si.full(wk)
    queries = [si.full(si.custom("graph_split_q", B, H, Nq, D, False, seed=si.BASE_SEED + 91 + i))[0] for i in range(3)]
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(to_dev(k), 64)
    vd = to_dev(v)
    qd = torch.empty((B, H, Nq, D), dtype=torch.float16, device="cuda")
    q_i8 = torch.empty((B, H, Nq, D), dtype=torch.int8, device="cuda")
    q_scale = torch.empty((B, H, 1), dtype=torch.float32, device="cuda")
    out = torch.empty((B, H, Nq, D), dtype=torch.float16, device="cuda")
    assert sage.sage_attn_split_count(B, H, Nq, Nkv, True, chunks) == chunks
    ws = torch.empty(sage.sage_attn_split_workspace(B, H, Nq, Nkv, D, True, chunks), dtype=torch.uint8, device="cuda")

    def step():
        sage.sage_quant_q(qd, wk.sm_scale, 128, q_i8, q_scale)
        sage.sage_attn_cross_split_fwd(q_i8, q_scale, k_i8, k_scale, vd, True, wk.sm_scale, 128, 64, chunks, out, ws)

    eager = []
    for q in queries:
        qd.copy_(to_dev(q))
        step()
        torch.cuda.synchronize()
        eager.append(out.clone())
    assert not torch.equal(eager[0], eager[1])

    qd.copy_(to_dev(queries[0]))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for i in (1, 2, 0, 1):
        qd.copy_(to_dev(queries[i]))
        for t in (q_i8, q_scale, out, ws):
            t.fill_(1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager[i].view(torch.int16)), f"replay with queries {i} differs from the eager run"
