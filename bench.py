#!/usr/bin/env python3
"""Benchmark of the SageAttention forward hot path on one MI355X.

A step = one pass of the whole path (K pre-pass, Q pre-pass, fused attention) over one batch of
synthetic input that is already resident in HBM.  Prints ONE JSON line.

  metric   attention TOPS = 4*B*H*N^2*D / t (halved when causal), t = time of one step
  roofline the fused attention kernel against the dense INT8 MFMA peak, its duration measured
           with HIP events on the launch stream inside the timed region
  cpu_baseline the CPU oracle timed on a bounded sample of the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0      # MI355X dense INT8 MFMA, published
FP16_PEAK_TFLOPS = 2500.0    # MI355X dense FP16 MFMA, published
HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published



def profiled_traffic(workload: str, pv_int8: bool):
    """HBM bytes per attention launch from the hardware counters (FETCH_SIZE and WRITE_SIZE, one profiler
    run each, scaled by what the same counter reads for a 1 GiB copy kernel).  The profiler cannot run
    inside this script, so the figure is read from the committed summary of that run under profiles/
    (its line "traffic_bytes_per_launch = ..."); None when there is no summary for the workload."""
    import re
    name = f"hotpath_{workload}{'_int8_pv' if pv_int8 else ''}_hbm_traffic.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


# Probes of sage_microbench (include/sage.h): operations per instruction group
PROBE_OPS = {0: 8 * 65536.0, 1: 8 * 32768.0, 2: 8 * 65536.0 + 16 * 32768.0, 4: 8 * 32768.0, 5: 8 * 32768.0,
             6: 8 * 65536.0 + 16 * 32768.0, 9: 8 * 65536.0 + 16 * 32768.0,
             15: 8 * 65536.0 + 16 * 32768.0, 16: 8 * 65536.0 + 16 * 32768.0, 17: 8 * 32768.0, 18: 8 * 65536.0, 19: 8 * 65536.0 + 16 * 32768.0, 20: 2 * (8 * 65536.0 + 16 * 32768.0),
             11: 16 * 32768.0, 12: 16 * 32768.0, 13: 16 * 32768.0, 14: 8 * 65536.0}      # kinds 11 to 13: the 16 P~V instructions only
PROBE_NAMES = {0: "INT8 32x32x32 stream", 1: "FP16 32x32x16 stream", 2: "attention mix: 8 INT8 + 16 FP16, matrix only",
               3: "softmax chunks only (24 per group)", 4: "FP16 matrix instruction + softmax chunk, one stream",
               5: "FP16 matrix stream and softmax stream on separate wavefronts of a SIMD",
               6: "attention step: 8 INT8 + 16 FP16 + 16 chunks + 8 maxima, one stream",
               7: "LDS reads of 16 B per lane (K^ operands), 24 KB per group",
               8: "transposing LDS reads of 8 B per lane (V^T operands), 24 KB per group",
               9: "attention step as kind 6, every matrix operand read from LDS 3 ahead",
               10: "16 x 4x4x4 FP16 matrix instruction (the row-sum instruction)",
               11: "4 x (4 FP16 32x32x16 + 2 of the 4x4x4): P~V with row sums",
               12: "4 x (4 FP16 32x32x16 + 1 FP16 16x16x32)",
               13: "4 x (4 + 1 FP16 32x32x16)",
               14: "INT8 32x32x32 stream, one accumulator (dependent chain)",
               15: "attention step in the kernel's order: maxima, chunks behind 16 instructions, row sums",
               16: "kind 15 with the chunks spread over 20 instructions",
               17: "FP16 16x16x32 stream (16 instructions = kind 1's operations)",
               18: "INT8 16x16x64 stream (16 instructions = kind 0's operations)",
               19: "kind 15 with the 16x16 instructions (every LDS operand feeds two of them)",
               20: "kind 19 for 64 queries per wavefront (every LDS operand feeds four instructions)"}
# matrix-pipe clocks per group (32 per 32x32 instruction) -- what a fully busy pipe needs
PROBE_PIPE_CLOCKS = {0: 256, 1: 256, 2: 768, 4: 256, 5: 256, 6: 768, 9: 768, 11: 512, 12: 512, 13: 512, 14: 256, 15: 768, 16: 768, 17: 256, 18: 256, 19: 768, 20: 1536}
# LDS bytes a wavefront reads per group (kinds 7 to 9)
PROBE_LDS_BYTES = {7: 24 * 1024, 8: 24 * 1024, 9: 24 * 1024, 15: 24 * 1024, 16: 24 * 1024, 19: 24 * 1024, 20: 24 * 1024}


def run_probe(sage, torch, data, kind, waves, seconds, workgroups=1024):
    """One probe launch sized to last about `seconds`; returns (ms, TOPS or None, mean shader-clock ticks per
    group, implied clock in GHz from the two in-kernel counters)."""
    def launch(iters):
        out = torch.zeros((workgroups * 4 * waves, 4), dtype=torch.int64, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        sage.sage_microbench(kind, waves, workgroups, iters, data, out)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1), out
    ms, _ = launch(200)
    iters = int(max(200, min(2.0e8, 200 * seconds * 1e3 / max(ms, 1e-3))))
    launch(iters)                      # warm
    ms, out = launch(iters)
    o = out.cpu().numpy().astype(np.float64)
    wavefronts = workgroups * 4 * waves
    matrix_waves = wavefronts // 2 if kind == 5 else wavefronts
    tops = PROBE_OPS[kind] * iters * matrix_waves / (ms * 1e-3) / 1e12 if kind in PROBE_OPS else None
    ticks = float(o[:, 0].mean()) / iters
    # the constant-rate counter runs at 100 MHz
    ghz = float((o[:, 0] / np.maximum(o[:, 1], 1.0)).mean()) * 0.1
    return ms, tops, ticks, ghz, iters


def microbench(seconds: float):
    """What the matrix pipe of this chip sustains with the attention kernel's own instructions (table on
    stdout; not part of the one-line benchmark contract).  1024 workgroups = 4 per compute unit at one
    wavefront per SIMD each, i.e. every SIMD holds 4 (or 8) probe wavefronts."""
    import torch

    import paper_2410_02367_amd as sage

    torch.cuda.set_device(0)
    g = torch.Generator(device="cuda").manual_seed(20241002)
    data = torch.randint(-2 ** 31, 2 ** 31 - 1, (1024,), generator=g, device="cuda", dtype=torch.int64).to(torch.int32)
    print(f"instruction-stream probes, about {seconds:g} s per launch, random operand bits; "
          f"nominal peaks: INT8 {INT8_PEAK_TOPS:.0f} TOPS, FP16 {FP16_PEAK_TFLOPS:.0f} TFLOP/s at 2.4 GHz")
    print("%-4s %-78s %5s %9s %9s %8s %10s %9s %8s" % ("kind", "probe", "waves", "ms", "TOPS", "% peak", "ticks/grp", "pipe busy", "GHz"))
    for kind, waves in ((0, 1), (0, 2), (1, 1), (1, 2), (2, 1), (2, 2), (3, 1), (3, 2), (4, 1), (4, 2), (5, 2), (6, 1), (6, 2), (7, 1), (7, 2), (8, 1), (8, 2), (9, 1), (9, 2), (10, 1), (11, 1), (11, 2), (12, 1), (12, 2), (13, 1), (14, 1), (14, 2), (15, 1), (15, 2), (16, 1), (16, 2), (17, 1), (17, 2), (18, 1), (18, 2), (19, 1), (19, 2), (20, 1), (20, 2)):
        # 256 workgroups: one per compute unit, `waves` wavefronts per SIMD
        ms, tops, ticks, ghz, iters = run_probe(sage, torch, data, kind, waves, seconds, workgroups=256)
        peak = {0: INT8_PEAK_TOPS, 14: INT8_PEAK_TOPS, 18: INT8_PEAK_TOPS, 17: FP16_PEAK_TFLOPS, 1: FP16_PEAK_TFLOPS, 4: FP16_PEAK_TFLOPS, 5: FP16_PEAK_TFLOPS, 11: FP16_PEAK_TFLOPS,
                12: FP16_PEAK_TFLOPS, 13: FP16_PEAK_TFLOPS}.get(kind, INT8_PEAK_TOPS)
        busy = PROBE_PIPE_CLOCKS[kind] * (1 if kind == 5 else waves) / ticks if kind in PROBE_PIPE_CLOCKS else float("nan")
        lds = ""
        if kind in PROBE_LDS_BYTES:     # LDS bytes per clock and compute unit: 4 SIMDs x waves wavefronts
            per_clock = PROBE_LDS_BYTES[kind] * 4 * waves * iters / (ms * 1e-3 * ghz * 1e9)
            lds = "  LDS %.1f B/clk/CU" % per_clock
        print("%-4d %-78s %5d %9.2f %9s %8s %10.1f %9.3f %8.3f%s" % (
            kind, PROBE_NAMES[kind], waves, ms, "%.0f" % tops if tops else "-",
            "%.1f" % (100.0 * tops / peak) if tops else "-", ticks, busy, ghz, lds), flush=True)


def clock_study(workload: str):
    """The attention kernel (FP16 P~V, D = 128) on the workload's tensors, with the key scales multiplied by a
    factor: what is computed per tile stays the same, the spread of the scores -- and with it the bit patterns
    the softmax and the second product work on -- changes.  Per factor: time of the plain kernel, and from its
    measurement build the clock the chip held, the clocks per tile and the rare-path count (table on stdout;
    not part of the one-line benchmark contract)."""
    import torch

    import paper_2410_02367_amd as sage
    import sage_inputs as si

    w = si.WORKLOADS[workload]
    torch.cuda.set_device(0)
    qd, kd, vd = (torch.from_numpy(a).cuda() for a in si.full(w))
    B, H, N, D = w.B, w.H, w.N, w.D
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(kd, w.block_k)
    q_i8, q_scale = sage.sage_quant_q(qd, w.sm_scale, w.block_q)
    out = torch.empty_like(qd)
    ops = 4.0 * B * H * N * N * D
    print(f"attention kernel on {w.name} (B={B} H={H} N={N} D={D}), key scales x factor; "
          f"TOPS = 4 B H N^2 D (halved if causal) / time; pipe busy = 2 * 832 clocks per tile / clocks per tile and wavefront")
    print("%-8s %-7s %8s %7s %7s %14s %10s %12s" % ("causal", "factor", "ms", "TOPS", "GHz", "clocks/tile/wf", "pipe busy", "raises/wf"))
    for causal in (False, True):
        for factor in (1e-9, 0.25, 1.0, 4.0, 100.0):
            ks = (k_scale * factor).contiguous()
            for _ in range(3):
                sage.sage_attn_fwd(q_i8, q_scale, k_i8, ks, vd, causal, w.sm_scale, w.block_q, w.block_k, out)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                sage.sage_attn_fwd(q_i8, q_scale, k_i8, ks, vd, causal, w.sm_scale, w.block_q, w.block_k, out)
            e1.record()
            torch.cuda.synchronize()
            ms = [e0.elapsed_time(e1) / 10]
            for _ in range(10):      # back to back, so that the last launch sees the clock the load settles at
                _, clocks = sage.sage_attn_clock_debug(q_i8, q_scale, k_i8, ks, vd, out, causal, w.block_q, w.block_k)
            torch.cuda.synchronize()
            c = clocks.cpu().numpy().astype(np.float64)
            c = c[c[:, 3] > 0]
            t = float(np.mean(ms))
            print("%-8s %-7g %8.3f %7.0f %7.3f %14.0f %10.3f %12.1f" % (
                causal, factor, t, ops / (2 if causal else 1) / (t * 1e-3) / 1e12, c[:, 0].sum() / c[:, 1].sum() * 0.1,
                c[:, 0].sum() / c[:, 3].sum(), 2.0 * 832.0 * c[:, 3].sum() / c[:, 0].sum(), c[:, 2].mean()), flush=True)


def cpu_baseline(w, seconds_budget=20.0, per_token=False, gpu_out_head0=None, pv_int8=False):
    """Oracle (Algorithm-1 level, as it stands) on one head of the workload: the full pre-pass of that
    head plus a spread of Q blocks, scaled to the head's block-pair count."""
    import numpy as np

    import oracle
    import sage_inputs as si

    q, k, v = si.slab(w, 0, 0)
    t0 = time.perf_counter()
    gran = dict(gran_q=1, gran_k=1) if per_token else {}
    kq, ks, km = oracle.smooth_quant_k(k[None, None], 1 if per_token else w.block_k)
    qq, qs = oracle.quant_q(q[None, None], w.sm_scale, 1 if per_token else w.block_q)
    if pv_int8:
        vq, vs = oracle.quant_v(v[None, None])

        def run(blocks):
            return oracle.attn_pv8_slab(qq[0, 0], qs[0, 0], kq[0, 0], ks[0, 0], vq[0, 0], vs[0, 0], w.causal,
                                        w.block_q, w.block_k, q_blocks=blocks, **gran)
    else:
        def run(blocks):
            return oracle.attn_l2_slab(qq[0, 0], qs[0, 0], kq[0, 0], ks[0, 0], v, w.causal, w.block_q, w.block_k,
                                       q_blocks=blocks, **gran)
    t_pre = time.perf_counter() - t0
    Tm = (w.N + w.block_q - 1) // w.block_q
    Tn = (w.N + w.block_k - 1) // w.block_k

    def pairs(i):
        if not w.causal:
            return Tn
        last_row = min(w.N, (i + 1) * w.block_q) - 1
        return last_row // w.block_k + 1

    total_pairs = sum(pairs(i) for i in range(Tm))
    # probe one block to size the sample
    mid = Tm // 2
    t0 = time.perf_counter()
    run([mid])
    t_one = time.perf_counter() - t0
    per_pair = t_one / pairs(mid)
    threads = oracle.num_threads()
    avg_pairs = total_pairs / Tm
    n_blocks = int(max(threads, min(Tm, seconds_budget * threads / max(per_pair * avg_pairs, 1e-9))))
    n_blocks = max(threads, (n_blocks // threads) * threads)
    blocks = sorted(set(np.linspace(0, Tm - 1, n_blocks).round().astype(int).tolist()))
    t0 = time.perf_counter()
    o_l2 = run(blocks)
    t_blocks = time.perf_counter() - t0
    # accuracy of the method (not timed): the GPU's rows of three Q blocks of this head against exact
    # fp64 attention on the fp16 inputs, with the paper's three metrics; the oracle's rows beside them
    accuracy = None
    if gpu_out_head0 is not None:
        acc_blocks = sorted({blocks[0], blocks[len(blocks) // 2], blocks[-1]})
        rows = np.concatenate([np.arange(i * w.block_q, min(w.N, (i + 1) * w.block_q)) for i in acc_blocks])
        exact = np.concatenate([oracle.attn_l0_slab(q, k, v, w.causal, w.sm_scale, int(i * w.block_q),
                                                    int(min(w.N, (i + 1) * w.block_q) - i * w.block_q)) for i in acc_blocks])
        mg = oracle.accuracy_metrics(exact, gpu_out_head0[rows])
        mo = oracle.accuracy_metrics(exact, o_l2[rows])
        accuracy = {"reference": "exact fp64 attention on the fp16 inputs, %d rows of head 0" % len(rows),
                    "gpu": {key: float(mg[key]) for key in ("cos", "rel_l1", "rmse")},
                    "oracle": {key: float(mo[key]) for key in ("cos", "rel_l1", "rmse")},
                    "gpu_vs_oracle_max_abs": float(np.abs(gpu_out_head0[rows].astype(np.float64) - o_l2[rows].astype(np.float64)).max())}
    sampled_pairs = sum(pairs(i) for i in blocks)
    t_head = t_pre + t_blocks * total_pairs / sampled_pairs
    ops_head = w.ops / (w.B * w.H)
    return {
        "value": ops_head / t_head / 1e12,
        "unit": "TOPS",
        "cores": threads,
        "kind": "oracle",
        "sample": (f"1 of {w.B * w.H} heads: full pre-pass ({t_pre:.2f}s) + {len(blocks)} of {Tm} Q blocks "
                   f"({t_blocks:.2f}s, {sampled_pairs} of {total_pairs} block pairs), scaled to the head"),
        "accuracy": accuracy,
    }


def sweep(per_token: bool, pv_int8: bool = False):
    """Attention-kernel speed over sequence length, head dimension and mask (the axes of the paper's
    kernel-speed figures): N(0,1) inputs, H = 32, B = max(1, 16384 / N).  Prints one table row per
    shape; not part of the one-line benchmark contract."""
    import torch

    import paper_2410_02367_amd as sage

    torch.cuda.set_device(0)
    bq, bk = (1, 1) if per_token else (128, 64)
    print("scales: " + ("one per token" if per_token else "per block 128 x 64")
          + ("; INT8 second product" if pv_int8 else "; FP16 second product"))
    print("%7s %4s %7s %3s  %10s %9s" % ("N", "D", "causal", "B", "attn ms", "TOPS"))
    for D in (64, 128):
        for causal in (False, True):
            for N in (1024, 2048, 4096, 8192, 16384, 32768):
                B, H = max(1, 16384 // N), 32
                g = torch.Generator(device="cuda").manual_seed(N + D)
                q, k, v = (torch.randn((B, H, N, D), generator=g, device="cuda", dtype=torch.float32).half() for _ in range(3))
                sm = float(D) ** -0.5
                k_i8, k_scale, _ = sage.sage_smooth_quant_k(k, bk)
                q_i8, q_scale = sage.sage_quant_q(q, sm, bq)
                out = torch.empty_like(v)
                if pv_int8:
                    v_i8t, v_scale = sage.sage_quant_v(v)

                    def attn():
                        sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, causal, sm, bq, bk, out)
                else:
                    def attn():
                        sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, v, causal, sm, bq, bk, out)
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                for _ in range(3):
                    attn()
                reps = 10
                ev[0].record()
                for _ in range(reps):
                    attn()
                ev[1].record()
                torch.cuda.synchronize()
                ms = ev[0].elapsed_time(ev[1]) / reps
                ops = 4.0 * B * H * N * N * D / (2 if causal else 1)
                print("%7d %4d %7s %3d  %10.3f %9.0f" % (N, D, causal, B, ms, ops / (ms * 1e-3) / 1e12), flush=True)
                del q, k, v, k_i8, q_i8, out


def cross(workload: str, nqs, pv_int8: bool = False):
    """Speed of sage_attn_cross_fwd and sage_attn_cross_split_fwd: the last Nq tokens of the workload's
    sequence as queries against all of its keys and values (chunked prefill / decode shapes; the mask,
    if causal, is aligned at the end); with pv_int8 the same for the calls with the INT8 second product.
    Prints one table row per Nq; not part of the one-line benchmark contract."""
    import torch

    import paper_2410_02367_amd as sage
    import sage_inputs as si

    w = si.WORKLOADS[workload]
    torch.cuda.set_device(0)
    q, k, v = si.full(w)
    kd, vd = torch.from_numpy(k).cuda(), torch.from_numpy(v).cuda()
    B, H, N, D = w.B, w.H, w.N, w.D
    k_i8, k_scale, _ = sage.sage_smooth_quant_k(kd, w.block_k)
    if pv_int8:
        v_i8t, v_scale = sage.sage_quant_v(vd)
    print(f"{w.name}: B={B} H={H} Nkv={N} D={D} causal={w.causal}, block_q={w.block_q} block_k={w.block_k}, "
          f"{'INT8' if pv_int8 else 'FP16'} second product; ops = 4 B H D x visible (query, key) pairs")
    print("%8s  %10s %9s   %7s %10s %9s" % ("Nq", "attn ms", "TOPS", "chunks", "split ms", "TOPS"))

    def timed(call):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        for _ in range(10):
            call()
        reps = 20
        ev[0].record()
        for _ in range(reps):
            call()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps

    for nq in nqs:
        qd = torch.from_numpy(np.ascontiguousarray(q[:, :, N - nq:])).cuda()
        q_i8, q_scale = sage.sage_quant_q(qd, w.sm_scale, w.block_q)
        out = torch.empty((B, H, nq, D), dtype=torch.float16, device="cuda")
        if pv_int8:
            whole = lambda: sage.sage_attn_pv_int8_cross_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, w.causal,
                                                             w.sm_scale, w.block_q, w.block_k, out)
        else:
            whole = lambda: sage.sage_attn_cross_fwd(q_i8, q_scale, k_i8, k_scale, vd, w.causal, w.sm_scale,
                                                     w.block_q, w.block_k, out)
        ms = timed(whole)
        pairs = float(nq) * N - (float(nq) * (nq - 1) / 2 if w.causal else 0.0)
        ops = 4.0 * B * H * D * pairs
        # the same with the keys cut into the number of chunks the library chooses (the *_cross_split_fwd call)
        n = sage.sage_attn_split_count(B, H, nq, N, w.causal, 0)
        ws = torch.empty(max(sage.sage_attn_split_workspace(B, H, nq, N, D, w.causal, 0), 16), dtype=torch.uint8, device="cuda")
        if pv_int8:
            split = lambda: sage.sage_attn_pv_int8_cross_split_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, w.causal,
                                                                   w.sm_scale, w.block_q, w.block_k, 0, out, ws)
        else:
            split = lambda: sage.sage_attn_cross_split_fwd(q_i8, q_scale, k_i8, k_scale, vd, w.causal, w.sm_scale,
                                                           w.block_q, w.block_k, 0, out, ws)
        ms_s = timed(split)
        print("%8d  %10.4f %9.0f   %7d %10.4f %9.0f" % (nq, ms, ops / (ms * 1e-3) / 1e12, n, ms_s, ops / (ms_s * 1e-3) / 1e12),
              flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg3_prefill16k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scales", choices=("block", "token"), default="block",
                    help="block: one scale per block_q / block_k tokens (Algorithm 1, the headline); "
                         "token: one scale per token of Q and K (the SAGEAttn-T kernel)")
    ap.add_argument("--pv", choices=("fp16", "int8"), default="fp16",
                    help="fp16: P~V in FP16 (Algorithm 1, the headline); int8: the INT8 second product of Section 4.3 "
                         "(SAGEAttn-vB, or -vT with --scales token): the step gains the per-channel pre-pass of V")
    ap.add_argument("--rope", action="store_true",
                    help="the pre-pass applies RoPE to Q and K on the fly (the fused calls of Section 4.6's "
                         "fusion trick); not the headline configuration")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph that holds one step (the library's calls only enqueue "
                         "kernels, so they can be captured); for the short-sequence shapes, where launches dominate")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line, print the attention kernel's speed over N = 1K..32K, "
                         "D = 64/128, with and without the causal mask")
    ap.add_argument("--cross", default=None,
                    help="instead of the benchmark line, time sage_attn_cross_fwd and sage_attn_cross_split_fwd with the "
                         "last Nq tokens of the workload as queries against all of its keys; comma-separated list of Nq")
    ap.add_argument("--rotate", type=int, default=1,
                    help="number of distinct input allocations used in turn (1 = every step reads the same buffers)")
    ap.add_argument("--prepass", choices=("separate", "fused"), default="fused",
                    help="fused: sage_quant_qk, both pre-passes in two launches (one for short sequences); "
                         "separate: sage_smooth_quant_k + sage_quant_q, the same work and the same bits in one launch more")
    ap.add_argument("--clock-study", action="store_true",
                    help="table: the attention kernel's time, clock and clocks per tile on the workload's tensors with the "
                         "key scales multiplied by several factors (the spread of the scores changes, the work does not)")
    ap.add_argument("--microbench", type=float, nargs="?", const=0.05, default=None, metavar="SECONDS",
                    help="instead of the benchmark line, print what the matrix pipe sustains with the attention "
                         "kernel's instructions (pure INT8 / FP16 streams, the attention mix, with and without the "
                         "softmax arithmetic), each probe launch lasting about SECONDS (default 0.05)")
    ap.add_argument("--sustain", type=float, default=1.0,
                    help="after the timed steps, keep stepping for this many seconds and report that rate as well "
                         "(extra key 'sustained'; 0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain elementwise copy kernel of 1 GiB before the warm-up, so that a "
                         "hardware-counter run holds a kernel of known HBM traffic beside the library's kernels")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2410_02367_amd as sage
    import sage_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)
    sage.load()
    if args.rotate < 1 or (args.graph and args.rotate > 1):
        print("bench.py: --rotate must be >= 1, and 1 with --graph (a captured step reads fixed buffers)", file=sys.stderr)
        sys.exit(2)
    if args.microbench is not None:
        microbench(args.microbench)
        return
    if args.clock_study:
        clock_study(args.workload)
        return
    if args.sweep:
        sweep(args.scales == "token", args.pv == "int8")
        return
    if args.cross:
        cross(args.workload, [int(x) for x in args.cross.split(",")], args.pv == "int8")
        return
    w = si.WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    q, k, v = si.full(w)
    qd, kd, vd = (torch.from_numpy(a).cuda() for a in (q, k, v))
    del q, k, v
    # --rotate R: R distinct allocations of the inputs, used in turn, so that no step finds its inputs
    # in the last-level cache because the step before read the same addresses
    inputs = [(qd, kd, vd)] + [(qd.clone(), kd.clone(), vd.clone()) for _ in range(args.rotate - 1)]
    B, H, N, D = w.B, w.H, w.N, w.D
    per_token = args.scales == "token"
    bq, bk = (1, 1) if per_token else (w.block_q, w.block_k)
    nbq, nbk = (N + bq - 1) // bq, (N + bk - 1) // bk
    q_i8 = torch.empty((B, H, N, D), dtype=torch.int8, device="cuda")
    k_i8 = torch.empty_like(q_i8)
    q_scale = torch.empty((B, H, nbq), dtype=torch.float32, device="cuda")
    k_scale = torch.empty((B, H, nbk), dtype=torch.float32, device="cuda")
    k_mean = torch.empty((B, H, D), dtype=torch.float32, device="cuda")
    ws = torch.empty(sage.sage_smooth_quant_k_workspace(B, H, N, D) // 8, dtype=torch.int64, device="cuda")
    out = torch.empty((B, H, N, D), dtype=torch.float16, device="cuda")
    stream = torch.cuda.current_stream()
    pv_int8 = args.pv == "int8"
    if pv_int8:
        v_i8t = torch.empty((B, H, D, sage.sage_quant_v_pitch(N)), dtype=torch.int8, device="cuda")
        v_scale = torch.empty((B, H, D), dtype=torch.float32, device="cuda")
        ws_v = torch.empty(sage.sage_quant_v_workspace(B, H, N, D) // 4, dtype=torch.int32, device="cuda")
    if args.rope:
        pos = torch.arange(N, dtype=torch.float64, device="cuda")[:, None]
        freq = 10000.0 ** (-2.0 * torch.arange(D // 2, dtype=torch.float64, device="cuda") / D)[None, :]
        rope_cos, rope_sin = torch.cos(pos * freq).float().contiguous(), torch.sin(pos * freq).float().contiguous()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]

    turn = [0]

    def step(i=None, stream=stream):
        qd, kd, vd = inputs[turn[0] % len(inputs)]
        turn[0] += 1
        if i is not None:
            ev[i][0].record(stream)
        if args.rope:
            sage.sage_rope_smooth_quant_k(kd, rope_cos, rope_sin, bk, k_i8, k_scale, k_mean, ws, stream)
            sage.sage_rope_quant_q(qd, rope_cos, rope_sin, w.sm_scale, bq, q_i8, q_scale, stream)
        elif args.prepass == "fused":
            sage.sage_quant_qk(qd, kd, w.sm_scale, bq, bk, q_i8, q_scale, k_i8, k_scale, k_mean, ws, stream)
        else:
            sage.sage_smooth_quant_k(kd, bk, k_i8, k_scale, k_mean, ws, stream)
            sage.sage_quant_q(qd, w.sm_scale, bq, q_i8, q_scale, stream)
        if pv_int8:
            sage.sage_quant_v(vd, v_i8t, v_scale, ws_v, stream)
        if i is not None:
            ev[i][1].record(stream)
        if pv_int8:
            sage.sage_attn_pv_int8_fwd(q_i8, q_scale, k_i8, k_scale, v_i8t, v_scale, w.causal, w.sm_scale, bq, bk, out, stream)
        else:
            sage.sage_attn_fwd(q_i8, q_scale, k_i8, k_scale, vd, w.causal, w.sm_scale, bq, bk, out, stream)
        if i is not None:
            ev[i][2].record(stream)

    if args.calibrate_copy:
        # y = x + 0 over 2^28 int32: reads 1 GiB and writes 1 GiB, nothing else
        cx = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
        cy = torch.empty_like(cx)
        torch.add(cx, 0, out=cy)
        torch.cuda.synchronize()
        del cx, cy

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            step(stream=side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(stream=side)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(args.steps):      # untimed eager steps: per-kernel durations for the roofline object
            step(i)
        torch.cuda.synchronize()
    else:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    attn_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    pre_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    assert bool(torch.isfinite(out[0, 0, :64].float()).all())

    # the same steps for about --sustain seconds: what the chip holds once clocks and power have settled
    sustained = None
    if args.sustain > 0 and not args.graph:
        n_sus = int(max(args.steps, min(20000, args.sustain * 1e3 / ms_per_step)))
        ts0 = time.perf_counter()
        for _ in range(n_sus):
            step()
        torch.cuda.synchronize()
        ts1 = time.perf_counter()
        sus_ms = (ts1 - ts0) * 1e3 / n_sus
        sustained = {"steps": n_sus, "seconds": ts1 - ts0, "ms_per_step": sus_ms,
                     "value": w.ops / (sus_ms * 1e-3) / 1e12, "unit": "TOPS"}

    # the attention kernel's own counters (its measurement build, same arithmetic): the clock the chip holds
    # while it runs, the clocks a wavefront spends per 64-key tile, and from them the share of the matrix
    # pipe's clocks that carry a matrix instruction (a tile is 24 instructions of 32 clocks and 4 of 16 per
    # wavefront at D = 128, two wavefronts share a SIMD's pipe)
    kernel_clock = None
    if not pv_int8 and not per_token and D == 128:
        for _ in range(10):      # back to back, so that the last launch sees the clock the load settles at
            _, clocks = sage.sage_attn_clock_debug(q_i8, q_scale, k_i8, k_scale, inputs[0][2], out, w.causal, bq, bk, stream)
        torch.cuda.synchronize()
        c = clocks.cpu().numpy().astype(np.float64)
        c = c[c[:, 3] > 0]
        kernel_clock = {"ghz": float(c[:, 0].sum() / c[:, 1].sum() * 0.1),
                        "clocks_per_tile_and_wavefront": float(c[:, 0].sum() / c[:, 3].sum()),
                        "matrix_pipe_busy": float(2.0 * 832.0 * c[:, 3].sum() / c[:, 0].sum()),
                        "raises_of_the_maximum_per_wavefront": float(c[:, 2].mean()),
                        "how": "sage_attn_clock_debug, last of ten launches back to back after the timed steps"}

    # what the matrix pipe sustains with this kernel's own instructions, measured now on this GPU:
    # the pure INT8 stream (the peak `frac` is quoted against, as measured) and the kernel's instruction
    # mix without anything else (the ceiling of this algorithm on this chip)
    g = torch.Generator(device="cuda").manual_seed(20241002)
    probe_data = torch.randint(-2 ** 31, 2 ** 31 - 1, (1024,), generator=g, device="cuda", dtype=torch.int64).to(torch.int32)
    _, int8_measured, _, int8_ghz, _ = run_probe(sage, torch, probe_data, 0, 2, 0.05, workgroups=256)
    mix_kind = 0 if pv_int8 else 2
    _, mix_measured, _, mix_ghz, _ = run_probe(sage, torch, probe_data, mix_kind, 2, 0.05, workgroups=256)
    # what a plain device-to-device copy of 1 GiB reaches on this GPU (read + written bytes per second): the
    # practical HBM rate the pre-pass is compared with, beside the published peak
    cx = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
    cy = torch.empty_like(cx)
    copy_ms = []
    for _ in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        cy.copy_(cx)
        e1.record()
        torch.cuda.synchronize()
        copy_ms.append(e0.elapsed_time(e1))
    copy_gbs = 2.0 * cx.numel() * 4 / (min(copy_ms[1:]) * 1e-3) / 1e9
    del cx, cy

    ops = w.ops
    value = ops / (ms_per_step * 1e-3) / 1e12
    attn_tops = ops / (attn_ms * 1e-3) / 1e12
    result = {
        "metric": "attention TOPS (4*B*H*N^2*D/t, halved if causal) at N=16K D=128; % MFMA peak",
        "value": value,
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 QK^T (int32 acc) + " + ("int8 PV (int32 acc)" if pv_int8 else "fp16 PV (fp32 acc)"),
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} H={H} N={N} D={D} causal={w.causal} fp16 in/out, "
                               + ("one scale per token of Q and K (SAGEAttn-T)" if per_token else
                                  f"block_q={w.block_q} block_k={w.block_k}")
                               + ("; RoPE applied inside the pre-pass" if args.rope else "")
                               + ("; timed as replays of a HIP graph of one step" if args.graph else "")
                               + ("; INT8 P~V (SAGEAttn-v%s)" % ("T" if per_token else "B") if pv_int8 else "")
                               + "; step = K pre-pass + Q pre-pass " + ("(sage_quant_qk) + " if args.prepass == "fused" and not args.rope else "(separate calls) + ")
                               + ("V pre-pass + " if pv_int8 else "") + "attention"},
        "attn_kernel_ms": attn_ms,
        "prepass_ms": pre_ms,
        "attn_only_tops": attn_tops,
        "pct_int8_mfma_peak_whole_step": 100.0 * value / INT8_PEAK_TOPS,
        "roofline": {
            "bound": "mfma",
            "achieved": attn_tops,
            "peak": INT8_PEAK_TOPS,
            "unit": "TOPS",
            "frac": attn_tops / INT8_PEAK_TOPS,
            "frac_of_measured_peak": attn_tops / int8_measured,
            "frac_of_blended_ceiling": attn_tops / (INT8_PEAK_TOPS if pv_int8 else INT8_PEAK_TOPS * 2 / 3),
            "frac_of_measured_ceiling": attn_tops / mix_measured,
            "measured": {"int8_stream_tops": int8_measured, "int8_stream_ghz": int8_ghz,
                         "kernel_mix_stream_tops": mix_measured, "kernel_mix_stream_ghz": mix_ghz,
                         "attention_kernel": kernel_clock,
                         "how": "sage_microbench kinds 0 and " + str(mix_kind) + ", 2 wavefronts per SIMD on every SIMD, "
                                "about 50 ms each, run after the timed steps (see profiles/mfma_peak_microbench.txt)"},
            "traffic": None if per_token else profiled_traffic(w.name, pv_int8),
            "traffic_unit": "bytes per launch (algorithmic: %.1f MB)" % ((5.0 if pv_int8 else 6.0) * B * H * N * D / 1e6),
            "kernel": "sage_attn_pv8_kernel" if pv_int8 else "sage_attn_kernel",
            "note": ("achieved = counted ops (all INT8) / mean attention-kernel time from HIP events on the launch "
                     "stream; peak = dense INT8 MFMA" if pv_int8 else
                     "achieved = counted ops (half INT8 ops, half FP16 flops) / mean attention-kernel time from HIP "
                     "events on the launch stream; peak = dense INT8 MFMA. Against the blended ceiling of this "
                     "algorithm (2/3 of the INT8 peak, because P~V runs at the FP16 rate) the fraction is "
                     f"{attn_tops / (INT8_PEAK_TOPS * 2 / 3):.4f}"),
        },
        "prepass_roofline": {
            "bound": "hbm",
            "achieved": (13.0 if pv_int8 else 8.0) * B * H * N * D / (pre_ms * 1e-3) / 1e9,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": (13.0 if pv_int8 else 8.0) * B * H * N * D / (pre_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "measured_copy_gbs": copy_gbs,
            "frac_of_measured_copy": (13.0 if pv_int8 else 8.0) * B * H * N * D / (pre_ms * 1e-3) / 1e9 / copy_gbs,
            "note": "algorithmic bytes: Q 2 read + 1 written, K 2 + 2 read (mean is a global dependency) + 1 written "
                    "= 8 B per element pair" + (", V 2 + 2 read (the channel maximum is a global dependency) + 1 written = 13"
                                                if pv_int8 else "")
                    + ("; the inputs are not rotated between steps" if args.rotate == 1 else f"; {args.rotate} input allocations in turn")
                    + "; within a step the second read of K (and V) may hit the last-level cache",
        },
        "paper_context": "paper reports ~2.1x over FlashAttention2 and ~2.7x over xformers on RTX4090 (340 TOPS, 52% of its INT8 peak)",
    }
    if sustained is not None:
        result["sustained"] = sustained
    if not args.no_cpu_baseline and not args.rope:      # the oracle leg times the headline path only
        del qd, kd, vd
        result["cpu_baseline"] = cpu_baseline(w, per_token=per_token, gpu_out_head0=out[0, 0].cpu().numpy(), pv_int8=pv_int8)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
