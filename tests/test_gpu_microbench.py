"""The instruction-stream probes (sage_microbench) run and report what their documentation says: a 32x32
matrix instruction occupies the matrix pipe for 32 clocks, whatever the clock the chip holds -- the fact the
measured rooflines of bench.py rest on.  Timing-derived figures are only checked for plausibility."""
import numpy as np
import pytest
import torch

import paper_2410_02367_amd as sage

pytestmark = pytest.mark.gpu


def probe(kind, waves, iters=4000, workgroups=256):
    g = torch.Generator(device="cuda").manual_seed(7)
    data = torch.randint(-2 ** 31, 2 ** 31 - 1, (1024,), generator=g, device="cuda", dtype=torch.int64).to(torch.int32)
    out = sage.sage_microbench(kind, waves, workgroups, iters, data)
    torch.cuda.synchronize()
    o = out.cpu().numpy().astype(np.float64)
    assert o.shape == (workgroups * 4 * waves, 4)
    return o, iters


def test_matrix_streams_take_32_clocks_per_instruction():
    for kind, groups in ((0, 8), (1, 8), (2, 24), (14, 8)):
        print(f"[case] microbench kind {kind}", flush=True)
        o, iters = probe(kind, 1)
        ticks = o[:, 0] / iters / groups            # shader clocks per matrix instruction, per wavefront
        assert np.all(o[:, 1] > 0)
        assert 31.5 <= np.median(ticks) <= 34.0, f"kind {kind}: {np.median(ticks):.2f} clocks per matrix instruction"
        ghz = np.median(o[:, 0] / o[:, 1]) * 0.1      # the constant-rate counter runs at 100 MHz
        assert 0.5 <= ghz <= 2.6, ghz
        print(f"  {np.median(ticks):.2f} clocks per instruction at {ghz:.2f} GHz", flush=True)


def test_every_probe_runs_and_is_deterministic():
    for kind in range(21):
        waves = 2 if kind == 5 else 1
        a, _ = probe(kind, waves, iters=50, workgroups=16)
        b, _ = probe(kind, waves, iters=50, workgroups=16)
        assert np.array_equal(a[:, 2], b[:, 2]), f"kind {kind}: checksums differ between two runs"
        assert np.all(a[:, 0] > 0)
    with pytest.raises(sage.SageError) as e:
        probe(21, 1, iters=10, workgroups=4)
    assert e.value.status == 3
