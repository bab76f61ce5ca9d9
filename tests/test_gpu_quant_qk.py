"""sage_quant_qk (both pre-passes of a (Q, K) pair in one launch less) against the two separate calls: the
same bodies run, so every output must be the same bits; and against the oracle on one case of each kind."""
import numpy as np
import pytest
import torch

import oracle
import paper_2410_02367_amd as sage
import sage_inputs as si
from gpu_util import to_dev

pytestmark = pytest.mark.gpu

# (name, B, H, Nq, Nkv, D, block_q, block_k) -- short keys take the single-launch K job (Nkv <= 512), long ones
# the column sums; every Q kernel variant (1, 2, 4, 8 rows per thread; 256 and 512 threads; per token)
CASES = [
    ("vit_like", 3, 4, 197, 197, 64, 128, 64),
    ("short_d128", 2, 3, 300, 300, 128, 128, 64),
    ("short_keys_long_queries", 1, 2, 1500, 512, 128, 128, 128),
    ("short_per_token", 2, 2, 130, 130, 128, 1, 1),
    ("short_per_token_d64", 1, 3, 257, 100, 64, 1, 1),
    ("mid_d128", 2, 4, 1536, 1536, 128, 128, 64),
    ("mid_d64", 2, 3, 1105, 1105, 64, 128, 64),
    ("mid_blocks_64", 1, 2, 1000, 1300, 128, 64, 32),
    ("mid_blocks_32_d64", 1, 2, 777, 2049, 64, 32, 128),
    ("mid_blocks_64_d64", 1, 3, 600, 900, 64, 64, 64),
    ("one_query", 2, 2, 1, 3000, 128, 128, 64),
    ("per_token_long", 1, 2, 2100, 2100, 128, 1, 1),
    ("per_token_long_d64", 1, 2, 513, 4100, 64, 1, 1),
    ("long", 1, 2, 9000, 9000, 128, 128, 64),
]


def make(name, B, H, Nq, Nkv, D, seed):
    wq = si.custom(name + "_q", B, H, Nq, D, False, seed=si.BASE_SEED + 1300 + seed)
    wk = si.custom(name + "_k", B, H, Nkv, D, False, k_noise=1.0, k_bias=3.0, seed=si.BASE_SEED + 1350 + seed)
    q, _, _ = si.full(wq)
    _, k, _ = si.full(wk)
    return q, k, wq.sm_scale


@pytest.mark.parametrize("name,B,H,Nq,Nkv,D,bq,bk", CASES, ids=[c[0] for c in CASES])
def test_quant_qk_is_the_two_calls(name, B, H, Nq, Nkv, D, bq, bk):
    print(f"[case] quant_qk {name} B{B} H{H} Nq{Nq} Nkv{Nkv} D{D} scales {bq}x{bk}", flush=True)
    q, k, sm = make(name, B, H, Nq, Nkv, D, len(name))
    qd, kd = to_dev(q), to_dev(k)
    k_i8, k_scale, k_mean = sage.sage_smooth_quant_k(kd, bk)
    q_i8, q_scale = sage.sage_quant_q(qd, sm, bq)
    # poisoned outputs: every element must be written by the fused call
    fq = torch.full_like(q_i8, 99)
    fk = torch.full_like(k_i8, 99)
    fqs = torch.full_like(q_scale, -1.0)
    fks = torch.full_like(k_scale, -1.0)
    fm = torch.full_like(k_mean, 123.0)
    sage.sage_quant_qk(qd, kd, sm, bq, bk, q_i8=fq, q_scale=fqs, k_i8=fk, k_scale=fks, k_mean=fm)
    torch.cuda.synchronize()
    assert torch.equal(fq, q_i8) and torch.equal(fqs, q_scale), f"{name}: Q side differs"
    assert torch.equal(fk, k_i8) and torch.equal(fks, k_scale) and torch.equal(fm, k_mean), f"{name}: K side differs"


@pytest.mark.parametrize("name", ["vit_like", "mid_d128", "per_token_long_d64"])
def test_quant_qk_against_the_oracle(name):
    _, B, H, Nq, Nkv, D, bq, bk = next(c for c in CASES if c[0] == name)
    print(f"[case] quant_qk vs oracle {name}", flush=True)
    q, k, sm = make(name, B, H, Nq, Nkv, D, len(name))
    q_i8, q_scale, k_i8, k_scale, k_mean = sage.sage_quant_qk(to_dev(q), to_dev(k), sm, bq, bk)
    torch.cuda.synchronize()
    kq, ks, km = oracle.smooth_quant_k(k, bk)
    qq, qs = oracle.quant_q(q, sm, bq)
    assert np.array_equal(q_i8.cpu().numpy(), qq) and np.array_equal(q_scale.cpu().numpy(), qs)
    assert np.array_equal(k_i8.cpu().numpy(), kq) and np.array_equal(k_scale.cpu().numpy(), ks)
    assert np.array_equal(k_mean.cpu().numpy(), km)


def test_quant_qk_needs_the_k_workspace():
    q = torch.zeros((1, 1, 64, 64), dtype=torch.float16, device="cuda")
    k = torch.zeros((1, 1, 1024, 64), dtype=torch.float16, device="cuda")
    small = torch.empty(1, dtype=torch.int64, device="cuda")
    with pytest.raises(sage.SageError) as e:
        sage.sage_quant_qk(q, k, 0.125, workspace=small)
    assert e.value.status == 4
