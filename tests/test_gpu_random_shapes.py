"""Seeded sweep over random shapes (1 to 2600 keys): batch, head grouping, N_q, N_k, head dimension, value
distribution with its dtype (the normal fp16 and bf16 workloads, and the heavy-tailed one: Student-t queries, four
K channels x 20), mask and memory layout are drawn independently, every case goes through the strided entry point
and is compared with the oracle on the whole output."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import assert_parity, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        d = int(rng.choice([64, 128]))
        hkv = int(rng.integers(1, 4))
        group = int(rng.choice([1, 1, 2, 3, 4, 8]))
        nk = int(rng.choice([rng.integers(1, 40), rng.integers(40, 300), rng.integers(300, 700), rng.integers(700, 2600)]))
        nq = nk if rng.random() < 0.5 else int(rng.integers(1, nk + 1))
        if rng.random() < 0.15:
            nq = int(rng.integers(nk, nk + 200))          # more queries than keys: non-causal only
        causal = bool(rng.random() < 0.5) and nk >= nq
        out.append((i, int(rng.integers(1, 3)), hkv * group, hkv, nq, nk, d, int(rng.choice([1, 3, 5])), causal,
                    str(rng.choice(["bhnd", "bnhd"]))))
    return out


@pytest.mark.parametrize("i,B,Hq,Hkv,Nq,Nk,d,idx,causal,layout", _cases(60, 20250521))
def test_random_shape(i, B, Hq, Hkv, Nq, Nk, d, idx, causal, layout):
    base = wl.CONFIGS[idx - 1]
    say(f"[random] #{i} B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} {base.name}-like {base.dtype} causal={causal} {layout}")
    q, _, _ = wl.generate(wl.Workload("q", base.index, B, Hq, Nq, d, False, base.dtype, base.q_dist,
                                      base.k_outlier_channels), seed=wl.SEED0 + 700 + i)
    _, k, v = wl.generate(wl.Workload("kv", base.index, B, Hkv, Nk, d, False, base.dtype, base.q_dist,
                                      base.k_outlier_channels), seed=wl.SEED0 + 800 + i)
    sm = np.float32(1.0 / np.sqrt(d))
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    if layout == "bnhd":
        qd, kd, vd = (t.transpose(1, 2).contiguous() for t in (qd, kd, vd))
    out = torch.full(qd.shape, float("nan"), dtype=qd.dtype, device=DEV)
    sage.sage_attn_fwd_strided(qd, kd, vd, causal=causal, sm_scale=float(sm), layout=layout, out=out)
    torch.cuda.synchronize()
    got = (out.transpose(1, 2) if layout == "bnhd" else out).float().cpu().numpy()
    assert np.isfinite(got).all()
    ref = oracle.sage_attention(wl.as_f32(q), wl.as_f32(k), wl.as_f32(v), causal=causal, sm_scale=sm,
                                out_dtype=base.dtype)
    assert_parity(ref, got, base.dtype, f"random #{i}")
