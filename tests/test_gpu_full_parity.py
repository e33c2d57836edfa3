"""Every element of the full-size outputs against the oracle (not a sample): the GPU runs the whole forward
pass in the launch configuration the benchmark times, the oracle recomputes head after head on the host and
every head goes through the parity gate (norms, worst row, largest difference, fraction beyond one ulp).
cfg2, cfg3 and cfg4 take 10 to 60 seconds of oracle time on 16 host threads and are compared in full; of cfg5
(the benchmark's workload: 5 to 15 seconds per head) six whole heads spread over the 24 are compared in every
run and all 24 with `--full-sizes`."""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import COS_MIN, REL_L1_MAX, format_metrics, parity_failures, parity_metrics, record_metrics, say

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]
DEV = "cuda:0"


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_every_element_of_the_full_size_output(idx, request):
    cfg = wl.CONFIGS[idx - 1]
    heads = [(b, h) for b in range(cfg.B) for h in range(cfg.H)]
    if idx == 5 and not request.config.getoption("--full-sizes"):
        heads = [(0, h) for h in (0, 5, 10, 14, 19, 23)]
    say(f"[full parity] {cfg.name} B{cfg.B} H{cfg.H} N{cfg.N} d{cfg.d} {cfg.dtype} causal={cfg.causal}: "
        f"{len(heads)} of {cfg.B * cfg.H} heads, every element")
    q, k, v = wl.generate(cfg)
    sm = np.float32(cfg.sm_scale)
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device=DEV)
    sage.sage_attn_fwd(q.to(DEV), k.to(DEV), v.to(DEV), causal=cfg.causal, sm_scale=float(sm), out=out)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())       # the whole output, also the heads not compared below
    dot = n_ref = n_got = l1 = a_ref = 0.0
    worst = dict(rel_l1=0.0, row_l1=0.0, max_abs=0.0, beyond=0.0)
    t0 = time.time()
    for (b, h) in heads:
        ref, _ = oracle.sage_attention_head(wl.as_f32(q[b, h]), wl.as_f32(k[b, h]), wl.as_f32(v[b, h]),
                                            causal=cfg.causal, sm_scale=sm, out_dtype=cfg.dtype)
        ref = ref.astype(np.float64)
        got = out[b, h].float().cpu().numpy().astype(np.float64)
        m = parity_metrics(ref, got, cfg.dtype)
        say(f"   head ({b},{h}): {format_metrics(m)}  [{time.time() - t0:.0f}s]")
        record_metrics(f"{cfg.name} head ({b},{h})", m)
        bad = parity_failures(m)
        assert not bad, f"{cfg.name} head ({b},{h}): " + "; ".join(bad)
        for key in worst:
            worst[key] = max(worst[key], m[key])
        dot += float((ref * got).sum())
        n_ref += float((ref * ref).sum())
        n_got += float((got * got).sum())
        l1 += float(np.abs(ref - got).sum())
        a_ref += float(np.abs(ref).sum())
    cos, rel = dot / np.sqrt(n_ref * n_got), l1 / a_ref
    say(f"   {cfg.name}, {len(heads) * cfg.N * cfg.d} elements: cos={cos:.8f} relL1={rel:.3e}; worst head relL1="
        f"{worst['rel_l1']:.3e}, worst row relL1={worst['row_l1']:.3e}, max|d|/rms={worst['max_abs']:.3e}, "
        f"beyond-1ulp={worst['beyond']:.2e}")
    assert cos >= COS_MIN and rel <= REL_L1_MAX
