"""GPU parity at the documented size limits of the library: the longest sequence (N = 2^22 keys, where
byte offsets inside a head reach 2^29 and a causal workgroup walks 32768 key steps) and the largest
batch*heads (65535, the grid limit).  The oracle evaluates sampled rows / heads."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import assert_parity, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.timeout(900)
def test_longest_sequence():
    N, d = 1 << 22, 128
    cfg = wl.Workload("nmax", 2, 1, 1, N, d, True, "fp16")
    say(f"[limits] B1 H1 N{N} d{d} fp16 causal: generating")
    q, k, v = wl.generate(cfg, seed=wl.SEED0 + 900)
    sm = np.float32(cfg.sm_scale)
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device=DEV)
    say("   launching")
    sage.sage_attn_fwd(q.to(DEV), k.to(DEV), v.to(DEV), causal=True, sm_scale=float(sm), out=out)
    torch.cuda.synchronize()
    say("   gpu done")
    assert bool(torch.isfinite(out).all())
    qf, kf, vf = (wl.as_f32(t[0, 0]) for t in (q, k, v))
    quant = oracle.quantize_head(qf, kf, vf)
    say("   oracle quantisation done")
    refs, gots = [], []
    # first block, a block in the middle, the last rows (which see all 2^22 keys)
    for r0, r1 in ((0, 128), (N // 2 + 5, N // 2 + 13), (N - 8, N)):
        ref, _ = oracle.sage_attention_head(qf, kf, vf, causal=True, sm_scale=sm, out_dtype="fp16", row0=r0, row1=r1,
                                            quant=quant)
        refs.append(ref)
        gots.append(out[0, 0, r0:r1].float().cpu().numpy())
        say(f"   oracle rows {r0}:{r1} done")
    assert_parity(np.concatenate(refs), np.concatenate(gots), "fp16", "N = 2^22")


def test_most_heads():
    B, H, N, d = 5, 13107, 16, 64          # B*H = 65535
    cfg = wl.Workload("bhmax", 3, B, H, N, d, False, "bf16")
    say(f"[limits] B{B} H{H} N{N} d{d} bf16")
    q, k, v = wl.generate(cfg, seed=wl.SEED0 + 901)
    sm = np.float32(cfg.sm_scale)
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device=DEV)
    sage.sage_attn_fwd(q.to(DEV), k.to(DEV), v.to(DEV), causal=False, sm_scale=float(sm), out=out)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    refs, gots = [], []
    for b, h in ((0, 0), (2, 7000), (B - 1, H - 1)):
        ref, _ = oracle.sage_attention_head(*(wl.as_f32(t[b, h]) for t in (q, k, v)), causal=False, sm_scale=sm,
                                            out_dtype="bf16")
        refs.append(ref)
        gots.append(out[b, h].float().cpu().numpy())
    assert_parity(np.concatenate(refs), np.concatenate(gots), "bf16", "B*H = 65535")
    # one more head is refused
    assert sage.lib().sage_workspace_bytes(5, 13108, N, d) == 0
