"""GPU parity of the grouped-query / cross-attention entry points (Hq a multiple of Hkv, Nq != Nk,
causal mask aligned to the end of both sequences) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import assert_parity, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(base, B, Hq, Hkv, Nq, Nk, d):
    cq = wl.Workload("q", base.index, B, Hq, Nq, d, False, base.dtype, base.q_dist, 0)
    ck = wl.Workload("kv", base.index, B, Hkv, Nk, d, False, base.dtype, "normal", base.k_outlier_channels)
    q, _, _ = wl.generate(cq)
    _, k, v = wl.generate(ck, seed=wl.SEED0 + 100 + base.index)
    return q, k, v


@pytest.mark.parametrize("idx,d", [(1, 128), (3, 64)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk", [
    (2, 8, 2, 300, 300),      # GQA, self-attention lengths
    (1, 4, 1, 100, 700),      # MQA, prefill continuation
    (1, 4, 2, 1, 1000),       # decode-shaped
    (1, 2, 2, 17, 129),       # ragged both ways
    (1, 6, 3, 257, 384),      # shift not a block multiple
    (1, 2, 1, 640, 128),      # more queries than keys (non-causal only)
])
def test_gqa_and_rectangular(idx, d, causal, B, Hq, Hkv, Nq, Nk):
    if causal and Nk < Nq:
        pytest.skip("rejected by the library, see test_gqa_argument_checks")
    base = wl.CONFIGS[idx - 1]
    q, k, v = _inputs(base, B, Hq, Hkv, Nq, Nk, d)
    say(f"[gqa] B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} {base.dtype} causal={causal}")
    sm = np.float32(1.0 / np.sqrt(d))
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device=DEV)
    sage.sage_attn_fwd_gqa(q.to(DEV), k.to(DEV), v.to(DEV), causal=causal, sm_scale=float(sm), out=out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all()
    ref = oracle.sage_attention(wl.as_f32(q), wl.as_f32(k), wl.as_f32(v), causal=causal, sm_scale=sm,
                                out_dtype=base.dtype)
    assert_parity(ref, got, base.dtype, "gqa")


def test_gqa_equals_repeated_kv_heads():
    base = wl.CONFIGS[0]
    q, k, v = _inputs(base, 1, 8, 2, 200, 200, 128)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    a = sage.sage_attn_fwd_gqa(qd, kd, vd, causal=True)
    b = sage.sage_attn_fwd(qd, kd.repeat_interleave(4, dim=1).contiguous(), vd.repeat_interleave(4, dim=1).contiguous(),
                           causal=True)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_stage_calls_equal_the_fused_call():
    base = wl.CONFIGS[0]
    q, k, v = _inputs(base, 1, 4, 2, 150, 400, 128)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    q_i8, q_scale = sage.sage_quant_q(qd)
    k_i8, k_scale, _ = sage.sage_quant_k(kd)
    v_fp8, v_scale = sage.sage_quant_v(vd)
    a = sage.sage_attn_fwd_quantized_gqa(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, causal=True, sm_scale=0.0,
                                         out_dtype=q.dtype)
    b = sage.sage_attn_fwd_gqa(qd, kd, vd, causal=True)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_gqa_argument_checks():
    base = wl.CONFIGS[0]
    q, k, v = _inputs(base, 1, 4, 3, 64, 64, 128)       # 4 % 3 != 0
    with pytest.raises(sage.SageError):
        sage.sage_attn_fwd_gqa(q.to(DEV), k.to(DEV), v.to(DEV), causal=False)
    q, k, v = _inputs(base, 1, 2, 2, 200, 100, 128)     # causal with Nk < Nq
    with pytest.raises(sage.SageError):
        sage.sage_attn_fwd_gqa(q.to(DEV), k.to(DEV), v.to(DEV), causal=True)
