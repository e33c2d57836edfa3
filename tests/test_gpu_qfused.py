"""GPU tests of the attention entry point that quantises Q in its own prologue
(`sage_attn_fwd_kvquantized_gqa`).

Its Q codes and scales must be the very bits the stand-alone quantiser writes (which the
quantisation tests compare bit for bit with the oracle), so its output must equal the output of the
three-stage path exactly; that equality is checked here on every shape class, and one case goes
against the oracle directly.
"""
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
    _, k, v = wl.generate(ck, seed=wl.SEED0 + 200 + base.index)
    return q.to(DEV), k.to(DEV), v.to(DEV)


def _both_paths(q, k, v, causal, sm):
    """(three-stage output, fused-Q output) on the same quantised K^, V^."""
    k_i8, k_scale, _ = sage.sage_quant_k(k)
    v_fp8, v_scale = sage.sage_quant_v(v, 4.5)
    q_i8, q_scale = sage.sage_quant_q(q)
    staged = sage.sage_attn_fwd_quantized_gqa(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, causal=causal,
                                              sm_scale=sm, out_dtype=q.dtype)
    fused = torch.full(q.shape, float("nan"), dtype=q.dtype, device=q.device)
    sage.sage_attn_fwd_kvquantized_gqa(q, k_i8, v_fp8, k_scale, v_scale, causal=causal, sm_scale=sm, out=fused)
    torch.cuda.synchronize()
    return staged, fused


# cfg1/cfg2: fp16, cfg3: bf16, cfg5: bf16 with heavy-tailed Q (large block maxima, many saturated codes)
@pytest.mark.parametrize("idx,d", [(1, 128), (3, 64), (5, 128), (2, 64)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk", [
    (1, 2, 2, 1, 1),          # one row
    (1, 2, 2, 63, 63),        # less than one Q block
    (2, 3, 3, 128, 128),      # exactly one block
    (1, 2, 2, 129, 129),      # one row into the second block
    (1, 4, 2, 777, 777),      # several blocks and a ragged tail, GQA
    (1, 4, 1, 200, 900),      # rectangular, MQA
])
def test_fused_q_equals_staged(idx, d, causal, B, Hq, Hkv, Nq, Nk):
    base = wl.CONFIGS[idx - 1]
    q, k, v = _inputs(base, B, Hq, Hkv, Nq, Nk, d)
    say(f"[qfused] B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} {base.dtype} causal={causal}")
    staged, fused = _both_paths(q, k, v, causal, 1.0 / np.sqrt(d))
    assert torch.isfinite(fused.float()).all()
    assert torch.equal(staged.view(torch.int16), fused.view(torch.int16))


def test_fused_q_zero_block_and_zero_rows():
    """An all-zero Q block (scale 0, codes 0) gives the plain mean of V^ over the visible keys in both paths."""
    base = wl.CONFIGS[0]
    q, k, v = _inputs(base, 1, 2, 2, 300, 300, 128)
    q[:, :, 128:256] = 0
    q[:, 0, 5] = 0
    staged, fused = _both_paths(q, k, v, True, 1.0 / np.sqrt(128))
    assert torch.isfinite(fused.float()).all()
    assert torch.equal(staged.view(torch.int16), fused.view(torch.int16))


def test_fused_q_against_oracle():
    base = wl.CONFIGS[4]  # bf16, Student-t Q, K outlier channels
    q, k, v = _inputs(base, 1, 2, 1, 333, 333, 128)
    sm = np.float32(1.0 / np.sqrt(128))
    k_i8, k_scale, _ = sage.sage_quant_k(k)
    v_fp8, v_scale = sage.sage_quant_v(v, 4.5)
    out = sage.sage_attn_fwd_kvquantized_gqa(q, k_i8, v_fp8, k_scale, v_scale, causal=True, sm_scale=float(sm))
    torch.cuda.synchronize()
    ref = oracle.sage_attention(wl.as_f32(q.cpu()), wl.as_f32(k.cpu()), wl.as_f32(v.cpu()), causal=True, sm_scale=sm,
                                out_dtype=base.dtype)
    assert_parity(ref, out.float().cpu().numpy(), base.dtype, "qfused")


def test_fused_q_argument_checks():
    L = sage.lib()
    q = torch.zeros((1, 2, 64, 128), dtype=torch.float16, device=DEV)
    k_i8 = torch.zeros((1, 2, 64, 128), dtype=torch.int8, device=DEV)
    v_fp8 = torch.zeros(sage.v_fp8_bytes(1, 2, 64, 128), dtype=torch.uint8, device=DEV)
    ks = torch.zeros((1, 2, 1), dtype=torch.float32, device=DEV)
    vs = torch.zeros((1, 2, 128), dtype=torch.float32, device=DEV)
    out = torch.zeros_like(q)

    def call(qp=q.data_ptr(), Hq=2, Hkv=2, Nq=64, Nk=64, d=128, causal=0, p_r=224.0, dt=0):
        return L.sage_attn_fwd_kvquantized_gqa(qp, k_i8.data_ptr(), v_fp8.data_ptr(), ks.data_ptr(), vs.data_ptr(),
                                               out.data_ptr(), 1, Hq, Hkv, Nq, Nk, d, causal, 0.0, p_r, dt, 0)

    assert call() == 0
    assert call(qp=0) == -1
    assert call(qp=q.data_ptr() + 2) == -1       # misaligned
    assert call(Hq=3) == -1                      # not a multiple of Hkv
    assert call(d=96) == -1
    assert call(Nq=64, Nk=32, causal=1) == -1    # causal needs Nk >= Nq
    assert call(p_r=0.0) == -1
    assert call(dt=7) == -1
    torch.cuda.synchronize()
