"""GPU tests of the strided entry point (`sage_attn_fwd_strided`): token-major [B,N,H,d] tensors,
slices of a packed QKV projection, broadcast K/V heads and an output written into a slice.

The strides only change addresses, so every result must equal, bit for bit, the result of the
contiguous entry point on contiguous copies (which the other GPU tests compare with the oracle);
one case is also compared with the oracle directly.
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
    _, k, v = wl.generate(ck, seed=wl.SEED0 + 300 + base.index)
    return q.to(DEV), k.to(DEV), v.to(DEV)


def _bits(t):
    return t.contiguous().view(torch.int16)


@pytest.mark.parametrize("idx,d", [(1, 128), (3, 64), (5, 128)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk", [(2, 4, 4, 300, 300), (1, 6, 2, 129, 500), (1, 2, 1, 1, 77)])
def test_token_major_layout(idx, d, causal, B, Hq, Hkv, Nq, Nk):
    base = wl.CONFIGS[idx - 1]
    q, k, v = _inputs(base, B, Hq, Hkv, Nq, Nk, d)
    say(f"[layout] bnhd B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} {base.dtype} causal={causal}")
    want = sage.sage_attn_fwd_gqa(q, k, v, causal=causal)
    qn, kn, vn = (t.transpose(1, 2).contiguous() for t in (q, k, v))     # [B,N,H,d] in memory
    got = sage.sage_attn_fwd_strided(qn, kn, vn, causal=causal, layout="bnhd")
    torch.cuda.synchronize()
    assert got.shape == qn.shape and got.is_contiguous()
    assert torch.equal(_bits(got.transpose(1, 2)), _bits(want))
    # the same memory described as a [B,H,N,d] view with permuted strides
    got2 = sage.sage_attn_fwd_strided(qn.transpose(1, 2), kn.transpose(1, 2), vn.transpose(1, 2), causal=causal,
                                      layout="bhnd")
    torch.cuda.synchronize()
    assert torch.equal(_bits(got2), _bits(want))


@pytest.mark.parametrize("d", [64, 128])
def test_packed_qkv_slices_and_output_slice(d):
    base = wl.CONFIGS[1]
    B, H, N = 2, 3, 260
    q, k, v = _inputs(base, B, H, H, N, N, d)
    want = sage.sage_attn_fwd(q, k, v, causal=True)
    qkv = torch.empty((B, N, 3, H, d), dtype=q.dtype, device=DEV)      # one projection output
    qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2] = (t.transpose(1, 2) for t in (q, k, v))
    big = torch.full((B, N, H, 2 * d), 7.0, dtype=q.dtype, device=DEV)
    out = big[..., d:]                                                  # rows of d inside rows of 2d
    sage.sage_attn_fwd_strided(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], causal=True, layout="bnhd", out=out)
    torch.cuda.synchronize()
    assert torch.equal(_bits(out.transpose(1, 2)), _bits(want))
    assert bool((big[..., :d] == 7.0).all())                            # nothing outside the slice is written


def test_broadcast_kv_heads_equal_grouped_query():
    base = wl.CONFIGS[0]
    q, k, v = _inputs(base, 1, 4, 1, 200, 333, 128)
    want = sage.sage_attn_fwd_gqa(q, k, v, causal=False)                # Hkv = 1
    got = sage.sage_attn_fwd_strided(q, k.expand(1, 4, 333, 128), v.expand(1, 4, 333, 128), causal=False)
    torch.cuda.synchronize()
    assert torch.equal(_bits(got), _bits(want))


def test_token_major_against_oracle():
    base = wl.CONFIGS[2]
    q, k, v = _inputs(base, 1, 4, 2, 150, 270, 64)
    sm = np.float32(1.0 / np.sqrt(64))
    got = sage.sage_attn_fwd_strided(*(t.transpose(1, 2).contiguous() for t in (q, k, v)), causal=True,
                                     sm_scale=float(sm), layout="bnhd")
    torch.cuda.synchronize()
    ref = oracle.sage_attention(wl.as_f32(q.cpu()), wl.as_f32(k.cpu()), wl.as_f32(v.cpu()), causal=True, sm_scale=sm,
                                out_dtype=base.dtype)
    assert_parity(ref, got.transpose(1, 2).float().cpu().numpy(), base.dtype, "bnhd")
