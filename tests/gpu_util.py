"""Helpers of the GPU parity tests: run the oracle per head and compare with libsage outputs."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl

COS_MIN = 0.9999      # parity bar against the oracle (benchmark definition)
REL_L1_MAX = 1e-3


def say(*a):
    print(*a, flush=True)


def oracle_quant_all(qf, kf, vf, v_r=4.5, workers=16):
    """Oracle quantisation of every head of [B,H,N,d] float32 arrays -> dict of stacked arrays."""
    B, H, N, d = qf.shape
    jobs = [(b, h) for b in range(B) for h in range(H)]

    def one(bh):
        b, h = bh
        return oracle.quantize_head(qf[b, h], kf[b, h], vf[b, h], v_r=v_r)

    with ThreadPoolExecutor(max_workers=workers) as ex:
        res = list(ex.map(one, jobs))
    out = {}
    for key in res[0]:
        out[key] = np.stack([r[key] for r in res]).reshape((B, H) + res[0][key].shape)
    return out


def gpu_quant_all(q, k, v, v_r=4.5):
    """libsage quantisation on the GPU -> dict of numpy arrays in the oracle's layouts."""
    B, H, N, d = q.shape
    q_i8, k_i8, q_scale, k_scale, k_mean = sage.sage_quant_qk(q, k)
    v_fp8, v_scale = sage.sage_quant_v(v, v_r)
    torch.cuda.synchronize()
    host = dict(q_codes=q_i8, q_scale=q_scale, k_codes=k_i8, k_scale=k_scale, k_mean=k_mean,
                v_codes=sage.v_fp8_to_token_major(v_fp8, N), v_scale=v_scale)
    dev = dict(q_i8=q_i8, k_i8=k_i8, v_fp8=v_fp8, q_scale=q_scale, k_scale=k_scale, v_scale=v_scale)
    return {k_: t.cpu().numpy() for k_, t in host.items()}, dev


def assert_quant_bit_exact(got, want):
    for key in ("k_mean", "q_scale", "k_scale", "v_scale"):
        a, b = got[key], want[key]
        assert a.shape == b.shape, key
        # compare bit patterns (also distinguishes -0.0 / NaN payloads)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), f"{key}: {np.sum(a != b)} of {a.size} differ"
    for key in ("q_codes", "k_codes", "v_codes"):
        a, b = got[key], want[key]
        assert a.shape == b.shape and a.dtype == b.dtype, key
        bad = int(np.count_nonzero(a != b))
        assert bad == 0, f"{key}: {bad} of {a.size} codes differ"


def oracle_rows(wq, b, h, row0, row1, *, causal, sm_scale, out_dtype, p_r=224.0):
    """Oracle attention for rows [row0,row1) of head (b,h) from the oracle's own quantised operands."""
    return oracle.attn_rows(wq["q_codes"][b, h], wq["k_codes"][b, h], wq["v_codes"][b, h],
                            wq["q_scale"][b, h], wq["k_scale"][b, h], wq["v_scale"][b, h],
                            causal=causal, sm_scale=sm_scale, p_r=p_r, row0=row0, row1=row1,
                            out_dtype=out_dtype)


def assert_parity(ref, got, what=""):
    cos, l1 = wl.cos_sim(ref, got), wl.rel_l1(ref, got)
    say(f"   {what}: cos={cos:.7f} relL1={l1:.3e} rmse={wl.rmse(ref, got):.3e}")
    assert np.isfinite(got).all(), what
    assert cos >= COS_MIN and l1 <= REL_L1_MAX, f"{what}: cos={cos} relL1={l1}"
    return cos, l1
