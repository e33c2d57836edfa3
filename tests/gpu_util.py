"""Helpers of the GPU parity tests: run the oracle per head and compare with libsage outputs."""
import json
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from parity_gate import COS_MIN, REL_L1_MAX, format_metrics, parity_failures, parity_metrics  # noqa: F401


def say(*a):
    print(*a, flush=True)


def record_metrics(what, m):
    """Append the gate's metrics of one comparison to the file named by SAGE_GATE_LOG (if set): how the limits
    in parity_gate.py are kept in touch with what the GPU path measures."""
    path = os.environ.get("SAGE_GATE_LOG")
    if path:
        with open(path, "a") as f:
            f.write(json.dumps(dict(what=what, **m)) + "\n")


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


def assert_parity(ref, got, dtype, what="", flip_factor=1.0):
    """The parity gate (tests/parity_gate.py): the two norms of the benchmark definition over the whole block
    plus the worst single row, the largest element-wise difference and the fraction beyond one 16-bit ulp."""
    m = parity_metrics(ref, got, dtype)
    say(f"   {what}: {format_metrics(m)}")
    record_metrics(what, m)
    bad = parity_failures(m, flip_factor)
    assert not bad, f"{what}: " + "; ".join(bad)
    return m["cos"], m["rel_l1"]
