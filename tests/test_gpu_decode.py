"""GPU parity of the decode-shaped path (sage_attn_fwd_decode): the query heads of a K/V head packed into one tile,
the keys evaluated in ranges and combined.  With one range it must reproduce the prefill kernel bit for bit (same
steps, same arithmetic); with several it is compared with the oracle's key-split mode on the same ranges."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import assert_parity, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(idx, B, Hq, Hkv, Nq, Nk, d, dtype=None):
    base = wl.CONFIGS[idx - 1]
    dt = dtype or base.dtype
    qcfg = wl.Workload("dq", base.index, B, Hq, Nq, d, False, dt, base.q_dist, base.k_outlier_channels)
    kcfg = wl.Workload("dk", base.index, B, Hkv, Nk, d, False, dt, base.q_dist, base.k_outlier_channels)
    q, _, _ = wl.generate(qcfg, seed=11 + Nq + Nk)
    _, k, v = wl.generate(kcfg, seed=13 + Nq + Nk)
    return q, k, v, 1.0 / np.sqrt(d)


def _oracle(q, k, v, causal, sm_scale, split_keys, heads=None):
    """Oracle output [B,Hq,Nq,d] (float64, rounded to the 16-bit type) with its own quantised operands."""
    B, Hq, Nq, d = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    qf, kf, vf = wl.as_f32(q), wl.as_f32(k), wl.as_f32(v)
    name = "bf16" if q.dtype == torch.bfloat16 else "fp16"
    out = np.zeros((B, Hq, Nq, d))
    for b in range(B):
        for hk in range(Hkv):
            if heads is not None and (b, hk) not in heads:
                continue
            kc, ks = oracle.quant_int8(kf[b, hk], oracle.k_mean(kf[b, hk]), 64)
            vc, vs = oracle.quant_v(vf[b, hk], 4.5)
            for h in range(hk * group, (hk + 1) * group):
                qc, qs = oracle.quant_int8(qf[b, h], None, 128)
                out[b, h] = oracle.attn_rows(qc, kc, vc, qs, ks, vs, causal=causal, sm_scale=sm_scale, out_dtype=name,
                                             split_keys=split_keys)
    return out


def _gpu(q, k, v, causal, sm_scale, split_keys):
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    k_i8, k_scale, _, v_fp8, v_scale = sage.sage_quant_kv(kd, vd, 4.5)
    out = sage.sage_attn_fwd_decode(qd, k_i8, v_fp8, k_scale, v_scale, causal=causal, sm_scale=sm_scale,
                                    split_keys=split_keys)
    ref = sage.sage_attn_fwd_kvquantized_gqa(qd, k_i8, v_fp8, k_scale, v_scale, causal=causal, sm_scale=sm_scale)
    torch.cuda.synchronize()
    return out, ref


ONE_RANGE = [  # idx, B, Hq, Hkv, Nq, Nk, d, causal
    (1, 2, 4, 4, 1, 700, 128, False), (2, 1, 8, 2, 2, 1000, 128, True), (3, 2, 6, 2, 5, 300, 64, True),
    (5, 1, 16, 1, 1, 129, 128, False), (4, 2, 2, 2, 16, 513, 64, True), (1, 1, 3, 3, 7, 64, 128, True),
    (5, 2, 8, 8, 1, 1, 128, True),
    # more than 16 rows per K/V head: several row tiles, heads that straddle them
    (2, 2, 8, 2, 5, 600, 128, True), (3, 1, 4, 1, 16, 1000, 64, True), (5, 1, 16, 2, 3, 257, 128, False),
    (1, 2, 2, 2, 33, 400, 128, True),
    # more than 64 rows per K/V head: the prefill kernel with key ranges (here: one range)
    (2, 1, 8, 2, 17, 700, 128, True), (3, 2, 2, 2, 130, 600, 64, True), (5, 1, 4, 1, 300, 300, 128, True),
    (1, 1, 2, 2, 200, 1000, 128, False),
]


@pytest.mark.parametrize("idx,B,Hq,Hkv,Nq,Nk,d,causal", ONE_RANGE)
def test_one_range_reproduces_the_prefill_kernel_bit_for_bit(idx, B, Hq, Hkv, Nq, Nk, d, causal):
    say(f"[decode] one range: cfg{idx} B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} causal={causal}")
    q, k, v, sm = _inputs(idx, B, Hq, Hkv, Nq, Nk, d)
    whole = -(-Nk // 128) * 128
    out, ref = _gpu(q, k, v, causal, sm, whole)
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    assert torch.isfinite(out.float()).all()


RANGES = [  # idx, B, Hq, Hkv, Nq, Nk, d, causal, split_keys (0: the library's choice)
    (1, 4, 8, 2, 1, 1000, 128, False, 128), (1, 4, 8, 2, 1, 1000, 128, False, 384),
    (2, 2, 16, 4, 2, 2049, 128, True, 256), (2, 2, 16, 4, 4, 2049, 128, True, 0),
    (3, 4, 8, 8, 3, 1500, 64, True, 512), (4, 2, 32, 4, 1, 4096, 64, False, 0),
    (5, 4, 8, 1, 2, 777, 128, True, 128), (5, 8, 4, 4, 16, 300, 128, True, 128),
    (1, 8, 4, 2, 8, 129, 64, True, 128),
    (2, 2, 8, 2, 5, 1500, 128, True, 256), (4, 2, 4, 1, 16, 2000, 64, True, 0), (5, 1, 24, 3, 7, 900, 128, False, 384),
    # more than 64 rows per K/V head: key ranges on the prefill kernel, rows that see nothing of the last ranges
    (2, 1, 8, 2, 40, 3000, 128, True, 512), (3, 2, 4, 4, 129, 2500, 64, True, 0), (5, 1, 2, 1, 256, 4096, 128, False, 1024),
    (1, 1, 4, 2, 700, 1900, 128, True, 256), (4, 1, 2, 2, 100, 5000, 64, False, 0),
]


@pytest.mark.parametrize("idx,B,Hq,Hkv,Nq,Nk,d,causal,split_keys", RANGES)
def test_ranges_against_the_oracle_on_the_same_ranges(idx, B, Hq, Hkv, Nq, Nk, d, causal, split_keys):
    used = split_keys or sage.decode_split_keys(B, Hq, Hkv, Nq, Nk)
    say(f"[decode] ranges of {used}: cfg{idx} B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} causal={causal}")
    assert used % 128 == 0 and used >= 128
    q, k, v, sm = _inputs(idx, B, Hq, Hkv, Nq, Nk, d)
    out, _ = _gpu(q, k, v, causal, sm, split_keys)
    want = _oracle(q, k, v, causal, sm, used)
    got = out.cpu().to(torch.float64).numpy()
    assert np.isfinite(got).all()
    assert_parity(want.reshape(-1, d), got.reshape(-1, d), "bf16" if q.dtype == torch.bfloat16 else "fp16",
                  f"decode B{B} Hq{Hq}/{Hkv} Nq{Nq} Nk{Nk} d{d} split {used}", flip_factor=2.0)


def _random_case(seed):
    rng = np.random.default_rng(9000 + seed)
    group = int(rng.choice([1, 2, 3, 4, 8, 16]))
    Nq = int(rng.integers(1, (16 if seed % 3 else 64) // group + 1))
    Hkv = int(rng.choice([1, 2, 3]))
    B = int(rng.integers(1, 5))
    d = int(rng.choice([64, 128]))
    Nk = int(rng.choice([rng.integers(Nq, 130), rng.integers(130, 700), rng.integers(700, 3000)]))
    causal = bool(rng.integers(0, 2))
    split = int(rng.choice([0, 128, 256, 512]))
    idx = int(rng.choice([1, 3, 5]))
    return idx, B, Hkv * group, Hkv, Nq, Nk, d, causal, split


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_decode_shapes(seed):
    idx, B, Hq, Hkv, Nq, Nk, d, causal, split_keys = _random_case(seed)
    used = split_keys or sage.decode_split_keys(B, Hq, Hkv, Nq, Nk)
    say(f"[decode] seed {seed}: cfg{idx} B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} causal={causal} ranges of {used}")
    q, k, v, sm = _inputs(idx, B, Hq, Hkv, Nq, Nk, d)
    out, _ = _gpu(q, k, v, causal, sm, split_keys)
    want = _oracle(q, k, v, causal, sm, used)
    got = out.cpu().to(torch.float64).numpy()
    assert np.isfinite(got).all()
    # few rows: the norms of the gate and the worst row, not the flip statistics of large blocks
    m_cos = float((want * got).sum() / np.sqrt((want * want).sum() * (got * got).sum()))
    rel = float(np.abs(want - got).sum() / np.abs(want).sum())
    assert m_cos >= 0.9999 and rel <= 1e-3, (m_cos, rel)
    assert_parity(want.reshape(-1, d), got.reshape(-1, d), "bf16" if q.dtype == torch.bfloat16 else "fp16",
                  f"decode seed {seed}", flip_factor=4.0)


def test_decode_call_can_be_replayed_from_a_hip_graph():
    """Two launches, no memset, no allocation: captured once, replayed with other data in the same buffers."""
    B, Hq, Hkv, Nq, Nk, d = 2, 8, 2, 2, 1500, 128
    q, k, v, sm = _inputs(2, B, Hq, Hkv, Nq, Nk, d)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    k_i8, k_scale, _, v_fp8, v_scale = sage.sage_quant_kv(kd, vd, 4.5)
    ws = torch.empty(sage.decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, d, 256), dtype=torch.uint8, device=DEV)
    out = torch.empty_like(qd)
    eager = sage.sage_attn_fwd_decode(qd, k_i8, v_fp8, k_scale, v_scale, causal=True, sm_scale=sm, split_keys=256,
                                      workspace=ws).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):      # warm-up on the capture stream
        sage.sage_attn_fwd_decode(qd, k_i8, v_fp8, k_scale, v_scale, causal=True, sm_scale=sm, split_keys=256,
                                  out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sage.sage_attn_fwd_decode(qd, k_i8, v_fp8, k_scale, v_scale, causal=True, sm_scale=sm, split_keys=256,
                                  out=out, workspace=ws)
    for rep in range(3):
        out.fill_(float("nan"))
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), rep
    q2 = torch.flip(qd, dims=[1]).contiguous()
    want2 = sage.sage_attn_fwd_decode(q2, k_i8, v_fp8, k_scale, v_scale, causal=True, sm_scale=sm, split_keys=256).clone()
    qd.copy_(q2)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want2.view(torch.int16))


def test_long_cache_with_the_library_split():
    """The shape the path is for: B 8, 32 / 8 heads, one query row over 32768 keys; all heads of two K/V heads
    against the oracle."""
    B, Hq, Hkv, Nq, Nk, d = 8, 32, 8, 1, 32768, 128
    used = sage.decode_split_keys(B, Hq, Hkv, Nq, Nk)
    say(f"[decode] long cache, ranges of {used}")
    q, k, v, sm = _inputs(5, B, Hq, Hkv, Nq, Nk, d)
    out, _ = _gpu(q, k, v, True, sm, 0)
    heads = {(0, 0), (7, 5)}
    want = _oracle(q, k, v, True, sm, used, heads=heads)
    got = out.cpu().to(torch.float64).numpy()
    assert np.isfinite(got).all()
    rows_w, rows_g = [], []
    for (b, hk) in heads:
        rows_w.append(want[b, hk * 4:(hk + 1) * 4].reshape(-1, d))
        rows_g.append(got[b, hk * 4:(hk + 1) * 4].reshape(-1, d))
    assert_parity(np.concatenate(rows_w), np.concatenate(rows_g), "bf16", "decode long cache", flip_factor=2.0)


def test_argument_errors():
    q, k, v, sm = _inputs(1, 1, 4, 2, 9, 8, 128)          # causal with more query rows than keys
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    k_i8, k_scale, _, v_fp8, v_scale = sage.sage_quant_kv(kd, vd, 4.5)
    with pytest.raises(sage.SageError):
        sage.sage_attn_fwd_decode(qd, k_i8, v_fp8, k_scale, v_scale, causal=True, sm_scale=sm)
    q, k, v, sm = _inputs(1, 1, 4, 2, 1, 256, 128)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    k_i8, k_scale, _, v_fp8, v_scale = sage.sage_quant_kv(kd, vd, 4.5)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(sage.SageError):
        sage.sage_attn_fwd_decode(qd, k_i8, v_fp8, k_scale, v_scale, causal=False, sm_scale=sm, split_keys=100,
                                  workspace=ws)
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(sage.SageError):
        sage.sage_attn_fwd_decode(qd, k_i8, v_fp8, k_scale, v_scale, causal=False, sm_scale=sm, split_keys=128,
                                  workspace=small)
    torch.cuda.synchronize()
