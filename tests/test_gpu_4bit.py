"""GPU parity of the 4+8 variant (INT4 Q K^T with smoothing of Q and K; paper Sections 2.1, 3, 4.1) against the
oracle's 4+8 routines, through the C ABI.

Stage 1: block means of Q, INT4 codes and scales of Q and K, the K mean, the FP8 V codes -- bit-exact.  The score
correction (FP32 on the GPU, double in the oracle) to FP32 rounding.  Stage 2 and the whole path: through the
parity gate, like the 8+8 path."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import assert_parity, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LOG2E = 1.4426950408889634


def _inputs(base_idx, B, Hq, Hkv, Nq, Nk, d, q_offset, seed):
    base = wl.CONFIGS[base_idx - 1]
    mk = lambda H, N: wl.Workload("q4", base.index, B, H, N, d, False, base.dtype, base.q_dist, base.k_outlier_channels)
    q, _, _ = wl.generate(mk(Hq, Nq), seed=wl.SEED0 + 1000 + seed)
    _, k, v = wl.generate(mk(Hkv, Nk), seed=wl.SEED0 + 1100 + seed)
    if q_offset:
        # a per-(head, channel) offset on Q that drifts along the sequence: what smoothing of Q is there to remove
        g = torch.Generator().manual_seed(seed)
        off = q_offset * torch.randn((B, Hq, 1, d), generator=g)
        drift = torch.linspace(0.5, 1.5, Nq).reshape(1, 1, Nq, 1)
        q = (q.float() + off * drift).to(q.dtype)
    return q, k, v, base


def _oracle_quant(q, k, v, b, hq, hkv):
    return oracle.quantize_head_4bit(wl.as_f32(q[b, hq]), wl.as_f32(k[b, hkv]), wl.as_f32(v[b, hkv]))


@pytest.mark.parametrize("base_idx,d", [(1, 128), (3, 64), (5, 128)])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk", [(1, 2, 2, 300, 300), (2, 4, 2, 129, 515), (1, 2, 1, 1000, 1000)])
def test_stage1_of_the_4bit_variant_is_bit_exact(base_idx, d, B, Hq, Hkv, Nq, Nk):
    q, k, v, base = _inputs(base_idx, B, Hq, Hkv, Nq, Nk, d, 2.0, 1)
    say(f"[4bit] stage 1: B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} {base.dtype}")
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    q_mean, q_i4, q_scale = sage.sage_quant_q4(qd)
    k_i4, k_scale, k_mean, v_fp8, v_scale = sage.sage_quant_kv4(kd, vd)
    sm = float(np.float32(1.0 / np.sqrt(d)))
    dsx = sage.sage_delta_s(kd, k_mean, q_mean, Nq, causal=False, sm_scale=sm)
    torch.cuda.synchronize()
    ds_keys = sage.delta_s_to_key_order(dsx, Nk).cpu().numpy()
    v_codes = sage.v_fp8_to_token_major(v_fp8, Nk).cpu().numpy()
    group = Hq // Hkv
    for b in range(B):
        for hq in range(Hq):
            hkv = hq // group
            want = _oracle_quant(q, k, v, b, hq, hkv)
            for name, got in (("q_mean", q_mean[b, hq]), ("q_scale", q_scale[b, hq]), ("k_scale", k_scale[b, hkv]),
                              ("k_mean", k_mean[b, hkv]), ("v_scale", v_scale[b, hkv])):
                a = got.cpu().numpy()
                assert np.array_equal(a.view(np.uint32), want[name].view(np.uint32)), name
            assert np.array_equal(q_i4[b, hq].cpu().numpy(), want["q_codes"])
            assert np.array_equal(k_i4[b, hkv].cpu().numpy(), want["k_codes"])
            assert np.array_equal(v_codes[b, hkv], want["v_codes"])
            assert np.abs(want["q_codes"]).max() == 7 and np.abs(want["k_codes"]).max() == 7
            # the correction: FP32 dot products of d terms against the oracle's doubles
            ref = want["dS"] * (np.float64(np.float32(sm)) * LOG2E)
            err = np.abs(ds_keys[b, hq] - ref).max()
            bound = 4e-7 * d ** 0.5 * (np.abs(want["q_mean"]).max() * np.abs(wl.as_f32(k[b, hkv])).max() * d ** 0.5 * sm * LOG2E) + 1e-6
            assert err <= bound, (err, bound)


def _full_check(q, k, v, base, causal):
    B, Hq, Nq, d = q.shape
    Hkv, Nk = k.shape[1], k.shape[2]
    sm = np.float32(1.0 / np.sqrt(d))
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device=DEV)
    sage.sage_attn_fwd_4bit(q.to(DEV), k.to(DEV), v.to(DEV), causal=causal, sm_scale=float(sm), out=out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all()                       # every element was written
    ref = np.empty(q.shape, dtype=np.float64)
    group = Hq // Hkv
    for b in range(B):
        for hq in range(Hq):
            ref[b, hq], _ = oracle.sage_attention_head_4bit(wl.as_f32(q[b, hq]), wl.as_f32(k[b, hq // group]),
                                                            wl.as_f32(v[b, hq // group]), causal=causal, sm_scale=sm,
                                                            out_dtype=base.dtype)
    assert_parity(ref, got, base.dtype, "4+8", flip_factor=2.0)
    return got, ref


@pytest.mark.parametrize("base_idx,d", [(1, 128), (3, 64)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N", [1, 17, 64, 127, 128, 129, 333, 512, 1000])
def test_4bit_small_and_ragged(base_idx, d, causal, N):
    q, k, v, base = _inputs(base_idx, 1, 2, 2, N, N, d, 1.5, N)
    say(f"[4bit] N{N} d{d} {base.dtype} causal={causal}")
    _full_check(q, k, v, base, causal)


@pytest.mark.parametrize("base_idx,d", [(1, 128), (3, 64), (5, 128), (5, 64)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("B,Hq,Hkv,Nq,Nk", [(2, 4, 2, 300, 300), (1, 4, 1, 100, 700), (1, 2, 2, 1500, 1500),
                                            (1, 6, 3, 257, 384), (1, 4, 2, 1, 1000)])
def test_4bit_gqa_and_rectangular(base_idx, d, causal, B, Hq, Hkv, Nq, Nk):
    q, k, v, base = _inputs(base_idx, B, Hq, Hkv, Nq, Nk, d, 2.0, Nq + Nk)
    say(f"[4bit] B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} d{d} {base.name}-like {base.dtype} causal={causal}")
    _full_check(q, k, v, base, causal)


def test_4bit_stage_calls_equal_the_whole_path():
    q, k, v, base = _inputs(1, 1, 4, 2, 200, 450, 128, 2.0, 7)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    q_mean, _, _ = sage.sage_quant_q4(qd, codes=False)
    k_i4, k_scale, k_mean, v_fp8, v_scale = sage.sage_quant_kv4(kd, vd)
    dsx = sage.sage_delta_s(kd, k_mean, q_mean, 200, causal=True)
    a = sage.sage_attn_fwd_q4(qd, q_mean, k_i4, v_fp8, k_scale, v_scale, dsx, causal=True)
    b = sage.sage_attn_fwd_4bit(qd, kd, vd, causal=True)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("idx", [2, 3])
def test_4bit_full_size_sampled(idx):
    """The causal d=128 and the d=64 benchmark workloads at full size (with an offset on Q), sampled query blocks."""
    cfg = wl.CONFIGS[idx - 1]
    q, k, v = wl.generate(cfg)
    g = torch.Generator().manual_seed(idx)
    q = (q.float() + 2.0 * torch.randn((cfg.B, cfg.H, 1, cfg.d), generator=g)).to(q.dtype)
    say(f"[4bit] full size {cfg.name} B{cfg.B} H{cfg.H} N{cfg.N} d{cfg.d} {cfg.dtype} causal={cfg.causal}")
    sm = np.float32(cfg.sm_scale)
    out = torch.full(q.shape, float("nan"), dtype=q.dtype, device=DEV)
    sage.sage_attn_fwd_4bit(q.to(DEV), k.to(DEV), v.to(DEV), causal=cfg.causal, sm_scale=float(sm), out=out)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    refs, gots, fps = [], [], []
    nq = cfg.N // 128
    for (b, h) in ((0, 0), (cfg.B - 1, cfg.H - 1)):
        qf, kf, vf = (wl.as_f32(t[b, h]) for t in (q, k, v))
        quant = oracle.quantize_head_4bit(qf, kf, vf)
        for i in (0, nq // 2, nq - 1):
            ref, _ = oracle.sage_attention_head_4bit(qf, kf, vf, causal=cfg.causal, sm_scale=sm, out_dtype=cfg.dtype,
                                                     row0=i * 128, row1=(i + 1) * 128, quant=quant)
            refs.append(ref)
            gots.append(out[b, h, i * 128:(i + 1) * 128].float().cpu().numpy())
            fps.append(oracle.attn_rows_fp(qf, kf, vf, causal=cfg.causal, sm_scale=sm, row0=i * 128, row1=(i + 1) * 128))
    ref, got, fp = np.concatenate(refs), np.concatenate(gots), np.concatenate(fps)
    assert_parity(ref, got, cfg.dtype, f"4+8 {cfg.name} sampled {ref.shape[0]} rows", flip_factor=2.0)
    say(f"   vs full precision (reported, parity unpinned): cos={wl.cos_sim(fp, got):.6f} relL1={wl.rel_l1(fp, got):.4f}")


def test_4bit_argument_checks():
    L = sage.lib()
    assert L.sage_workspace_bytes_4bit(1, 3, 2, 64, 64, 128) == 0          # Hq not a multiple of Hkv
    assert L.sage_delta_s_bytes(1, 2, 300, 515) == 2 * 3 * 5 * 128 * 4
    q = torch.zeros((1, 2, 64, 128), dtype=torch.float16, device=DEV)
    ws = torch.zeros(1024, dtype=torch.uint8, device=DEV)
    rc = L.sage_attn_fwd_4bit(q.data_ptr(), q.data_ptr(), q.data_ptr(), q.data_ptr(), 1, 2, 2, 64, 64, 128, 0, 0.0, 0, 0,
                              ws.data_ptr(), ws.numel())
    assert rc == -2                                                        # workspace too small
    qm = torch.zeros((1, 2, 1, 128), dtype=torch.float32, device=DEV)
    assert L.sage_quant_q4(q.data_ptr(), qm.data_ptr(), q.data_ptr(), None, 1, 2, 64, 128, 0, 0) == -1   # codes without scales
    torch.cuda.synchronize()
