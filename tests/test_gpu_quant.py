"""GPU parity, stage 1: codes and scales of libsage must equal the oracle's bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import assert_quant_bit_exact, gpu_quant_all, oracle_quant_all, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(cfg, v_r=4.5, seed=None):
    say(f"[quant] {cfg.name} B{cfg.B} H{cfg.H} N{cfg.N} d{cfg.d} {cfg.dtype} v_r={v_r}")
    q, k, v = wl.generate(cfg, seed=seed)
    got, _ = gpu_quant_all(q.to(DEV), k.to(DEV), v.to(DEV), v_r)
    want = oracle_quant_all(wl.as_f32(q), wl.as_f32(k), wl.as_f32(v), v_r)
    assert_quant_bit_exact(got, want)


@pytest.mark.parametrize("idx", [1, 3, 5])
@pytest.mark.parametrize("N", [1, 3, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000])
def test_quant_small_and_ragged(idx, N):
    _run(wl.CONFIGS[idx - 1].scaled(B=2, H=3, N=N))


@pytest.mark.parametrize("v_r", [448.0, 2.25, 9.0])
def test_quant_other_ranges(v_r):
    _run(wl.CONFIGS[0].scaled(B=1, H=2, N=300), v_r=v_r)


def test_quant_cfg1_full():
    _run(wl.CONFIGS[0])


def test_fp8_conversion_exhaustive_through_v():
    """Every fp16 value of magnitude <= 4.5 goes through the hardware FP8 conversion with
    multiplier exactly 1 (channel maximum 4.5): all FP8 midpoints, subnormals and signed zeros."""
    bits = np.arange(0x10000, dtype=np.uint32).astype(np.uint16)
    vals = bits.view(np.float16)
    keep = np.isfinite(vals) & (np.abs(vals.astype(np.float32)) <= 4.5)
    vals = vals[keep]
    d = 64
    n = -(-vals.size // d)
    pad = np.zeros(n * d, dtype=np.float16)
    pad[:vals.size] = vals
    mat = pad.reshape(n, d).copy()
    mat[0, :] = 4.5       # every channel has maximum exactly 4.5 -> multiplier 1
    mat = np.concatenate([mat, pad.reshape(n, d)[:1]])    # keep the values row 0 displaced
    v = torch.from_numpy(mat)[None, None].contiguous()
    say(f"[quant] exhaustive fp8: {v.shape}")
    v_fp8, v_scale = sage.sage_quant_v(v.to(DEV))
    torch.cuda.synchronize()
    got = sage.v_fp8_to_token_major(v_fp8, mat.shape[0]).cpu().numpy()[0, 0]
    codes, delta = oracle.quant_v(mat.astype(np.float32), 4.5)
    assert np.array_equal(v_scale.cpu().numpy()[0, 0], delta) and np.all(delta == 1.0)
    assert np.array_equal(got, codes)
    # and against an independent library rounding
    lib = torch.from_numpy(mat.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, lib)


def test_degenerate_inputs():
    cfg = wl.CONFIGS[0].scaled(B=1, H=2, N=200)
    q, k, v = wl.generate(cfg)
    k[0, 0] = k[0, 0, :1]          # identical keys: smoothed K is zero, scale 0
    q[0, 1, 128:] = 0              # an all-zero Q block
    v[0, 1, :, 7] = 0              # an all-zero V channel
    got, _ = gpu_quant_all(q.to(DEV), k.to(DEV), v.to(DEV))
    want = oracle_quant_all(wl.as_f32(q), wl.as_f32(k), wl.as_f32(v))
    assert_quant_bit_exact(got, want)
    assert not got["k_scale"][0, 0].any() and got["q_scale"][0, 1, 1] == 0 and got["v_scale"][0, 1, 7] == 0


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_quant_full_size_configs(idx):
    _run(wl.CONFIGS[idx - 1])


@pytest.mark.parametrize("idx,shape", [(1, (1, 2, 1024, 128)), (2, (2, 3, 777, 128)), (3, (1, 4, 1, 64)),
                                       (4, (1, 2, 4500, 64)), (5, (1, 2, 2049, 128))])
def test_joint_kv_quantiser_equals_the_separate_calls(idx, shape):
    """sage_quant_kv shares the launches of K and V; every output must be the same bits."""
    base = wl.CONFIGS[idx - 1]
    B, H, N, d = shape
    cfg = wl.Workload("kv", base.index, B, H, N, d, False, base.dtype, base.q_dist, base.k_outlier_channels)
    _, k, v = wl.generate(cfg)
    k, v = k.to("cuda:0"), v.to("cuda:0")
    k_i8, k_scale, k_mean = sage.sage_quant_k(k)
    v_fp8, v_scale = sage.sage_quant_v(v, 4.5)
    joint = sage.sage_quant_kv(k, v, 4.5)
    torch.cuda.synchronize()
    for name, a, b in zip(("k_i8", "k_scale", "k_mean", "v_fp8", "v_scale"), (k_i8, k_scale, k_mean, v_fp8, v_scale),
                          joint):
        assert a.shape == b.shape and a.dtype == b.dtype, name
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), name
