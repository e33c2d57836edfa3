"""GPU parity of the two ways libsage quantises K and V together (Sec. 2.1 scales, Sec. 3 smoothing): the
single-read kernel (a head's workgroups keep their tokens in registers and meet once) and the three launches
(statistics, finalize, codes).  Both must produce the oracle's bits: codes, scales and mean.  The single-read
kernel is also run with its wait switched off, so that every workgroup but the last of a head computes the head's
statistic alone from global memory — the branch a workgroup takes when its partners do not show up in time."""
import numpy as np
import pytest
import torch

import paper_2505_21136_amd as sage
import workloads as wl
from gpu_util import oracle_quant_all, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

THREE_LAUNCHES, SINGLE_READ = 1, 2
NAMES = ("k_i8", "k_scale", "k_mean", "v_fp8", "v_scale")


@pytest.fixture(autouse=True)
def _restore_default_path():
    yield
    sage.diag_quant_kv_path(0)


def _quant(k, v, v_r, path, wait_ticks=50_000):
    sage.diag_quant_kv_path(path, wait_ticks)
    out = sage.sage_quant_kv(k, v, v_r)
    torch.cuda.synchronize()
    return out


def _same_bits(a, b, what):
    for name, x, y in zip(NAMES, a, b):
        assert x.shape == y.shape and x.dtype == y.dtype, (what, name)
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), (what, name)


def _against_oracle(out, k, v, v_r, N):
    k_i8, k_scale, k_mean, v_fp8, v_scale = out
    want = oracle_quant_all(wl.as_f32(k.cpu()), wl.as_f32(k.cpu()), wl.as_f32(v.cpu()), v_r)
    for name, got in (("k_codes", k_i8), ("k_scale", k_scale), ("k_mean", k_mean), ("v_scale", v_scale),
                      ("v_codes", sage.v_fp8_to_token_major(v_fp8, N))):
        g, w = got.cpu().numpy(), want[name]
        assert g.shape == w.shape, name
        assert np.array_equal(g.view(np.uint8), w.view(np.uint8)), f"{name}: {np.sum(g != w)} of {g.size} differ"


def _inputs(idx, shape):
    base = wl.CONFIGS[idx - 1]
    B, H, N, d = shape
    cfg = wl.Workload("kv", base.index, B, H, N, d, False, base.dtype, base.q_dist, base.k_outlier_channels)
    _, k, v = wl.generate(cfg)
    return k.to(DEV), v.to(DEV)


# one chunk of a head is 256 tokens at d = 128 and 512 at d = 64: shapes below, at and across those borders,
# with ragged K blocks (64), V tiles (128) and chunks
SHAPES = [(1, (1, 2, 1, 128)), (1, (2, 3, 63, 128)), (2, (1, 3, 255, 128)), (2, (2, 2, 256, 128)),
          (5, (1, 3, 257, 128)), (5, (2, 3, 777, 128)), (1, (1, 2, 1024, 128)), (5, (1, 2, 2049, 128)),
          (3, (1, 4, 1, 64)), (3, (2, 3, 129, 64)), (4, (1, 2, 511, 64)), (4, (2, 2, 512, 64)),
          (3, (1, 3, 513, 64)), (4, (1, 2, 4500, 64))]


@pytest.mark.parametrize("idx,shape", SHAPES)
def test_single_read_kernel_equals_the_three_launches_and_the_oracle(idx, shape):
    say(f"[quant paths] cfg{idx} distributions, shape {shape}")
    k, v = _inputs(idx, shape)
    three = _quant(k, v, 4.5, THREE_LAUNCHES)
    single = _quant(k, v, 4.5, SINGLE_READ)
    _same_bits(three, single, "single-read vs three launches")
    _against_oracle(single, k, v, 4.5, shape[2])


@pytest.mark.parametrize("idx,shape", [(2, (2, 3, 777, 128)), (5, (1, 2, 2049, 128)), (4, (1, 2, 4500, 64)),
                                       (3, (2, 2, 512, 64))])
def test_workgroups_that_do_not_wait_compute_the_statistic_alone(idx, shape):
    say(f"[quant paths] no wait, cfg{idx} distributions, shape {shape}")
    k, v = _inputs(idx, shape)
    three = _quant(k, v, 4.5, THREE_LAUNCHES)
    alone = _quant(k, v, 4.5, SINGLE_READ, wait_ticks=-1)
    _same_bits(three, alone, "no-wait single-read vs three launches")


@pytest.mark.parametrize("wait_ticks", [0, 1, 100])
@pytest.mark.parametrize("idx,shape", [(2, (2, 3, 2049, 128)), (4, (1, 2, 4500, 64))])
def test_a_wait_that_runs_out_ends_in_the_stand_alone_branch(idx, shape, wait_ticks):
    """The bounded wait itself: with a bound of 0, 10 ns or 1 us a workgroup polls once or a few times and, unless all
    its partners are already there, gives up and computes the statistic alone.  Same bits, and the launch ends."""
    say(f"[quant paths] wait bound {wait_ticks} ticks, cfg{idx} distributions, shape {shape}")
    k, v = _inputs(idx, shape)
    three = _quant(k, v, 4.5, THREE_LAUNCHES)
    short = _quant(k, v, 4.5, SINGLE_READ, wait_ticks=wait_ticks)
    _same_bits(three, short, f"wait bound {wait_ticks}")


def test_repeated_calls_reuse_the_workspace():
    """The partial buffers, whose zero words mean "not there yet", are cleared by the call itself: back-to-back
    calls on one workspace that starts full of garbage, the second on other data, each give their own result."""
    k1, v1 = _inputs(2, (2, 4, 1500, 128))
    k2, v2 = _inputs(5, (2, 4, 1500, 128))
    want1 = _quant(k1, v1, 4.5, THREE_LAUNCHES)
    want2 = _quant(k2, v2, 2.25, THREE_LAUNCHES)
    sage.diag_quant_kv_path(SINGLE_READ)
    B, H, N, d = k1.shape
    ws = torch.empty(sage.quant_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=DEV).fill_(0xA5)
    outs = []
    for k, v, v_r in ((k1, v1, 4.5), (k2, v2, 2.25), (k1, v1, 4.5)):
        outs.append(sage.sage_quant_kv(k, v, v_r, workspace=ws))
    torch.cuda.synchronize()
    _same_bits(want1, outs[0], "call 1")
    _same_bits(want2, outs[1], "call 2")
    _same_bits(want1, outs[2], "call 3")


def test_partials_that_are_exactly_zero():
    """A partial column sum of +0.0 and a partial maximum of 0.0 travel as -0.0 (a zero word means "not there"):
    chunks of zeros, columns that cancel inside a chunk, a head of zeros."""
    k, v = _inputs(5, (1, 3, 1024, 128))
    k[0, 0, 256:512] = 0                      # a whole chunk of K is zero
    k[0, 1, 0:256:2] = 1.5
    k[0, 1, 1:256:2] = -1.5                   # every column of the first chunk sums to +0.0
    k[0, 2] = 0                               # a head of zeros
    v[0, 0, 0:256] = 0
    v[0, 2] = 0
    three = _quant(k, v, 4.5, THREE_LAUNCHES)
    single = _quant(k, v, 4.5, SINGLE_READ)
    _same_bits(three, single, "zero partials")
    _against_oracle(single, k, v, 4.5, 1024)


def test_single_read_kernel_next_to_a_kernel_that_holds_the_cus():
    """The workgroups of a head meet inside one launch.  With another stream's attention kernel holding the CUs the
    partners of a workgroup may arrive late or (after the wait bound) not in time at all; the result must be the
    same bits either way, and every launch must end."""
    cfg = wl.CONFIGS[4].scaled(H=8)                       # B1 H8 N32768 d128: an attention launch of ~2.5 ms
    q, kk, vv = (t.to(DEV) for t in wl.generate(cfg))
    k, v = _inputs(2, (4, 16, 4096, 128))
    want = _quant(k, v, 4.5, THREE_LAUNCHES)
    sage.diag_quant_kv_path(SINGLE_READ, 20_000)          # 0.2 ms: short enough for some waits to run out
    B, H, N, d = k.shape
    ws = torch.empty(sage.quant_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=DEV)
    ws_a = torch.empty(sage.workspace_bytes(cfg.B, cfg.H, cfg.N, cfg.d), dtype=torch.uint8, device=DEV)
    out_a = torch.empty_like(q)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    got = []
    for rep in range(3):
        with torch.cuda.stream(side):
            sage.sage_attn_fwd(q, kk, vv, causal=False, out=out_a, workspace=ws_a)
            sage.sage_attn_fwd(q, kk, vv, causal=False, out=out_a, workspace=ws_a)
        got.append(sage.sage_quant_kv(k, v, 4.5, workspace=ws))       # default stream, concurrent with `side`
        got.append(sage.sage_quant_kv(k, v, 4.5, workspace=ws))
        torch.cuda.synchronize()
    for i, g in enumerate(got):
        _same_bits(want, g, f"concurrent call {i}")


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_full_size_workloads_on_the_single_read_kernel(idx):
    cfg = wl.CONFIGS[idx - 1]
    say(f"[quant paths] full size {cfg.name}")
    _, k, v = wl.generate(cfg)
    k, v = k.to(DEV), v.to(DEV)
    three = _quant(k, v, 4.5, THREE_LAUNCHES)
    single = _quant(k, v, 4.5, SINGLE_READ)
    _same_bits(three, single, cfg.name)


def test_forced_single_read_above_its_group_limit_is_an_error():
    k, v = _inputs(3, (1, 1, 512 * 256 + 1, 64))       # 257 chunks of 512 tokens
    sage.diag_quant_kv_path(SINGLE_READ)
    with pytest.raises(RuntimeError):
        sage.sage_quant_kv(k, v, 4.5)
    sage.diag_quant_kv_path(0)
    out = sage.sage_quant_kv(k, v, 4.5)                 # by shape: the three launches
    torch.cuda.synchronize()
    assert out[0].shape == k.shape
