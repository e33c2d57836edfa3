"""Pins of the oracle's quantisation stage (paper Section 2.1, Section 3 and Eq. 2).

Independent checks: numpy's float64 mean, numpy.rint on float32 arrays and
torch's float8 cast as library roundings, error bounds, scale invariances and
structural properties.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def _head(cfg_index, N, seed=None):
    base = wl.CONFIGS[cfg_index - 1]
    q, k, v = wl.generate(base.scaled(B=1, H=1, N=N), seed=seed)
    return tuple(wl.as_f32(t)[0, 0] for t in (q, k, v))


@pytest.mark.parametrize("cfg,N", [(1, 300), (3, 257), (5, 200)])
def test_k_mean_is_the_channel_mean(cfg, N):
    _, k, _ = _head(cfg, N)
    mu = oracle.k_mean(k)
    want = (k.astype(np.float64).sum(axis=0) / N).astype(np.float32)
    assert mu.dtype == np.float32 and np.array_equal(mu, want)
    # the cfg bias (std 3, shared across tokens) dominates the mean: smoothing removes it
    assert np.abs(mu).mean() > 1.0
    assert np.abs((k - mu).mean(axis=0)).max() < 1e-5 * max(1.0, np.abs(k).max())


@pytest.mark.parametrize("cfg,N,block", [(1, 300, 128), (1, 300, 64), (3, 129, 64), (5, 200, 128), (4, 48, 64)])
def test_int8_blocks_follow_the_rounding_rule(cfg, N, block):
    q, k, _ = _head(cfg, N)
    for X, mu in ((q, None), (k, oracle.k_mean(k))):
        codes, delta = oracle.quant_int8(X, mu, block)
        Xs = X if mu is None else (X - mu[None, :]).astype(np.float32)
        nb = (N + block - 1) // block
        assert codes.shape == X.shape and delta.shape == (nb,)
        assert codes.min() >= -127 and codes.max() <= 127
        for j in range(nb):
            blk = Xs[j * block:(j + 1) * block]
            a = np.abs(blk).max()
            # scale definition of Section 2.1
            assert delta[j] == np.float32(a) / np.float32(127.0)
            # independent library rounding (numpy.rint is round-half-even) of the float32 product
            want = np.rint(blk * (np.float32(127.0) / np.float32(a))).astype(np.int8)
            got = codes[j * block:(j + 1) * block]
            assert np.array_equal(got, want)
            # nearest-code property against the real quotient, and the block maximum hits +-127
            err = np.abs(blk.astype(np.float64) - got.astype(np.float64) * float(delta[j]))
            assert err.max() <= 0.5 * float(delta[j]) * (1 + 1e-5)
            assert np.abs(got).max() == 127


def test_int8_ties_round_to_even_and_zero_blocks():
    # block maximum 127 => r = 1: codes are rint(x); halves are exact ties
    X = np.zeros((4, 8), dtype=np.float32)
    X[0] = [127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]
    X[1] = [126.5, 125.5, -126.5, 0.49999997, 0.50000006, -3.5, 64.5, 63.5]
    codes, delta = oracle.quant_int8(X, None, 2)
    assert delta[0] == 1.0
    assert codes[0].tolist() == [127, 0, 2, 2, 0, -2, -2, 4]
    assert codes[1].tolist() == [126, 126, -126, 0, 1, -4, 64, 64]
    # all-zero second block: scale 0, codes 0
    assert delta[1] == 0.0 and not codes[2:].any()


def test_int8_scale_invariance_power_of_two():
    q, _, _ = _head(1, 256)
    c0, d0 = oracle.quant_int8(q, None, 128)
    for k in (-3, 5):
        c1, d1 = oracle.quant_int8(q * np.float32(2.0 ** k), None, 128)
        assert np.array_equal(c0, c1) and np.array_equal(d1, d0 * np.float32(2.0 ** k))


def test_int8_partial_block_uses_valid_rows_only():
    q, _, _ = _head(1, 130)
    c_all, d_all = oracle.quant_int8(q, None, 64)
    c_tail, d_tail = oracle.quant_int8(q[128:], None, 64)
    assert d_all.shape == (3,) and d_all[2] == d_tail[0]
    assert np.array_equal(c_all[128:], c_tail)


def test_smoothing_changes_k_codes_but_uses_one_mean_per_channel():
    _, k, _ = _head(1, 256)
    mu = oracle.k_mean(k)
    c_s, d_s = oracle.quant_int8(k, mu, 64)
    c_n, d_n = oracle.quant_int8(k, None, 64)
    # with the bias removed the block range shrinks, i.e. finer steps (the point of smoothing)
    assert np.all(d_s < d_n)
    # quantising the explicitly smoothed tensor gives the same codes
    c_e, d_e = oracle.quant_int8((k - mu[None, :]).astype(np.float32), None, 64)
    assert np.array_equal(c_s, c_e) and np.array_equal(d_s, d_e)


@pytest.mark.parametrize("cfg,N,v_r", [(1, 300, 4.5), (3, 129, 4.5), (1, 200, 448.0), (1, 200, 2.25), (1, 77, 9.0)])
def test_v_fp8_per_channel(cfg, N, v_r):
    _, _, v = _head(cfg, N)
    codes, delta = oracle.quant_v(v, v_r)
    a = np.abs(v).max(axis=0)
    assert np.array_equal(delta, a / np.float32(v_r))                     # Eq. 2
    prod = v * (np.float32(v_r) / a)[None, :]                             # float32 products
    assert prod.dtype == np.float32
    want = torch.from_numpy(prod).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(codes, want)
    dec = oracle.e4m3_decode(codes)
    # every channel's extreme element maps onto +-V_r exactly
    assert np.array_equal(np.abs(dec).max(axis=0), np.full(v.shape[1], v_r))
    # reconstruction error: half an FP8 step (2^-4 relative above the subnormal range)
    rec = dec * delta[None, :].astype(np.float64)
    tol = np.maximum(np.abs(v) * 2.0 ** -4, delta[None, :] * 2.0 ** -10) * (1 + 1e-5)
    assert np.all(np.abs(rec - v) <= tol)


def test_v_scale_invariance_and_zero_channel():
    _, _, v = _head(1, 128)
    v[:, 5] = 0.0
    c0, d0 = oracle.quant_v(v, 4.5)
    c1, d1 = oracle.quant_v(v * np.float32(8.0), 4.5)
    assert np.array_equal(c0, c1) and np.array_equal(d1, d0 * np.float32(8.0))
    assert d0[5] == 0.0 and not c0[:, 5].any()


def test_generator_is_seeded_and_shaped():
    for cfg in wl.CONFIGS:
        small = cfg.scaled(B=1, H=2, N=96)
        a = wl.generate(small)
        b = wl.generate(small)
        for x, y in zip(a, b):
            assert x.dtype == wl.torch_dtype(cfg.dtype) and x.shape == (1, 2, 96, cfg.d)
            assert torch.equal(x, y)
    q, k, _ = wl.generate(wl.CONFIGS[4].scaled(B=1, H=1, N=4096))
    kf = wl.as_f32(k)[0, 0]
    # four outlier channels (x20) stand out in the per-channel spread
    spread = kf.std(axis=0)
    assert (spread > 10).sum() == 4 and (spread < 2).sum() == kf.shape[1] - 4
    # heavy-tailed Q
    assert np.abs(wl.as_f32(q)).max() > 15
