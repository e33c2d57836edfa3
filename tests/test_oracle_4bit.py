"""Pins of the oracle's 4+8 variant (paper Section 2.1 "INT4/INT8 with per-block granularity", Section 3
"smoothing of Q and K", Section 4.1 "SageAttn2++(4+8)"): INT4 codes, smoothing of Q by its block means, and the
score correction dS = qbar K'^T that puts back what the smoothing removed.

* each quantiser step against an independent library routine (numpy.rint, numpy float64 means / products);
* a lossless regime -- inputs on which every quantiser is exact although Q carries a different offset in every
  block -- where the whole pipeline must reproduce brute-force softmax(Q K^T) V on the UNSMOOTHED inputs: a
  dropped, mis-indexed or mis-signed correction term fails it;
* a one-step direct formula with torch's float8 cast as the rounding routine;
* identities: zero block means make the correction vanish; the correction is what makes the result independent
  of a constant added to a Q block's rows (up to quantisation noise, which smoothing is there to remove).
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_oracle_attention import LOG2E, brute_force


# --------------------------------------------------------------------------
# quantiser steps
# --------------------------------------------------------------------------
@pytest.mark.parametrize("qmax", [7, 127])
@pytest.mark.parametrize("N,d,block", [(100, 16, 32), (64, 8, 64), (130, 64, 128)])
def test_quant_int_matches_numpy_rint(qmax, N, d, block):
    rng = np.random.default_rng(N + qmax)
    X = rng.standard_normal((N, d)).astype(np.float32) * 3
    mu = rng.standard_normal(d).astype(np.float32)
    codes, delta = oracle.quant_int(X, mu, block, qmax)
    assert codes.min() >= -qmax and codes.max() <= qmax
    for j in range(-(-N // block)):
        xs = X[j * block:(j + 1) * block] - mu          # float32 arithmetic, as defined
        a = np.abs(xs).max()
        assert delta[j] == np.float32(a) / np.float32(qmax)
        r = np.float32(qmax) / np.float32(a)
        want = np.rint(xs * r).astype(np.int8)
        assert np.array_equal(codes[j * block:(j + 1) * block], want)
        assert np.abs(want).max() == qmax                # the block's extreme value maps to +-qmax
        assert np.abs(xs - delta[j] * want.astype(np.float32)).max() <= delta[j] * 0.5 * (1 + 1e-6)
    if qmax == 127:                                     # the general routine contains the 8-bit one
        c8, d8 = oracle.quant_int8(X, mu, block)
        assert np.array_equal(c8, codes) and np.array_equal(d8, delta)


def test_quant_int_ties_zero_block_and_block_means():
    X = np.array([[3.5, -3.5, 2.5, 7.0], [0.5, 1.5, -0.5, -7.0]], dtype=np.float32)   # a = 7: codes = rint(x)
    codes, delta = oracle.quant_int(X, None, 2, 7)
    assert delta[0] == 1.0 and codes.tolist() == [[4, -4, 2, 7], [0, 2, 0, -7]]       # ties go to even
    codes, delta = oracle.quant_int(np.zeros((5, 4), np.float32), None, 4, 7)
    assert not codes.any() and not delta.any()
    # per-block means: block 0 and block 1 of three rows each get their own offset removed
    X = np.array([[1, 2], [3, 2], [5, 2], [10, 0], [10, 7], [10, -7]], dtype=np.float32)
    qbar = oracle.block_mean(X, 3)
    assert qbar.tolist() == [[3.0, 2.0], [10.0, 0.0]]
    codes, delta = oracle.quant_int(X, qbar, 3, 7)
    assert codes.tolist() == [[-7, 0], [0, 0], [7, 0], [0, 0], [0, 7], [0, -7]]
    assert delta.tolist() == [np.float32(2) / np.float32(7), 1.0]


@pytest.mark.parametrize("N,d,block", [(300, 64, 128), (128, 128, 128), (77, 16, 32)])
def test_block_mean_smooth_and_delta_s_match_numpy(N, d, block):
    rng = np.random.default_rng(N)
    Q = (rng.standard_normal((N, d)) + 2.0).astype(np.float32)
    K = (rng.standard_normal((N + 5, d)) * 3).astype(np.float32)
    qbar = oracle.block_mean(Q, block)
    nb = -(-N // block)
    for i in range(nb):
        want = Q[i * block:(i + 1) * block].astype(np.float64).mean(axis=0).astype(np.float32)
        assert np.array_equal(qbar[i], want)
    assert np.array_equal(oracle.smooth(Q, qbar, block), Q - qbar[np.arange(N) // block])     # float32 subtraction
    mu = oracle.k_mean(K)
    Kp = oracle.smooth(K, mu)
    assert np.array_equal(Kp, K - mu)
    dS = oracle.delta_s(qbar, Kp)
    want = qbar.astype(np.float64) @ Kp.astype(np.float64).T
    assert dS.shape == (nb, N + 5) and np.abs(dS - want).max() <= 1e-12 * np.abs(want).max()


# --------------------------------------------------------------------------
# whole pipeline, lossless regime
# --------------------------------------------------------------------------
def _lossless_problem_4bit(N, bq, bk, q_exps, k_exps, two_hot, seed):
    """Inputs on which every quantiser of the 4+8 variant is exact.

    K^ has entries in {-1,0,1} on six channels in +/- row pairs (zero channel means) plus a +-7 channel that
    fixes each block's range; K = K^ * 2^b_j.  Q^ rows are one- or two-hot with weight +-7, also in +/- row
    pairs, so every block of Q^ has zero channel sums; Q = Q^ * 2^a_i + o_i with a one-hot offset o_i = +-7 that
    differs from block to block: the block mean of Q is exactly o_i and Q - mean is exactly Q^ * 2^a_i.  With
    sm_scale = ln2/7 every base-2 score -- the quantised part 2^(a+b) * {-2..2} plus the correction
    2^b * {-1,0,1} -- is a small integer, P~ a power of two and P~ * 224 an FP8 value."""
    assert N % 2 == 0 and bk % 2 == 0 and bq % 2 == 0
    rng = np.random.default_rng(seed)
    d = 8
    Kh = np.zeros((N, d))
    half = rng.integers(-1, 2, size=(N // 2, 6))
    Kh[0::2, :6], Kh[1::2, :6] = half, -half
    Kh[0::2, 6], Kh[1::2, 6] = 7, -7
    Qh = np.zeros((N, d))
    for r in range(0, N, 2):
        a, b = rng.choice(6, size=2, replace=False)
        Qh[r, a] = 7 * rng.choice([-1, 1])
        if two_hot:
            Qh[r, b] = 7 * rng.choice([-1, 1])
        Qh[r + 1] = -Qh[r]
    nq, nk = -(-N // bq), -(-N // bk)
    a_i = np.array([q_exps[i % len(q_exps)] for i in range(nq)])
    b_j = np.array([k_exps[j % len(k_exps)] for j in range(nk)])
    off = np.zeros((nq, d))
    off[np.arange(nq), rng.integers(0, 6, size=nq)] = 7 * rng.choice([-1, 1], size=nq)
    Q = Qh * np.exp2(a_i)[np.arange(N) // bq, None] + off[np.arange(N) // bq]
    K = Kh * np.exp2(b_j)[np.arange(N) // bk, None]
    fp8_vals = oracle.e4m3_decode(np.arange(256, dtype=np.uint8))
    fp8_vals = fp8_vals[np.isfinite(fp8_vals) & (np.abs(fp8_vals) <= 4.5)]
    Vh = rng.choice(fp8_vals, size=(N, d))
    Vh[rng.integers(0, N, size=d), np.arange(d)] = 4.5
    e_c = rng.integers(-2, 3, size=d)
    V = Vh * np.exp2(e_c)[None, :]
    return Q, K, V, dict(Qh=Qh, Kh=Kh, off=off, a_i=a_i, b_j=b_j)


@pytest.mark.parametrize("N,bq,bk,w,q_exps,k_exps,two_hot", [
    (64, 16, 8, 16, (0, 1), (0,), True),
    (64, 16, 8, 16, (0,), (0, 1), True),
    (64, 16, 8, 16, (0, 1), (1, 0), False),
    (50, 16, 8, 16, (1, 0), (0,), True),         # ragged tail in every blocking
    (260, 128, 64, 128, (0, 1, 0), (0,), True),  # the production block sizes, 3 steps
    (36, 8, 4, 12, (0,), (0, 1, 0), True),       # a step spans three K blocks
])
@pytest.mark.parametrize("causal", [False, True])
def test_4bit_pipeline_is_exact_when_quantisers_are_lossless(N, bq, bk, w, q_exps, k_exps, two_hot, causal):
    Q, K, V, t = _lossless_problem_4bit(N, bq, bk, q_exps, k_exps, two_hot, seed=N + w)
    sm_scale = math.log(2.0) / 7.0
    quant = oracle.quantize_head_4bit(Q.astype(np.float32), K.astype(np.float32), V.astype(np.float32), bq=bq, bk=bk)
    # the quantisers recovered the construction
    assert not quant["k_mean"].any() and np.array_equal(quant["q_mean"], t["off"])
    assert np.array_equal(quant["q_codes"], t["Qh"]) and np.array_equal(quant["k_codes"], t["Kh"])
    assert np.array_equal(quant["q_scale"], np.exp2(t["a_i"])) and np.array_equal(quant["k_scale"], np.exp2(t["b_j"]))
    assert np.abs(quant["dS"]).max() > 0
    out, _ = oracle.sage_attention_head_4bit(None, None, None, causal=causal, sm_scale=sm_scale, out_dtype=None,
                                             bq=bq, bk=bk, w=w, quant=quant)
    ref, _ = brute_force(Q, K, V, sm_scale, causal)          # on the unsmoothed inputs
    assert np.abs(out - ref).max() <= 1e-12 * np.abs(ref).max()
    # without the correction the same codes give a different answer: the regime does exercise it
    no_ds = oracle.attn_rows(quant["q_codes"], quant["k_codes"], quant["v_codes"], quant["q_scale"], quant["k_scale"],
                             quant["v_scale"], causal=causal, sm_scale=sm_scale, bq=bq, bk=bk, w=w, out_dtype=None)
    assert np.abs(no_ds - ref).max() > 1e-3 * np.abs(ref).max()


# --------------------------------------------------------------------------
# general inputs
# --------------------------------------------------------------------------
def _head(cfg_index, N, q_offset, seed):
    base = wl.CONFIGS[cfg_index - 1]
    cfg = wl.Workload("q4", base.index, 1, 1, N, base.d, False, base.dtype, base.q_dist, base.k_outlier_channels)
    q, k, v = (wl.as_f32(t[0, 0]).copy() for t in wl.generate(cfg, seed=seed))
    if q_offset:
        rng = np.random.default_rng(seed)
        q += (q_offset * rng.standard_normal(base.d)).astype(np.float32)      # what smoothing of Q is for
        q = torch.from_numpy(q).to(wl.torch_dtype(base.dtype)).float().numpy()
    return q, k, v, base


@pytest.mark.parametrize("cfg,N", [(1, 100), (3, 128), (5, 90)])
@pytest.mark.parametrize("causal", [False, True])
def test_one_step_matches_direct_formula(cfg, N, causal):
    """N <= W: one key step, so m is the row maximum and
    O = (sum_n fp8(P~_n P_r) V^_n) delta_V / (P_r sum_n P~_n),  P~ = 2^(x - rowmax x),
    x = (Q^ K^^T delta_Q delta_K + qbar K'^T) sm_scale log2 e, with torch's float8 cast as the rounding routine."""
    q, k, v, base = _head(cfg, N, 2.0, 21)
    quant = oracle.quantize_head_4bit(q, k, v)
    out, _ = oracle.sage_attention_head_4bit(q, k, v, causal=causal, sm_scale=base.sm_scale, out_dtype=None, quant=quant)
    S = quant["q_codes"].astype(np.int64) @ quant["k_codes"].astype(np.int64).T
    scale = quant["q_scale"].astype(np.float64)[0] * quant["k_scale"].astype(np.float64)[np.arange(N) // 64][None, :]
    Kp = (k - quant["k_mean"]).astype(np.float64)
    x = (S * scale + quant["q_mean"].astype(np.float64)[0][None, :] @ Kp.T) * base.sm_scale * LOG2E
    if causal:
        x = np.where(np.arange(N)[None, :] <= np.arange(N)[:, None], x, -np.inf)
    Pt = np.exp2(x - x.max(axis=1, keepdims=True))
    Ph = torch.from_numpy((Pt * 224.0).astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    Vh = torch.from_numpy(quant["v_codes"]).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ref = (Ph @ Vh) * quant["v_scale"].astype(np.float64)[None, :] / (224.0 * Pt.sum(axis=1, keepdims=True))
    close = np.isclose(out, ref, rtol=1e-9, atol=1e-12)
    assert close.mean() > 0.97 and wl.rel_l1(ref, out) < 2e-4


def test_zero_block_means_make_the_correction_vanish():
    q, k, v, base = _head(1, 256, 0.0, 22)
    q[:128] -= q[:128].astype(np.float64).mean(axis=0).astype(np.float32)
    q[128:] = q[:128]                                    # both blocks: channel means (nearly) zero
    quant = oracle.quantize_head_4bit(q, k, v)
    assert np.abs(quant["q_mean"]).max() < 1e-6
    a, _ = oracle.sage_attention_head_4bit(q, k, v, causal=False, sm_scale=base.sm_scale, out_dtype="fp16", quant=quant)
    b = oracle.attn_rows(quant["q_codes"], quant["k_codes"], quant["v_codes"], quant["q_scale"], quant["k_scale"],
                         quant["v_scale"], causal=False, sm_scale=base.sm_scale, out_dtype="fp16")
    assert wl.rel_l1(a, b) < 1e-4


@pytest.mark.parametrize("cfg", [1, 3])
def test_smoothing_of_q_is_what_keeps_int4_accurate(cfg):
    """Plausibility (parity unpinned: no figure of the paper covers synthetic data): with a large common offset
    on Q the INT4 grid of the unsmoothed Q is spent on the offset; smoothing removes it and the correction term
    restores the scores, so the 4+8 result stays close to full precision and far closer than without smoothing."""
    q, k, v, base = _head(cfg, 512, 4.0, 23)
    fp = oracle.attn_rows_fp(q, k, v, causal=False, sm_scale=base.sm_scale)
    smooth, _ = oracle.sage_attention_head_4bit(q, k, v, causal=False, sm_scale=base.sm_scale, out_dtype=None)
    quant = oracle.quantize_head_4bit(q, k, v)
    qc, qs = oracle.quant_int(q, None, 128, 7)          # INT4 of the unsmoothed Q
    plain = oracle.attn_rows(qc, quant["k_codes"], quant["v_codes"], qs, quant["k_scale"], quant["v_scale"],
                             causal=False, sm_scale=base.sm_scale, out_dtype=None)
    l_smooth, l_plain = wl.rel_l1(fp, smooth), wl.rel_l1(fp, plain)
    assert wl.cos_sim(fp, smooth) > 0.98 and l_smooth < 0.25
    assert l_plain > 1.5 * l_smooth


def test_rows_are_independent_and_output_is_on_the_16_bit_grid():
    q, k, v, base = _head(3, 300, 1.0, 24)
    quant = oracle.quantize_head_4bit(q, k, v)
    full, _ = oracle.sage_attention_head_4bit(q, k, v, causal=True, sm_scale=base.sm_scale, out_dtype="bf16", quant=quant)
    part, _ = oracle.sage_attention_head_4bit(q, k, v, causal=True, sm_scale=base.sm_scale, out_dtype="bf16", quant=quant,
                                              row0=130, row1=257)
    assert np.array_equal(full[130:257], part)
    assert np.array_equal(torch.from_numpy(full).to(torch.bfloat16).double().numpy(), full)
