"""Pins of the oracle's study mode delta_p="block_max" (paper Section 3.1, Eq. 2 read literally: the scale of
P~ is the maximum of each (Q block x key step) block over P_r).

* lossless regime: every quantiser exact -> the pipeline must reproduce brute-force softmax attention for any
  block maximum (a dropped or misplaced factor b shows wherever a block's maximum is below one);
* a two-step direct formula with torch's float8 cast as the rounding routine, on data where the extent of the
  maximum (block, not row) changes the FP8 codes;
* where every block holds some row's running maximum the mode coincides with the static scale.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_oracle_attention import LOG2E, _lossless_problem, brute_force


def _args(quant):
    return (quant["q_codes"], quant["k_codes"], quant["v_codes"], quant["q_scale"], quant["k_scale"], quant["v_scale"])


@pytest.mark.parametrize("N,bq,bk,w,q_exps,k_exps,two_hot", [
    (64, 16, 8, 16, (0, 1), (0,), True),
    (64, 4, 8, 8, (0,), (0, 1), True),           # small blocks: many blocks hold no row maximum
    (50, 2, 8, 8, (1, 0), (0,), True),           # ragged tail
    (260, 128, 64, 128, (0, 1, 0), (0,), True),  # the production block sizes, 3 steps
    (36, 1, 4, 4, (0,), (0, 1, 0), False),       # one-row blocks: the block maximum is the row's step maximum
    (36, 8, 4, 12, (0,), (0, 1, 0), True),
])
@pytest.mark.parametrize("causal", [False, True])
def test_block_max_pipeline_is_exact_when_quantisers_are_lossless(N, bq, bk, w, q_exps, k_exps, two_hot, causal):
    Q, K, V, _ = _lossless_problem(N, bq, bk, q_exps, k_exps, two_hot, seed=N + w)
    sm_scale = math.log(2.0) / 127.0
    quant = oracle.quantize_head(Q.astype(np.float32), K.astype(np.float32), V.astype(np.float32), v_r=4.5, bq=bq, bk=bk)
    out = oracle.attn_rows(*_args(quant), causal=causal, sm_scale=sm_scale, p_r=224.0, bq=bq, bk=bk, w=w,
                           out_dtype=None, delta_p="block_max")
    ref, Pref = brute_force(Q, K, V, sm_scale, causal)
    assert np.abs(out - ref).max() <= 1e-12 * np.abs(ref).max()
    # the regime must exercise block maxima below one, or a dropped factor b would go unnoticed
    x = (Q @ K.T) * sm_scale * LOG2E
    if causal:
        x = np.where(np.arange(N)[None, :] <= np.arange(N)[:, None], x, -np.inf)
    below_one = 0
    for i in range(0, N, bq):
        run = np.full(min(bq, N - i), -np.inf)
        for t in range(0, N, w):
            blk = x[i:i + bq, t:t + w]
            run = np.maximum(run, blk.max(axis=1))
            with np.errstate(invalid="ignore"):
                b = np.nanmax(np.where(np.isinf(blk), np.nan, np.exp2(blk - run[:, None]))) if np.isfinite(blk).any() else 0
            below_one += 0 < b < 1
    if bq <= 4:
        assert below_one > 0


def _direct_two_steps(quant, sm_scale, p_r, w):
    """Non-causal, N <= 2w, one Q block, every row's maximum in the first step: then m never changes after step
    one, P~ = 2^(x - rowmax x) throughout, the first block's maximum is 1 and the second's is
    b = max over ALL rows and the keys of step two of P~:
        O = (sum_{n<w} q(P~ P_r) V^ + b sum_{n>=w} q(P~ P_r / b) V^) delta_V / (P_r sum P~),   q = torch's FP8 cast."""
    Qc, Kc = quant["q_codes"].astype(np.int64), quant["k_codes"].astype(np.int64)
    Nk = Kc.shape[0]
    scale = quant["q_scale"].astype(np.float64)[0] * quant["k_scale"].astype(np.float64)[np.arange(Nk) // 64][None, :]
    x = (Qc @ Kc.T) * scale * sm_scale * LOG2E
    assert (x[:, :w].max(axis=1) >= x[:, w:].max(axis=1)).all(), "construction: row maxima must lie in step one"
    Pt = np.exp2(x - x.max(axis=1, keepdims=True))

    def q(a):
        return torch.from_numpy(a.astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()

    Vh = torch.from_numpy(quant["v_codes"]).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    b = Pt[:, w:].max()
    b_rows = Pt[:, w:].max(axis=1, keepdims=True)          # the WRONG extent, for the sensitivity check
    num = q(Pt[:, :w] * p_r) @ Vh[:w] + b * (q(Pt[:, w:] * p_r / b) @ Vh[w:])
    num_rows = q(Pt[:, :w] * p_r) @ Vh[:w] + (b_rows * q(Pt[:, w:] * p_r / b_rows)) @ Vh[w:]
    den = p_r * Pt.sum(axis=1, keepdims=True)
    dv = quant["v_scale"].astype(np.float64)[None, :]
    return num * dv / den, num_rows * dv / den, b


@pytest.mark.parametrize("cfg_idx,seed", [(1, 3), (3, 4), (5, 5)])
def test_two_steps_match_the_direct_formula(cfg_idx, seed):
    base = wl.CONFIGS[cfg_idx - 1]
    Nq, Nk, w = 6, 48, 32
    mk = lambda n: wl.Workload("bm", base.index, 1, 1, n, base.d, False, base.dtype, base.q_dist, base.k_outlier_channels)
    q = wl.as_f32(wl.generate(mk(Nq), seed=seed)[0][0, 0])
    _, k, v = (wl.as_f32(t[0, 0]) for t in wl.generate(mk(Nk), seed=seed + 100))
    quant = oracle.quantize_head(q[:1].repeat(Nk, axis=0), k, v)          # K, V side (one K block, one V scale set)
    quant["q_codes"], quant["q_scale"] = oracle.quant_int8(q, None, 128)  # the six query rows: one Q block
    # reorder the keys (inside their single K block nothing else changes) so that every row's best key comes first
    S = quant["q_codes"].astype(np.int64) @ quant["k_codes"].astype(np.int64).T
    best = list(dict.fromkeys(S.argmax(axis=1).tolist()))
    order = np.array(best + [n for n in range(Nk) if n not in best])
    quant["k_codes"], quant["v_codes"] = quant["k_codes"][order], quant["v_codes"][order]
    sm = base.sm_scale
    out = oracle.attn_rows(*_args(quant), causal=False, sm_scale=sm, w=w, out_dtype=None, delta_p="block_max")
    ref, ref_rows, b = _direct_two_steps(quant, sm, 224.0, w)
    assert 0 < b < 1
    close = np.isclose(out, ref, rtol=1e-9, atol=1e-12)
    assert close.mean() > 0.97 and wl.rel_l1(ref, out) < 2e-4
    # the extent matters on this data: a per-row maximum gives visibly different codes
    assert wl.rel_l1(ref, ref_rows) > 20 * wl.rel_l1(ref, out) + 1e-6
    # and so does the mode: the static scale rounds the second step differently
    static = oracle.attn_rows(*_args(quant), causal=False, sm_scale=sm, w=w, out_dtype=None)
    assert wl.rel_l1(ref, static) > 20 * wl.rel_l1(ref, out) + 1e-6


@pytest.mark.parametrize("causal", [False, True])
def test_identical_keys_make_both_modes_equal(causal):
    """All keys equal: K' = 0, every P~ is 1, every block maximum is 1 -> block_max is the static scale."""
    base = wl.CONFIGS[0]
    cfg = wl.Workload("eq", base.index, 1, 1, 300, 128, causal, base.dtype)
    q, k, v = (wl.as_f32(t[0, 0]).copy() for t in wl.generate(cfg, seed=9))
    k[:] = k[:1]
    quant = oracle.quantize_head(q, k, v)
    a = oracle.attn_rows(*_args(quant), causal=causal, sm_scale=base.sm_scale, out_dtype=None, delta_p="block_max")
    b = oracle.attn_rows(*_args(quant), causal=causal, sm_scale=base.sm_scale, out_dtype=None)
    assert np.array_equal(a, b)


def test_rows_of_a_block_are_returned_from_whole_blocks():
    """The block maximum couples the rows of a Q block: asking for a few rows must evaluate their whole blocks."""
    base = wl.CONFIGS[2]
    cfg = wl.Workload("rows", base.index, 1, 1, 200, 64, True, base.dtype)
    q, k, v = (wl.as_f32(t[0, 0]) for t in wl.generate(cfg, seed=10))
    quant = oracle.quantize_head(q, k, v, bq=16, bk=8)
    kw = dict(causal=True, sm_scale=base.sm_scale, bq=16, bk=8, w=16, out_dtype="bf16", delta_p="block_max")
    full = oracle.attn_rows(*_args(quant), **kw)
    part = oracle.attn_rows(*_args(quant), row0=37, row1=101, **kw)
    assert np.array_equal(full[37:101], part)
