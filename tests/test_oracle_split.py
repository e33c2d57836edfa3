"""Pins of the oracle's key-split mode (oracle.attn_rows(split_keys=...)): the keys are cut into ranges, every
range runs the step recurrence of Sec. 2.1 / Sec. 3.1 on its own, and the ranges are combined like partial softmax
sums.  Pinned by: the unsplit routine (one range), brute-force softmax in the regime where every quantiser is
exact (any split must then give the definition), a direct two-range formula evaluated with numpy and torch's FP8
cast, rows that see no key of a range, and a planted mistake in the combination."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from test_oracle_attention import LOG2E, _head, _lossless_problem, brute_force, brute_force_rect


def _quant(q, k, v, **kw):
    return oracle.quantize_head(q, k, v, **kw)


def _rows(quant, **kw):
    return oracle.attn_rows(quant["q_codes"], quant["k_codes"], quant["v_codes"], quant["q_scale"],
                            quant["k_scale"], quant["v_scale"], **kw)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N", [100, 300])
def test_one_range_is_the_unsplit_routine(N, causal):
    (q, k, v), base = _head(1, N)
    quant = _quant(q, k, v)
    a = _rows(quant, causal=causal, sm_scale=base.sm_scale, out_dtype=None)
    b = _rows(quant, causal=causal, sm_scale=base.sm_scale, out_dtype=None, split_keys=384)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("N,bq,bk,w,split", [(64, 16, 8, 16, 16), (64, 16, 8, 16, 32), (50, 16, 8, 16, 16),
                                             (260, 128, 64, 128, 128), (36, 8, 4, 4, 12), (36, 8, 4, 12, 24)])
@pytest.mark.parametrize("causal", [False, True])
def test_any_split_gives_the_definition_when_the_quantisers_are_lossless(N, bq, bk, w, split, causal):
    Q, K, V, _ = _lossless_problem(N, bq, bk, (0, 1), (1, 0), False, seed=7 * N + split)
    sm_scale = math.log(2.0) / 127.0
    quant = _quant(Q.astype(np.float32), K.astype(np.float32), V.astype(np.float32), v_r=4.5, bq=bq, bk=bk)
    out = _rows(quant, causal=causal, sm_scale=sm_scale, p_r=224.0, bq=bq, bk=bk, w=w, out_dtype=None,
                split_keys=split)
    ref, _ = brute_force(Q, K, V, sm_scale, causal)
    assert np.abs(out - ref).max() <= 1e-12 * np.abs(ref).max()


@pytest.mark.parametrize("Nq,Nk,bq,bk,w,split", [(1, 64, 16, 8, 16, 16), (3, 50, 16, 8, 16, 32), (4, 260, 128, 64, 128, 128),
                                                 (16, 64, 16, 8, 16, 16)])
@pytest.mark.parametrize("causal", [False, True])
def test_decode_shapes_in_the_lossless_regime(Nq, Nk, bq, bk, w, split, causal):
    """Few query rows over many keys, end-aligned causal mask: with Nq > 1 the last range holds keys that the
    first rows do not see, down to rows that see nothing of it."""
    Qfull, K, V, _ = _lossless_problem(Nk, bq, bk, (0, 1), (0,), True, seed=Nq + Nk)
    Q = Qfull[:Nq]
    sm_scale = math.log(2.0) / 127.0
    qc, qs = oracle.quant_int8(Q.astype(np.float32), None, bq)
    kc, ks = oracle.quant_int8(K.astype(np.float32), oracle.k_mean(K.astype(np.float32)), bk)
    vc, vs = oracle.quant_v(V.astype(np.float32), 4.5)
    out = oracle.attn_rows(qc, kc, vc, qs, ks, vs, causal=causal, sm_scale=sm_scale, bq=bq, bk=bk, w=w,
                           out_dtype=None, split_keys=split)
    ref, _ = brute_force_rect(Q, K, V, sm_scale, causal)
    assert np.abs(out - ref).max() <= 1e-12 * np.abs(ref).max()


def _direct_two_ranges(quant, sm_scale, p_r, cut, causal):
    """Two ranges of one step each, written out: per range P~ = 2^(x - max of the range), FP8 through torch."""
    Qc = quant["q_codes"].astype(np.int64)
    Kc = quant["k_codes"].astype(np.int64)
    N = Qc.shape[0]
    scale = (quant["q_scale"].astype(np.float64)[np.arange(N) // 128][:, None]
             * quant["k_scale"].astype(np.float64)[np.arange(N) // 64][None, :])
    x = (Qc @ Kc.T) * scale * sm_scale * LOG2E
    if causal:
        x = np.where(np.arange(N)[None, :] <= np.arange(N)[:, None], x, -np.inf)
    Vh = torch.from_numpy(quant["v_codes"]).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    num = np.zeros((N, Vh.shape[1]))
    den = np.zeros((N, 1))
    m_all = x.max(axis=1, keepdims=True)
    for lo, hi in ((0, cut), (cut, N)):
        xs = x[:, lo:hi]
        m = xs.max(axis=1, keepdims=True)
        seen = np.isfinite(m)
        m = np.where(seen, m, 0.0)
        Pt = np.where(seen, np.exp2(xs - m), 0.0)
        Ph = torch.from_numpy((Pt * p_r).astype(np.float32)).to(torch.float8_e4m3fn).to(torch.float64).numpy()
        wgt = np.where(seen, np.exp2(m - m_all), 0.0)
        num += wgt * (Ph @ Vh[lo:hi])
        den += wgt * Pt.sum(axis=1, keepdims=True)
    return num * quant["v_scale"].astype(np.float64)[None, :] / (p_r * den)


@pytest.mark.parametrize("cfg,N", [(1, 200), (3, 256), (5, 150)])
@pytest.mark.parametrize("causal", [False, True])
def test_two_ranges_match_the_direct_formula(cfg, N, causal):
    (q, k, v), base = _head(cfg, N)
    quant = _quant(q, k, v)
    out = _rows(quant, causal=causal, sm_scale=base.sm_scale, out_dtype=None, split_keys=128)
    ref = _direct_two_ranges(quant, base.sm_scale, 224.0, 128, causal)
    close = np.isclose(out, ref, rtol=1e-9, atol=1e-12)
    assert close.mean() > 0.97          # float32-vs-double products next to an FP8 tie (rare)
    assert wl.rel_l1(ref, out) < 2e-4


def test_split_changes_only_the_fp8_noise():
    """Against the unsplit result a split moves FP8 rounding decisions, nothing else: same distance from the
    full-precision answer, small distance from each other -- but not identical (it IS another mode)."""
    (q, k, v), base = _head(1, 1024)
    quant = _quant(q, k, v)
    one = _rows(quant, causal=False, sm_scale=base.sm_scale, out_dtype=None)
    four = _rows(quant, causal=False, sm_scale=base.sm_scale, out_dtype=None, split_keys=256)
    ref, _ = brute_force(q, k, v, base.sm_scale, False)
    e1, e4 = wl.rel_l1(ref, one), wl.rel_l1(ref, four)
    assert 0.67 < e1 / e4 < 1.5
    assert 0 < wl.rel_l1(one, four) < 0.06


def test_a_wrong_combination_would_be_caught():
    """Planted mistake, on the CPU: combining the ranges without their weights 2^(m_s - m) is far from the
    definition in the lossless regime where the oracle's own combination is exact."""
    N, bq, bk, w = 64, 16, 8, 16
    Q, K, V, _ = _lossless_problem(N, bq, bk, (0, 1), (0,), True, seed=5)
    sm_scale = math.log(2.0) / 127.0
    quant = _quant(Q.astype(np.float32), K.astype(np.float32), V.astype(np.float32), v_r=4.5, bq=bq, bk=bk)
    ref, _ = brute_force(Q, K, V, sm_scale, False)
    parts = []
    for lo in range(0, N, 16):   # each range alone, as a complete attention over its 16 keys
        sub = dict(quant, k_codes=quant["k_codes"][lo:lo + 16], v_codes=quant["v_codes"][lo:lo + 16],
                   k_scale=quant["k_scale"][lo // bk:(lo + 16) // bk])
        parts.append(oracle.attn_rows(quant["q_codes"], sub["k_codes"], sub["v_codes"], quant["q_scale"], sub["k_scale"],
                                      quant["v_scale"], causal=False, sm_scale=sm_scale, bq=bq, bk=bk, w=w,
                                      out_dtype=None))
    unweighted = np.mean(parts, axis=0)
    assert wl.rel_l1(ref, unweighted) > 0.05
    good = _rows(quant, causal=False, sm_scale=sm_scale, bq=bq, bk=bk, w=w, out_dtype=None, split_keys=16)
    assert np.abs(good - ref).max() <= 1e-12 * np.abs(ref).max()
