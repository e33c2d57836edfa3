"""The parity gate itself (tests/parity_gate.py), on the CPU: outputs that differ from the oracle's the way a
correct GPU result does must pass, and planted mistakes that the two norms of the benchmark definition do
not see -- one wrong row in a long head, one key missing from one row -- must fail.  The mistakes are
planted into copies of the oracle's own output."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from parity_gate import COS_MIN, REL_L1_MAX, parity_failures, parity_metrics, ulp16


def _head(cfg_idx, N, d, causal, seed):
    base = wl.CONFIGS[cfg_idx - 1]
    cfg = wl.Workload("gate", base.index, 1, 1, N, d, causal, base.dtype, base.q_dist, base.k_outlier_channels)
    q, k, v = (wl.as_f32(t[0, 0]) for t in wl.generate(cfg, seed=seed))
    quant = oracle.quantize_head(q, k, v)
    sm = np.float32(1.0 / np.sqrt(d))
    ref, _ = oracle.sage_attention_head(q, k, v, causal=causal, sm_scale=sm, out_dtype=base.dtype, quant=quant)
    return ref, quant, sm, base.dtype


def _one_ulp_noise(ref, dtype, frac, seed):
    """A copy of `ref` in which a fraction `frac` of the elements moved by one unit in the last place: what the
    final 16-bit rounding of a correct FP32 result does against the oracle's double."""
    rng = np.random.default_rng(seed)
    out = ref.copy()
    hit = rng.random(ref.shape) < frac
    out[hit] += np.where(rng.random(int(hit.sum())) < 0.5, -1.0, 1.0) * ulp16(ref[hit], dtype)
    return out


@pytest.mark.parametrize("dtype,tdtype", [("fp16", torch.float16), ("bf16", torch.bfloat16)])
def test_ulp16_is_the_spacing_of_the_16_bit_type(dtype, tdtype):
    x = torch.tensor([1.0, 1.5, 0.75, 3.0, 100.0, 1e-3, 6e-5, 2.0 ** -14, 2.0 ** -15, 65504.0 if dtype == "fp16" else 3e38])
    x16 = x.to(tdtype)
    bits = x16.view(torch.int16)
    nxt = (bits + 1).view(tdtype).double().numpy()
    cur = x16.double().numpy()
    ok = np.isfinite(nxt)
    assert np.array_equal(ulp16(cur, dtype)[ok], (nxt - cur)[ok])


def test_identical_and_rounding_noise_pass():
    ref, _, _, dtype = _head(3, 1000, 64, False, 11)
    assert parity_failures(parity_metrics(ref, ref, dtype)) == []
    noisy = _one_ulp_noise(ref, dtype, 0.05, 1)           # far more rounding flips than a GPU run shows
    m = parity_metrics(ref, noisy, dtype)
    assert m["beyond_count"] == 0 and parity_failures(m) == []


def test_one_wrong_row_in_a_long_head_fails_only_the_row_bound():
    ref, _, _, dtype = _head(3, 8192, 64, False, 12)
    bad = _one_ulp_noise(ref, dtype, 0.01, 2)
    bad[1234] = ref[77]                                   # a row written from the wrong place
    m = parity_metrics(ref, bad, dtype)
    # the norms of the benchmark definition do not see it ...
    assert m["cos"] >= COS_MIN and m["rel_l1"] <= REL_L1_MAX
    # ... the gate does, and names the row
    fails = parity_failures(m)
    assert fails and m["row_argmax"] == 1234 and any(f.startswith("row 1234") for f in fails), fails


def test_a_row_of_zeros_and_a_nan_fail():
    ref, _, _, dtype = _head(1, 512, 128, False, 13)
    z = ref.copy()
    z[300] = 0.0                                          # a row that was never accumulated
    assert parity_failures(parity_metrics(ref, z, dtype))
    n = ref.copy()
    n[5, 7] = np.nan                                      # an element that was never written
    assert "non-finite output" in parity_failures(parity_metrics(ref, n, dtype))


@pytest.mark.parametrize("cfg_idx,N,d,row", [(2, 4096, 128, 40), (3, 2000, 64, 100)])
def test_one_key_missing_from_one_causal_row_fails(cfg_idx, N, d, row):
    """Causal: a kernel that drops a row's last visible key (an off-by-one in the diagonal mask).  Planted into
    ONE early row of a long head: every other row stays exact and the norms over the head move by about 1e-5."""
    ref, quant, sm, dtype = _head(cfg_idx, N, d, True, 14)
    # row `row` without key `row`: that query against the first `row` keys, unmasked
    dropped = oracle.attn_rows(quant["q_codes"], quant["k_codes"][:row], quant["v_codes"][:row], quant["q_scale"],
                               quant["k_scale"][:(row + 63) // 64], quant["v_scale"], causal=False, sm_scale=sm,
                               row0=row, row1=row + 1, out_dtype=dtype)
    bad = ref.copy()
    bad[row] = dropped[0]
    m = parity_metrics(ref, bad, dtype)
    assert m["cos"] >= COS_MIN and m["rel_l1"] <= REL_L1_MAX      # invisible to the norms
    fails = parity_failures(m)
    assert fails and m["row_argmax"] == row, (fails, m)


def test_a_tail_key_missing_from_every_row_fails():
    """Non-causal, N not a multiple of the key step: a kernel that masks one key too many in the ragged last
    step loses key N-1 for every row."""
    ref, quant, sm, dtype = _head(3, 1000, 64, False, 16)
    N = 1000
    bad = oracle.attn_rows(quant["q_codes"], quant["k_codes"][:-1], quant["v_codes"][:-1], quant["q_scale"],
                           quant["k_scale"][:(N - 1 + 63) // 64], quant["v_scale"], causal=False, sm_scale=sm,
                           out_dtype=dtype)
    assert parity_failures(parity_metrics(ref, bad, dtype))


def test_a_few_fp8_flips_pass():
    """What a correct GPU result does differ by: single weights of single rows moved by one FP8 step."""
    ref, quant, sm, dtype = _head(2, 1024, 128, False, 15)
    # re-run three rows with one P^ decision forced the other way by nudging sm_scale by one part in 10^6:
    # the exponent moves by about 1e-5, the flips this causes are the flips an FP32 evaluation causes
    rows = oracle.attn_rows(quant["q_codes"], quant["k_codes"], quant["v_codes"], quant["q_scale"], quant["k_scale"],
                            quant["v_scale"], causal=False, sm_scale=float(sm) * (1.0 + 1e-6), out_dtype=dtype)
    m = parity_metrics(ref, rows, dtype)
    assert parity_failures(m) == [], m
    assert m["rel_l1"] < 2e-4


@pytest.mark.parametrize("cfg_idx", [2, 3])
def test_truncation_instead_of_rounding_fails(cfg_idx):
    """An epilogue that truncates to the 16-bit type instead of rounding to nearest moves about half of the
    elements by exactly one unit in the last place: invisible to the norms and to `beyond`, caught by `differ`."""
    ref, _, _, dtype = _head(cfg_idx, 1024, 64, False, 17)
    rng = np.random.default_rng(3)
    bad = ref.copy()
    hit = rng.random(ref.shape) < 0.5
    bad[hit] -= np.sign(ref[hit]) * ulp16(ref[hit] * (1 - 1e-9), dtype)
    m = parity_metrics(ref, bad, dtype)
    assert m["beyond_count"] == 0 and m["row_l1"] < 0.01
    fails = parity_failures(m)
    assert len(fails) >= 1 and any("differ" in f for f in fails), (fails, m)
