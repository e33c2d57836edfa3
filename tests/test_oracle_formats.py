"""Pins of the oracle's number formats and of the constants the paper prints.

The FP8 encoder is compared with an independent library rounding
(``torch.Tensor.to(torch.float8_e4m3fn)`` on the CPU), the 16-bit rounding with
torch's fp16/bf16 casts, and the constants with the paper's own arithmetic
(Section 3.1, Eq. 1-3; Table 2).
"""
import os

import numpy as np
import torch

import oracle


def _read_constants(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "paper_constants.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


def test_paper_constants(golden_dir):
    c = _read_constants(golden_dir)
    # Section 3.1: |32 * p * v| <= 65504  =>  P_r * V_r <= 2047
    assert c["fp16_max"] / c["mma_k"] == c["prvr_bound"] == 2047
    assert c["prvr_bound"] / 2 == c["prvr_bound_delayed"]
    assert c["p_r"] * c["v_r"] <= c["prvr_bound_delayed"]
    assert oracle.P_R == c["p_r"] and oracle.V_R == c["v_r"]
    # the FP8 format the oracle implements tops out where the paper says it does
    finite = oracle.e4m3_decode(np.arange(256, dtype=np.uint8))
    assert np.nanmax(finite) == c["e4m3_max"] and np.nanmin(finite) == -c["e4m3_max"]
    # the default ranges are themselves FP8 values (so a block/channel maximum maps onto them exactly)
    for r in (c["p_r"], c["v_r"]):
        assert oracle.e4m3_decode(oracle.e4m3_encode([r]))[0] == r


def test_table2_pairs_are_feasible(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "paper_table2_ranges.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, pr, vr, cs, l1 = line.split()
                rows.append((name, float(pr), float(vr)))
    assert len(rows) == 4
    for name, pr, vr in rows:
        if name == "SageAttn2++":
            assert pr * vr == 1008.0 <= 2047 / 2          # Eq. 3
        else:
            assert pr == vr == 448.0                       # full E4M3 range, Section 2.1
        for r in (pr, vr):
            assert oracle.e4m3_decode(oracle.e4m3_encode([r]))[0] == r


def test_e4m3_decode_matches_torch():
    codes = np.arange(256, dtype=np.uint8)
    ours = oracle.e4m3_decode(codes)
    theirs = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    nan = np.isnan(theirs)
    assert np.array_equal(nan, np.isnan(ours)) and nan.sum() == 2
    assert np.array_equal(ours[~nan], theirs[~nan])
    assert np.signbit(ours[0x80]) and ours[0x80] == 0.0
    # subnormal step 2^-9, smallest normal 2^-6
    assert ours[1] == 2.0 ** -9 and ours[8] == 2.0 ** -6 and ours[0x7e] == 448.0


def test_e4m3_encode_matches_torch_on_values_midpoints_and_neighbours():
    vals = oracle.e4m3_decode(np.arange(0, 0x7f, dtype=np.uint8))  # non-negative finite, ascending
    assert np.all(np.diff(vals) > 0)
    mids = (vals[:-1] + vals[1:]) / 2
    pts = [vals, mids]
    for p in (vals, mids):
        f = p.astype(np.float32)
        pts.append(np.nextafter(f, np.float32(np.inf)).astype(np.float64))
        pts.append(np.nextafter(f, np.float32(-np.inf)).astype(np.float64))
    rng = np.random.default_rng(1)
    pts.append(rng.uniform(0, 448, 4000))
    pts.append(np.exp2(rng.uniform(-14, 9, 4000)))
    x = np.concatenate(pts)
    x = x[(x >= 0) & (x <= 464.0)]
    x = np.concatenate([x, -x]).astype(np.float32)        # exactly representable inputs for torch
    theirs = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ours = oracle.e4m3_encode(x.astype(np.float64))
    # torch keeps the sign of zero; so do we
    assert np.array_equal(ours, theirs)
    # spot values: ties go to the even mantissa, the subnormal edge, the top of the range
    spot = {17.0: 16.0, 19.0: 20.0, 21.0: 20.0, 2.0 ** -10: 0.0, 3 * 2.0 ** -10: 2.0 ** -8,
            464.0: 448.0, 447.9: 448.0, 1e9: 448.0, -1e9: -448.0}
    for k, v in spot.items():
        assert oracle.e4m3_decode(oracle.e4m3_encode([k]))[0] == v, k


def test_e4m3_encode_is_nearest_everywhere():
    """Brute force: the chosen code is a closest representable value (never 2 steps away)."""
    vals = oracle.e4m3_decode(np.arange(0, 0x7f, dtype=np.uint8))
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.uniform(0, 448, 3000), np.exp2(rng.uniform(-12, 9, 3000))])
    x = x[x <= 448]
    got = oracle.e4m3_decode(oracle.e4m3_encode(x))
    best = np.abs(x[:, None] - vals[None, :]).min(axis=1)
    assert np.all(np.abs(got - x) <= best * (1 + 1e-15))


def test_e4m3_doubling_shifts_the_exponent():
    """P_r = 448 instead of 224 doubles the operand: codes move by one exponent step
    (+8) above the subnormal range, which is why Table 2's rows barely differ."""
    rng = np.random.default_rng(3)
    x = np.exp2(rng.uniform(-6, 7.5, 2000))
    x = x[x * 2 < 448]
    a = oracle.e4m3_encode(x).astype(int)
    b = oracle.e4m3_encode(2 * x).astype(int)
    assert np.array_equal(b, a + 8)


def test_round16_matches_torch_casts():
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.standard_normal(5000), rng.standard_normal(2000) * 1e-6,
                        rng.standard_normal(2000) * 3e4, [0.0, 1.0, -1.0, 65504.0, 65519.9, 65520.0]])
    for name, dt in (("fp16", torch.float16), ("bf16", torch.bfloat16)):
        # float32 inputs, so torch's cast is a single rounding
        xf = x.astype(np.float32)
        theirs = torch.from_numpy(xf).to(dt).to(torch.float64).numpy()
        ours = oracle.round16(xf.astype(np.float64), name)
        assert np.array_equal(ours, theirs), name
        # exact ties between neighbouring 16-bit values go to even
        base = torch.from_numpy(xf).to(dt)
        nxt = torch.nextafter(base.float(), torch.full_like(base.float(), float("inf"))).to(dt)
        # neighbour in the 16-bit grid: add one unit in the last place through integer views
        up = (base.view(torch.int16) + torch.where(base >= 0, 1, -1).to(torch.int16)).view(dt)
        ok = torch.isfinite(up.float()) & torch.isfinite(base.float())
        mid = ((base.double() + up.double()) / 2)[ok].numpy()
        want = torch.from_numpy(mid.astype(np.float32)).to(dt).to(torch.float64).numpy()
        assert np.array_equal(mid.astype(np.float32).astype(np.float64), mid)  # midpoints fit float32
        assert np.array_equal(oracle.round16(mid, name), want), name
        del nxt
    # direct rounding from double, not through float32: a value just above a bf16 tie
    # whose float32 rounding lands exactly on the tie must still round up
    tie = 1.0 + 2.0 ** -8                       # midway between bf16 neighbours 1 and 1 + 2^-7
    above = tie + 2.0 ** -40
    assert np.float32(above) == np.float32(tie)
    assert oracle.round16([tie], "bf16")[0] == 1.0
    assert oracle.round16([above], "bf16")[0] == 1.0 + 2.0 ** -7
