"""The C-ABI library loads on a machine without a GPU and exports every symbol the
header declares; argument checks return error codes before any GPU call."""
import ctypes
import os
import re

import pytest

import paper_2505_21136_amd as sage

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sage_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree():
    names = _declared_functions()
    assert sorted(sage.EXPORTS) == names
    L = sage.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_params_and_sizes():
    p = sage.get_params()
    assert (p["bq"], p["bk"], p["w"], p["v_tile"]) == (128, 64, 128, 128)
    assert p["p_r"] == 224.0 and p["v_r"] == 4.5          # paper Sec. 3.2
    assert p["w"] % p["bk"] == 0 and p["bq"] % 16 == 0
    assert sage.v_fp8_bytes(1, 48, 17776, 64) == 48 * 139 * 64 * 128
    assert sage.v_fp8_bytes(1, 1, 1, 128) == 128 * 128
    for shape in ((1, 2, 1024, 128), (1, 48, 17776, 64), (1, 1, 1, 64)):
        qb, wb = sage.quant_workspace_bytes(*shape), sage.workspace_bytes(*shape)
        B, H, N, d = shape
        assert qb > 0 and qb % 256 == 0 and wb % 256 == 0
        # K^ and V^ are staged; Q is quantised inside the attention kernel and needs no space
        assert wb >= qb + B * H * N * d + sage.v_fp8_bytes(*shape)
        if B * H * N * d >= 1 << 16:   # (tiny shapes: the 256-byte paddings dominate)
            assert wb < qb + 2 * B * H * N * d + sage.v_fp8_bytes(*shape)
    # unsupported shapes report size 0
    assert sage.workspace_bytes(1, 1, 16, 96) == 0 and sage.v_fp8_bytes(0, 1, 16, 64) == 0


def test_argument_checks_return_codes_without_touching_the_gpu():
    L = sage.lib()
    buf = (ctypes.c_char * 4096)()
    base = ctypes.addressof(buf)
    p = (base + 255) & ~255      # 256-byte aligned host address: never dereferenced, checks fail first
    EINVAL, EWS = -1, -2
    # head dimension
    assert L.sage_attn_fwd(p, p, p, p, 1, 1, 16, 96, 0, 0.0, None, 0, p, 1 << 20) == EINVAL
    # null pointer
    assert L.sage_attn_fwd(None, p, p, p, 1, 1, 16, 64, 0, 0.0, None, 0, p, 1 << 20) == EINVAL
    # misaligned pointer
    assert L.sage_attn_fwd(p + 2, p, p, p, 1, 1, 16, 64, 0, 0.0, None, 0, p, 1 << 20) == EINVAL
    # bad dtype, bad sizes
    assert L.sage_attn_fwd(p, p, p, p, 1, 1, 16, 64, 0, 0.0, None, 7, p, 1 << 20) == EINVAL
    assert L.sage_attn_fwd(p, p, p, p, 1, 1, 0, 64, 0, 0.0, None, 0, p, 1 << 20) == EINVAL
    # documented size limits: N <= 2^22, B*H <= 65535 (one more is refused, the limit itself passes the check)
    assert L.sage_attn_fwd(p, p, p, p, 1, 1, (1 << 22) + 1, 64, 0, 0.0, None, 0, p, 1 << 20) == EINVAL
    assert L.sage_attn_fwd(p, p, p, p, 1, 1, 1 << 22, 64, 0, 0.0, None, 0, p, 16) == EWS
    assert L.sage_attn_fwd(p, p, p, p, 256, 256, 16, 64, 0, 0.0, None, 0, p, 1 << 20) == EINVAL
    assert L.sage_attn_fwd(p, p, p, p, 5, 13107, 16, 64, 0, 0.0, None, 0, p, 16) == EWS
    # workspace too small / missing
    assert L.sage_attn_fwd(p, p, p, p, 1, 1, 16, 64, 0, 0.0, None, 0, p, 16) == EWS
    assert L.sage_attn_fwd(p, p, p, p, 1, 1, 16, 64, 0, 0.0, None, 0, None, 1 << 20) == EWS
    assert L.sage_quant_qk(p, p, p, p, p, p, p, 1, 1, 16, 64, 0, None, p, 0) == EWS
    assert L.sage_quant_v(p, p, p, 4.5, 1, 1, 16, 64, 0, None, None, 0) == EWS
    assert L.sage_quant_v(p, p, p, 0.0, 1, 1, 16, 64, 0, None, p, 1 << 20) == EINVAL
    assert L.sage_quant_v(p, p, p, 500.0, 1, 1, 16, 64, 0, None, p, 1 << 20) == EINVAL
    assert L.sage_attn_fwd_quantized(p, p, p, p, p, p, p, 1, 1, 16, 64, 0, 0.0, 1000.0, 0, None) == EINVAL
    assert L.sage_attn_fwd_quantized(p, p, None, p, p, p, p, 1, 1, 16, 64, 0, 0.0, 224.0, 0, None) == EINVAL
    # strided entry: stride rules are checked on the host before anything is enqueued
    def strided(qs=None, os_=None, B=1, H=2, N=16):
        qa = (ctypes.c_int64 * 3)(*qs) if qs else None      # (kept alive until the call returns)
        oa = (ctypes.c_int64 * 3)(*os_) if os_ else None
        return L.sage_attn_fwd_strided(p, p, p, p, B, H, H, N, N, 64, qa and ctypes.addressof(qa), None, None,
                                       oa and ctypes.addressof(oa), 0, 0.0, None, 0, p, 16)
        # (a valid call reaches the workspace check: EWS)
    assert strided() == EWS
    assert strided(qs=(2048, 64, 128)) == EWS                  # token-major input
    assert strided(qs=(0, 0, 64)) == EWS                       # broadcast input
    assert strided(qs=(2048, 1024, -64)) == EINVAL             # negative stride
    assert strided(qs=(2048, 1024, 68)) == EINVAL              # rows not 16-byte aligned
    assert strided(qs=(1 << 41, 1024, 64)) == EINVAL           # beyond the stride bound
    assert strided(os_=(2048, 64, 128)) == EWS                 # token-major output
    assert strided(os_=(2048, 1024, 32)) == EINVAL             # output rows overlap
    assert strided(os_=(2048, 0, 64)) == EINVAL                # output heads overlap
    assert strided(os_=(1024, 1024, 64), B=2) == EINVAL        # output batches overlap heads
    assert strided(os_=(0, 1024, 64), B=1) == EWS              # extent-1 dimensions do not matter
    for code in (0, -1, -2, -3, -99):
        assert isinstance(L.sage_strerror(code), bytes) and len(L.sage_strerror(code)) > 0


def test_decode_helpers_and_argument_checks_on_the_host():
    """Range length, workspace size and the argument checks of the decode entry point are host arithmetic."""
    L = sage.lib()
    for B, Hq, Hkv, Nq, Nk in ((8, 32, 8, 1, 32768), (1, 32, 8, 1, 131072), (64, 32, 8, 1, 4096), (1, 1, 1, 1, 1),
                               (2, 6, 3, 5, 129), (4096, 8, 8, 1, 1024), (1, 8, 2, 128, 32768), (2, 4, 4, 1000, 9000)):
        sk = sage.decode_split_keys(B, Hq, Hkv, Nq, Nk)
        nT = -(-Nk // 128)
        assert sk % 128 == 0 and 128 <= sk <= max(128, nT * 128)
        ranges = -(-nT // (sk // 128))
        packed = (Hq // Hkv) * Nq <= 64
        units = B * Hkv if packed else B * Hq * -(-Nq // 128)       # wavefronts (row tiles aside) or workgroups
        assert ranges >= 1 and (nT < 2 or sk >= 256)                # at least two key steps per range
        assert units * ranges <= max(units, 2 * 1024 + units)       # not many more than asked for
        for d in (64, 128):
            ws = sage.decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, d, 0)
            rows = B * Hkv * ranges * 16 * -(-(Hq // Hkv) * Nq // 16) if packed else units * ranges * 128
            assert ws % 256 == 0 and rows * (d + 2) * 4 <= ws <= rows * (d + 2) * 4 + 512
            assert sage.decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, d, sk) == ws
    assert sage.decode_workspace_bytes(1, 1, 1, 1, 1024, 128, 100) == 0      # not a multiple of 128
    assert sage.decode_workspace_bytes(1, 3, 2, 1, 1024, 128, 128) == 0      # Hq not a multiple of Hkv
    assert sage.decode_workspace_bytes(1, 1, 1, 1, 1024, 96, 128) == 0
    buf = (ctypes.c_char * 4096)()
    p = (ctypes.addressof(buf) + 255) & ~255                    # never dereferenced: the checks fail first
    EINVAL, EWS = -1, -2

    def dec(Hq=8, Hkv=2, Nq=1, Nk=1024, d=128, causal=0, split=0, ws=p, wsb=16, q=p, p_r=224.0, dt=1):
        return L.sage_attn_fwd_decode(q, p, p, p, p, p, 1, Hq, Hkv, Nq, Nk, d, causal, 0.0, p_r, split, dt, None, ws, wsb)

    assert dec() == EWS                                         # a valid call reaches the workspace check
    assert dec(Nq=16) == EWS and dec(Nq=17) == EWS              # 64 rows per K/V head packed, more on the prefill kernel
    assert dec(Hq=6, Hkv=4) == EINVAL                           # Hq not a multiple of Hkv
    assert dec(split=100) == EINVAL and dec(split=-128) == EINVAL and dec(split=256) == EWS
    assert dec(Nq=4, Nk=3, causal=1) == EINVAL                  # the end-aligned mask needs Nk >= Nq
    assert dec(d=96) == EINVAL and dec(dt=5) == EINVAL and dec(p_r=0.0) == EINVAL
    assert dec(q=None) == EINVAL and dec(q=p + 4) == EINVAL
    assert dec(ws=None, wsb=1 << 30) == EWS


def test_no_cpu_fallback():
    import torch
    q = torch.zeros((1, 1, 16, 64), dtype=torch.float16)
    with pytest.raises(sage.SageError):
        sage.sage_attn_fwd(q, q, q, causal=False)


def test_v_layout_helper_is_a_permutation():
    import torch
    T, d = 2, 64
    # fill each byte with (key mod 251) by writing through the documented formula
    buf = torch.zeros((1, 1, T, d, 128), dtype=torch.uint8)
    for tile in range(T):
        for g in range(4):
            for t in range(8):
                for i in range(4):
                    key = tile * 128 + 16 * t + 4 * g + i
                    buf[0, 0, tile, :, 64 * (t >> 2) + 16 * g + 4 * (t & 3) + i] = key % 251
    rows = sage.v_fp8_to_token_major(buf, 200)
    assert rows.shape == (1, 1, 200, d)
    want = (torch.arange(200) % 251).to(torch.uint8)[:, None].expand(200, d)
    assert torch.equal(rows[0, 0], want)


def test_product_path_and_oracle_are_independent():
    """Neither side imports, includes or names the other (only tests, smoke() and the CPU leg of bench.py use both)."""
    pkg = os.path.join(ROOT, "paper_2505_21136_amd")
    orc = os.path.join(ROOT, "oracle")

    def sources(top):
        for d, _, files in os.walk(top):
            if "_build" in d or "__pycache__" in d:
                continue
            for f in files:
                if f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                    yield os.path.join(d, f)

    for path in list(sources(pkg)) + [os.path.join(ROOT, "include", "sage.h")]:
        assert "oracle" not in open(path).read().lower(), path
    for path in sources(orc):
        text = open(path).read()
        for word in ("paper_2505_21136_amd", "libsage.so", "hip_runtime", "hipcc", "sage_internal", "sage.h"):
            assert word not in text, (path, word)


def test_missing_library_raises(monkeypatch):
    monkeypatch.setattr(sage, "_lib", None)
    monkeypatch.setattr(sage._build, "LIB", os.path.join(ROOT, "paper_2505_21136_amd", "no_such_libsage.so"))
    with pytest.raises(sage.SageError):
        sage.lib()
