"""CPU oracle of the SageAttention2++ "8+8" forward pass -- TEST INFRASTRUCTURE.

A thin numpy/ctypes front for ``sage_oracle.c`` (plain C, double precision).
Only the test-suite, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the GPU library never does, and this
package imports nothing of the GPU library.  The passages of the paper each
routine follows are cited in the C source.

The 8+8 variant (INT8 Q.K^T) is the library's main path; the 4+8 variant (INT4 Q.K^T with smoothing of Q and
the score correction it needs) has its routines in a section of its own.

Parity status of the pins (see tests/test_oracle_*.py): every routine here is
pinned by brute force, closed forms or an independent library rounding; the
only figure with no pin is the accuracy *relative to full-precision attention*
on synthetic data ("parity unpinned": the paper's Table 2 was measured on real
model activations that are not available; it serves as a plausibility band).

All tensors of one head are C-contiguous ``[N, d]`` numpy arrays.  Inputs are
``float32`` arrays holding values exactly representable in the 16-bit input
type (the caller converts).
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

# Defaults of the method: Section 3.2 selects P_r = 224 and V_r = 4.5.  Block
# sizes are this build's reading of "per-block" in Section 2.1.
P_R = 224.0
V_R = 4.5
BQ = 128
BK = 64
W = 128

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        lib = ctypes.CDLL(path)
        c_f, c_d, c_i = ctypes.c_float, ctypes.c_double, ctypes.c_int
        vp = ctypes.c_void_p
        lib.sage_oracle_e4m3_decode.restype = c_d
        lib.sage_oracle_e4m3_decode.argtypes = [ctypes.c_uint8]
        lib.sage_oracle_e4m3_encode.restype = ctypes.c_uint8
        lib.sage_oracle_e4m3_encode.argtypes = [c_d]
        lib.sage_oracle_round16.restype = c_d
        lib.sage_oracle_round16.argtypes = [c_d, c_i]
        lib.sage_oracle_k_mean.restype = None
        lib.sage_oracle_k_mean.argtypes = [vp, c_i, c_i, vp]
        lib.sage_oracle_quant_int8.restype = None
        lib.sage_oracle_quant_int8.argtypes = [vp, vp, c_i, c_i, c_i, vp, vp]
        lib.sage_oracle_quant_v.restype = None
        lib.sage_oracle_quant_v.argtypes = [vp, c_i, c_i, c_f, vp, vp]
        lib.sage_oracle_attn_rows.restype = None
        lib.sage_oracle_attn_rows.argtypes = [vp, vp, vp, vp, vp, vp, c_i, c_i, c_i, c_i, c_d, c_d,
                                              c_i, c_i, c_i, c_i, c_i, c_i, vp, vp, vp]
        lib.sage_oracle_block_mean.restype = None
        lib.sage_oracle_block_mean.argtypes = [vp, c_i, c_i, c_i, vp]
        lib.sage_oracle_smooth.restype = None
        lib.sage_oracle_smooth.argtypes = [vp, vp, c_i, c_i, c_i, c_i, vp]
        lib.sage_oracle_quant_int.restype = None
        lib.sage_oracle_quant_int.argtypes = [vp, vp, c_i, c_i, c_i, c_i, c_i, vp, vp]
        lib.sage_oracle_delta_s.restype = None
        lib.sage_oracle_delta_s.argtypes = [vp, vp, c_i, c_i, c_i, vp]
        lib.sage_oracle_attn_rows_split.restype = None
        lib.sage_oracle_attn_rows_split.argtypes = [vp, vp, vp, vp, vp, vp, c_i, c_i, c_i, c_i, c_d, c_d,
                                                    c_i, c_i, c_i, c_i, c_i, c_i, c_i, vp]
        lib.sage_oracle_attn_rows_blockmax.restype = None
        lib.sage_oracle_attn_rows_blockmax.argtypes = [vp, vp, vp, vp, vp, vp, c_i, c_i, c_i, c_i, c_d, c_d,
                                                       c_i, c_i, c_i, c_i, c_i, c_i, vp]
        lib.sage_oracle_attn_rows_fp.restype = None
        lib.sage_oracle_attn_rows_fp.argtypes = [vp, vp, vp, c_i, c_i, c_i, c_i, c_d, c_i, c_i, c_i, vp, vp]
        lib.sage_oracle_num_threads.restype = c_i
        lib.sage_oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().sage_oracle_num_threads())


# --------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------
def e4m3_decode(codes) -> np.ndarray:
    lib = _load()
    table = np.array([lib.sage_oracle_e4m3_decode(i) for i in range(256)], dtype=np.float64)
    return table[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(x) -> np.ndarray:
    lib = _load()
    x = np.asarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint8)
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = lib.sage_oracle_e4m3_encode(float(flat_in[i]))
    return out


def round16(x, dtype: str) -> np.ndarray:
    lib = _load()
    code = {"fp16": 0, "bf16": 1}[dtype]
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    fi, fo = x.reshape(-1), out.reshape(-1)
    for i in range(fi.size):
        fo[i] = lib.sage_oracle_round16(float(fi[i]), code)
    return out


# --------------------------------------------------------------------------
# quantisation stage (one head)
# --------------------------------------------------------------------------
def k_mean(K: np.ndarray) -> np.ndarray:
    K = _c(K, np.float32)
    N, d = K.shape
    mu = np.empty(d, dtype=np.float32)
    _load().sage_oracle_k_mean(_p(K), N, d, _p(mu))
    return mu


def quant_int8(X: np.ndarray, mu, block: int):
    """Per-block INT8 codes [N, d] and scales [ceil(N/block)] of X - mu."""
    X = _c(X, np.float32)
    N, d = X.shape
    nb = (N + block - 1) // block
    codes = np.empty((N, d), dtype=np.int8)
    delta = np.empty(nb, dtype=np.float32)
    mu_p = None
    if mu is not None:
        mu = _c(mu, np.float32)
        assert mu.shape == (d,)
        mu_p = _p(mu)
    _load().sage_oracle_quant_int8(_p(X), mu_p, N, d, block, _p(codes), _p(delta))
    return codes, delta


def quant_v(V: np.ndarray, v_r: float = V_R):
    """Per-channel FP8-E4M3 codes [N, d] (token-major) and scales [d]."""
    V = _c(V, np.float32)
    N, d = V.shape
    codes = np.empty((N, d), dtype=np.uint8)
    delta = np.empty(d, dtype=np.float32)
    _load().sage_oracle_quant_v(_p(V), N, d, float(v_r), _p(codes), _p(delta))
    return codes, delta


# --------------------------------------------------------------------------
# 4+8 variant: smoothing of Q, INT4 codes, the score correction (one head)
# --------------------------------------------------------------------------
QMAX4 = 7      # INT4 codes lie in [-7, 7]


def block_mean(Q: np.ndarray, block: int = BQ) -> np.ndarray:
    """Per-block channel means of Q: [ceil(N/block), d] float32."""
    Q = _c(Q, np.float32)
    N, d = Q.shape
    qbar = np.empty(((N + block - 1) // block, d), dtype=np.float32)
    _load().sage_oracle_block_mean(_p(Q), N, d, block, _p(qbar))
    return qbar


def smooth(X: np.ndarray, mu: np.ndarray, block: int = BQ) -> np.ndarray:
    """X - mu in binary32; mu is [d] (one vector) or [ceil(N/block), d] (one per block)."""
    X, mu = _c(X, np.float32), _c(mu, np.float32)
    N, d = X.shape
    per_block = mu.ndim == 2
    assert mu.shape == (((N + block - 1) // block, d) if per_block else (d,))
    out = np.empty_like(X)
    _load().sage_oracle_smooth(_p(X), _p(mu), int(per_block), N, d, block, _p(out))
    return out


def quant_int(X: np.ndarray, mu, block: int, qmax: int):
    """Per-block integer codes in [-qmax, qmax] (one per byte) and scales of X - mu; mu as in smooth() or None."""
    X = _c(X, np.float32)
    N, d = X.shape
    nb = (N + block - 1) // block
    codes = np.empty((N, d), dtype=np.int8)
    delta = np.empty(nb, dtype=np.float32)
    mu_p, per_block = None, 0
    if mu is not None:
        mu = _c(mu, np.float32)
        per_block = int(mu.ndim == 2)
        assert mu.shape == ((nb, d) if per_block else (d,))
        mu_p = _p(mu)
    _load().sage_oracle_quant_int(_p(X), mu_p, per_block, N, d, block, int(qmax), _p(codes), _p(delta))
    return codes, delta


def delta_s(qbar: np.ndarray, k_smoothed: np.ndarray) -> np.ndarray:
    """dS[i, n] = qbar[i] . K'[n] in double: [nQ, Nk]."""
    qbar, Kp = _c(qbar, np.float32), _c(k_smoothed, np.float32)
    nQ, d = qbar.shape
    N = Kp.shape[0]
    assert Kp.shape == (N, d)
    dS = np.empty((nQ, N), dtype=np.float64)
    _load().sage_oracle_delta_s(_p(qbar), _p(Kp), nQ, N, d, _p(dS))
    return dS


def quantize_head_4bit(q, k, v, *, v_r: float = V_R, bq: int = BQ, bk: int = BK):
    """Quantisation stage of the 4+8 variant for one head (q [Nq,d]; k, v [Nk,d]): K smoothed by its channel
    mean and Q by its block means, both to INT4 codes; V to FP8 as in 8+8; plus the score correction dS."""
    mu = k_mean(k)
    qbar = block_mean(q, bq)
    q_codes, q_scale = quant_int(q, qbar, bq, QMAX4)
    k_codes, k_scale = quant_int(k, mu, bk, QMAX4)
    v_codes, v_scale = quant_v(v, v_r)
    return dict(k_mean=mu, q_mean=qbar, q_codes=q_codes, q_scale=q_scale, k_codes=k_codes, k_scale=k_scale,
                v_codes=v_codes, v_scale=v_scale, dS=delta_s(qbar, smooth(k, mu)))


def sage_attention_head_4bit(q, k, v, *, causal: bool, sm_scale: float, out_dtype: str, p_r: float = P_R,
                             v_r: float = V_R, bq: int = BQ, bk: int = BK, w: int = W, row0: int = 0, row1=None,
                             quant=None):
    """Whole 4+8 path for one head; returns (output rows as float64, quantised operands)."""
    if quant is None:
        quant = quantize_head_4bit(q, k, v, v_r=v_r, bq=bq, bk=bk)
    out = attn_rows(quant["q_codes"], quant["k_codes"], quant["v_codes"], quant["q_scale"], quant["k_scale"],
                    quant["v_scale"], causal=causal, sm_scale=sm_scale, p_r=p_r, bq=bq, bk=bk, w=w, row0=row0,
                    row1=row1, out_dtype=out_dtype, dS=quant["dS"])
    return out, quant


# --------------------------------------------------------------------------
# attention stage (one head)
# --------------------------------------------------------------------------
def attn_rows(Qc, Kc, Vc, dq, dk, dv, *, causal: bool, sm_scale: float, p_r: float = P_R,
              bq: int = BQ, bk: int = BK, w: int = W, row0: int = 0, row1=None,
              out_dtype="bf16", want_p: bool = False, delta_p: str = "static", dS=None, split_keys=None):
    """Quantised attention of query rows [row0, row1): Q^ is [Nq, d], K^ and V^ are [Nk, d].

    split_keys (a multiple of w, or None): evaluate key ranges of that many keys independently and combine
    them (the library's decode path; see sage_oracle_attn_rows_split).

    delta_p = "static" (the method as built: delta_P = 1/P_r) or "block_max" (Section 3.1 Eq. 2 read literally:
    delta_P = max(P~)/P_r per (Q block x key step); a study mode, CPU only).
    dS: the score correction of the 4+8 variant, [ceil(Nq/bq), Nk] float64 (see delta_s), or None."""
    Qc, Kc = _c(Qc, np.int8), _c(Kc, np.int8)
    Vc = _c(Vc, np.uint8)
    dq, dk, dv = _c(dq, np.float32), _c(dk, np.float32), _c(dv, np.float32)
    Nq, d = Qc.shape
    Nk = Kc.shape[0]
    assert Kc.shape == (Nk, d) and Vc.shape == (Nk, d) and dv.shape == (d,)
    assert dq.shape == ((Nq + bq - 1) // bq,) and dk.shape == ((Nk + bk - 1) // bk,)
    assert w % bk == 0 or bk % w == 0
    assert not causal or Nk >= Nq, "the end-aligned causal mask needs Nk >= Nq"
    row1 = Nq if row1 is None else row1
    assert 0 <= row0 <= row1 <= Nq
    code = {"fp16": 0, "bf16": 1, None: -1}[out_dtype]
    out = np.empty((row1 - row0, d), dtype=np.float64)
    if dS is not None:
        dS = _c(dS, np.float64)
        assert dS.shape == ((Nq + bq - 1) // bq, Nk) and delta_p == "static"
    if split_keys is not None:
        assert delta_p == "static" and dS is None and not want_p and split_keys >= w and split_keys % w == 0
        _load().sage_oracle_attn_rows_split(_p(Qc), _p(Kc), _p(Vc), _p(dq), _p(dk), _p(dv), Nq, Nk, d, int(causal),
                                            float(sm_scale), float(p_r), bq, bk, w, int(split_keys), row0, row1, code,
                                            _p(out))
        return out
    if delta_p == "block_max":
        assert not want_p
        _load().sage_oracle_attn_rows_blockmax(_p(Qc), _p(Kc), _p(Vc), _p(dq), _p(dk), _p(dv), Nq, Nk, d, int(causal),
                                               float(sm_scale), float(p_r), bq, bk, w, row0, row1, code, _p(out))
        return out
    assert delta_p == "static", delta_p
    P = np.empty((row1 - row0, Nk), dtype=np.float64) if want_p else None
    _load().sage_oracle_attn_rows(_p(Qc), _p(Kc), _p(Vc), _p(dq), _p(dk), _p(dv), Nq, Nk, d, int(causal),
                                  float(sm_scale), float(p_r), bq, bk, w, row0, row1, code,
                                  _p(out), _p(P) if want_p else None, _p(dS) if dS is not None else None)
    return (out, P) if want_p else out


def attn_rows_fp(Q, K, V, *, causal: bool, sm_scale: float, w: int = W, row0: int = 0, row1=None,
                 want_p: bool = False):
    """Block-wise online softmax on unquantised double operands (quantisers off); Q [Nq,d], K,V [Nk,d]."""
    Q, K, V = _c(Q, np.float64), _c(K, np.float64), _c(V, np.float64)
    Nq, d = Q.shape
    Nk = K.shape[0]
    assert K.shape == (Nk, d) and V.shape == (Nk, d)
    assert not causal or Nk >= Nq
    row1 = Nq if row1 is None else row1
    out = np.empty((row1 - row0, d), dtype=np.float64)
    P = np.empty((row1 - row0, Nk), dtype=np.float64) if want_p else None
    _load().sage_oracle_attn_rows_fp(_p(Q), _p(K), _p(V), Nq, Nk, d, int(causal), float(sm_scale), w,
                                     row0, row1, _p(out), _p(P) if want_p else None)
    return (out, P) if want_p else out


def quantize_head(q, k, v, *, v_r: float = V_R, bq: int = BQ, bk: int = BK):
    """Quantisation stage of one head: smoothing statistic, INT8 Q/K, FP8 V."""
    mu = k_mean(k)
    q_codes, q_scale = quant_int8(q, None, bq)
    k_codes, k_scale = quant_int8(k, mu, bk)
    v_codes, v_scale = quant_v(v, v_r)
    return dict(k_mean=mu, q_codes=q_codes, q_scale=q_scale, k_codes=k_codes, k_scale=k_scale,
                v_codes=v_codes, v_scale=v_scale)


def sage_attention_head(q, k, v, *, causal: bool, sm_scale: float, out_dtype: str,
                        p_r: float = P_R, v_r: float = V_R, bq: int = BQ, bk: int = BK, w: int = W,
                        row0: int = 0, row1=None, quant=None, delta_p: str = "static"):
    """Whole path for one head; returns (output rows as float64, quantised operands)."""
    if quant is None:
        quant = quantize_head(q, k, v, v_r=v_r, bq=bq, bk=bk)
    out = attn_rows(quant["q_codes"], quant["k_codes"], quant["v_codes"], quant["q_scale"],
                    quant["k_scale"], quant["v_scale"], causal=causal, sm_scale=sm_scale, p_r=p_r,
                    bq=bq, bk=bk, w=w, row0=row0, row1=row1, out_dtype=out_dtype, delta_p=delta_p)
    return out, quant


def sage_attention(q, k, v, *, causal: bool, sm_scale: float, out_dtype: str, **kw):
    """Whole path for q [B, Hq, Nq, d] and k, v [B, Hkv, Nk, d] (small sizes only).

    Hq may be a multiple of Hkv (grouped-query attention: query head h uses K/V head h // (Hq/Hkv),
    quantised once per K/V head); Nq may differ from Nk (causal: end-aligned)."""
    B, Hq, Nq, d = q.shape
    Hkv = k.shape[1]
    assert Hq % Hkv == 0 and v.shape == k.shape
    group = Hq // Hkv
    out = np.empty((B, Hq, Nq, d), dtype=np.float64)
    for b in range(B):
        for hk in range(Hkv):
            kv = dict(k_mean=k_mean(k[b, hk]))
            kv["k_codes"], kv["k_scale"] = quant_int8(k[b, hk], kv["k_mean"], kw.get("bk", BK))
            kv["v_codes"], kv["v_scale"] = quant_v(v[b, hk], kw.get("v_r", V_R))
            for h in range(hk * group, (hk + 1) * group):
                quant = dict(kv)
                quant["q_codes"], quant["q_scale"] = quant_int8(q[b, h], None, kw.get("bq", BQ))
                out[b, h], _ = sage_attention_head(q[b, h], k[b, hk], v[b, hk], causal=causal, sm_scale=sm_scale,
                                                   out_dtype=out_dtype, quant=quant, **kw)
    return out
