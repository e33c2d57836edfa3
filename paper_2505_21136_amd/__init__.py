"""Python binding of libsage (SageAttention2++ 8+8 forward, MI355X / gfx950).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libsage.so`` behind the C ABI declared in ``include/sage.h``.  PyTorch is used
for device memory and the current stream.  There is no CPU fallback: importing
works without a GPU (the library loads lazily), but any compute call raises if
the shared library is missing or fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

__all__ = [
    "SageError", "lib", "get_params", "v_fp8_bytes", "quant_workspace_bytes", "workspace_bytes",
    "sage_quant_qk", "sage_quant_q", "sage_quant_k", "sage_quant_v", "sage_attn_fwd_quantized",
    "sage_attn_fwd_quantized_gqa", "sage_attn_fwd_kvquantized_gqa", "sage_attn_fwd", "sage_attn_fwd_gqa",
    "sage_attn_fwd_strided", "sage_quant_kv", "sage_quant_kv_static", "workspace_bytes_gqa",
    "v_fp8_to_token_major", "diag_mfma_rate", "diag_quant_kv_path", "decode_split_keys", "decode_workspace_bytes",
    "sage_attn_fwd_decode", "EXPORTS", "sage_quant_q4", "sage_quant_kv4", "sage_delta_s",
    "sage_attn_fwd_q4", "sage_attn_fwd_4bit", "workspace_bytes_4bit", "delta_s_to_key_order",
]

SAGE_F16, SAGE_BF16 = 0, 1
EXPORTS = ["sage_get_params", "sage_strerror", "sage_v_fp8_bytes", "sage_quant_workspace_bytes",
           "sage_workspace_bytes", "sage_workspace_bytes_gqa", "sage_quant_qk", "sage_quant_q", "sage_quant_k",
           "sage_quant_v", "sage_attn_fwd_quantized", "sage_attn_fwd_quantized_gqa",
           "sage_attn_fwd_kvquantized_gqa", "sage_attn_fwd", "sage_attn_fwd_gqa", "sage_attn_fwd_strided",
           "sage_quant_kv", "sage_quant_kv_static", "sage_diag_mfma_rate", "sage_diag_quant_kv_path", "sage_decode_split_keys", "sage_decode_workspace_bytes",
           "sage_attn_fwd_decode", "sage_delta_s_bytes",
           "sage_workspace_bytes_4bit", "sage_quant_q4", "sage_quant_kv4", "sage_delta_s", "sage_attn_fwd_q4",
           "sage_attn_fwd_4bit"]


class SageError(RuntimeError):
    pass


class _Params(ctypes.Structure):
    _fields_ = [("bq", ctypes.c_int), ("bk", ctypes.c_int), ("w", ctypes.c_int), ("v_tile", ctypes.c_int),
                ("p_r", ctypes.c_float), ("v_r", ctypes.c_float)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C library (raises SageError if it has not been built)."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            raise SageError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                            "(there is no fallback path)")
        L = ctypes.CDLL(path)
        i, f, vp, sz = ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
        L.sage_get_params.restype = i
        L.sage_get_params.argtypes = [ctypes.POINTER(_Params)]
        L.sage_strerror.restype = ctypes.c_char_p
        L.sage_strerror.argtypes = [i]
        for name in ("sage_v_fp8_bytes", "sage_quant_workspace_bytes", "sage_workspace_bytes"):
            fn = getattr(L, name)
            fn.restype = sz
            fn.argtypes = [i, i, i, i]
        L.sage_workspace_bytes_gqa.restype = sz
        L.sage_workspace_bytes_gqa.argtypes = [i, i, i, i, i, i]
        L.sage_quant_q.restype = i
        L.sage_quant_q.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.sage_quant_k.restype = i
        L.sage_quant_k.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, vp, sz]
        L.sage_attn_fwd_quantized_gqa.restype = i
        L.sage_attn_fwd_quantized_gqa.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, f, i, vp]
        L.sage_attn_fwd_kvquantized_gqa.restype = i
        L.sage_attn_fwd_kvquantized_gqa.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, f, i, vp]
        L.sage_attn_fwd_gqa.restype = i
        L.sage_attn_fwd_gqa.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, f, vp, i, vp, sz]
        L.sage_attn_fwd_strided.restype = i
        L.sage_attn_fwd_strided.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp, vp, vp, vp, i, f, vp, i, vp, sz]
        L.sage_quant_kv.restype = i
        L.sage_quant_kv.argtypes = [vp, vp, vp, vp, vp, vp, vp, f, i, i, i, i, i, vp, vp, sz]
        L.sage_quant_kv_static.restype = i
        L.sage_quant_kv_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, f, i, i, i, i, i, vp]
        L.sage_diag_mfma_rate.restype = i
        L.sage_diag_mfma_rate.argtypes = [i, i, i, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.sage_decode_split_keys.restype = i
        L.sage_decode_split_keys.argtypes = [i, i, i, i, i]
        L.sage_decode_workspace_bytes.restype = sz
        L.sage_decode_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
        L.sage_attn_fwd_decode.restype = i
        L.sage_attn_fwd_decode.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, f, i, i, vp, vp, sz]
        L.sage_diag_quant_kv_path.restype = i
        L.sage_diag_quant_kv_path.argtypes = [i, ctypes.c_longlong]
        L.sage_delta_s_bytes.restype = sz
        L.sage_delta_s_bytes.argtypes = [i, i, i, i]
        L.sage_workspace_bytes_4bit.restype = sz
        L.sage_workspace_bytes_4bit.argtypes = [i, i, i, i, i, i]
        L.sage_quant_q4.restype = i
        L.sage_quant_q4.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp]
        L.sage_quant_kv4.restype = i
        L.sage_quant_kv4.argtypes = [vp, vp, vp, vp, vp, vp, vp, f, i, i, i, i, i, vp, vp, sz]
        L.sage_delta_s.restype = i
        L.sage_delta_s.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, f, i, vp]
        L.sage_attn_fwd_q4.restype = i
        L.sage_attn_fwd_q4.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, i, f, f, i, vp]
        L.sage_attn_fwd_4bit.restype = i
        L.sage_attn_fwd_4bit.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, f, vp, i, vp, sz]
        L.sage_quant_qk.restype = i
        L.sage_quant_qk.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, vp, vp, sz]
        L.sage_quant_v.restype = i
        L.sage_quant_v.argtypes = [vp, vp, vp, f, i, i, i, i, i, vp, vp, sz]
        L.sage_attn_fwd_quantized.restype = i
        L.sage_attn_fwd_quantized.argtypes = [vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i, f, f, i, vp]
        L.sage_attn_fwd.restype = i
        L.sage_attn_fwd.argtypes = [vp, vp, vp, vp, i, i, i, i, i, f, vp, i, vp, sz]
        _lib = L
    return _lib


def _check(code: int):
    if code != 0:
        raise SageError(f"libsage error {code}: {lib().sage_strerror(code).decode()}")


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return SAGE_F16
    if t.dtype == torch.bfloat16:
        return SAGE_BF16
    raise SageError(f"unsupported dtype {t.dtype}: fp16 or bf16 expected")


def _dev(*ts: torch.Tensor):
    for t in ts:
        if not t.is_cuda:
            raise SageError("libsage needs device tensors (no CPU path exists)")
        if not t.is_contiguous():
            raise SageError("tensors must be contiguous [B, H, N, d]")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def get_params() -> dict:
    p = _Params()
    _check(lib().sage_get_params(ctypes.byref(p)))
    return dict(bq=p.bq, bk=p.bk, w=p.w, v_tile=p.v_tile, p_r=p.p_r, v_r=p.v_r)


def v_fp8_bytes(B, H, N, d) -> int:
    return int(lib().sage_v_fp8_bytes(B, H, N, d))


def quant_workspace_bytes(B, H, N, d) -> int:
    return int(lib().sage_quant_workspace_bytes(B, H, N, d))


def workspace_bytes(B, H, N, d) -> int:
    return int(lib().sage_workspace_bytes(B, H, N, d))


def workspace_bytes_gqa(B, Hq, Hkv, Nq, Nk, d) -> int:
    return int(lib().sage_workspace_bytes_gqa(B, Hq, Hkv, Nq, Nk, d))


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def sage_quant_qk(q: torch.Tensor, k: torch.Tensor, workspace: torch.Tensor | None = None):
    """-> (q_i8 [B,H,N,d], k_i8 [B,H,N,d], q_scale [B,H,nQ], k_scale [B,H,nK], k_mean [B,H,d])."""
    _dev(q, k)
    B, H, N, d = q.shape
    if k.shape != q.shape or k.dtype != q.dtype:
        raise SageError("q and k must have the same shape and dtype")
    dev = q.device
    nq, nk = -(-N // 128), -(-N // 64)
    q_i8 = torch.empty((B, H, N, d), dtype=torch.int8, device=dev)
    k_i8 = torch.empty((B, H, N, d), dtype=torch.int8, device=dev)
    q_scale = torch.empty((B, H, nq), dtype=torch.float32, device=dev)
    k_scale = torch.empty((B, H, nk), dtype=torch.float32, device=dev)
    k_mean = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    need = quant_workspace_bytes(B, H, N, d)
    ws = workspace if workspace is not None else _workspace(need, dev)
    _check(lib().sage_quant_qk(q.data_ptr(), k.data_ptr(), q_i8.data_ptr(), k_i8.data_ptr(), q_scale.data_ptr(),
                               k_scale.data_ptr(), k_mean.data_ptr(), B, H, N, d, _dt(q), _stream(),
                               ws.data_ptr(), ws.numel()))
    return q_i8, k_i8, q_scale, k_scale, k_mean


def sage_quant_q(q: torch.Tensor):
    """-> (q_i8 [B,H,N,d], q_scale [B,H,ceil(N/128)])."""
    _dev(q)
    B, H, N, d = q.shape
    q_i8 = torch.empty((B, H, N, d), dtype=torch.int8, device=q.device)
    q_scale = torch.empty((B, H, -(-N // 128)), dtype=torch.float32, device=q.device)
    _check(lib().sage_quant_q(q.data_ptr(), q_i8.data_ptr(), q_scale.data_ptr(), B, H, N, d, _dt(q), _stream()))
    return q_i8, q_scale


def sage_quant_k(k: torch.Tensor, workspace: torch.Tensor | None = None):
    """-> (k_i8 [B,H,N,d], k_scale [B,H,ceil(N/64)], k_mean [B,H,d])."""
    _dev(k)
    B, H, N, d = k.shape
    dev = k.device
    k_i8 = torch.empty((B, H, N, d), dtype=torch.int8, device=dev)
    k_scale = torch.empty((B, H, -(-N // 64)), dtype=torch.float32, device=dev)
    k_mean = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    ws = workspace if workspace is not None else _workspace(quant_workspace_bytes(B, H, N, d), dev)
    _check(lib().sage_quant_k(k.data_ptr(), k_i8.data_ptr(), k_scale.data_ptr(), k_mean.data_ptr(), B, H, N, d,
                              _dt(k), _stream(), ws.data_ptr(), ws.numel()))
    return k_i8, k_scale, k_mean


def sage_quant_kv(k: torch.Tensor, v: torch.Tensor, v_r: float = 4.5, workspace: torch.Tensor | None = None):
    """K and V of one shape in one call -> (k_i8, k_scale, k_mean, v_fp8, v_scale), as sage_quant_k / sage_quant_v."""
    _dev(k, v)
    if k.shape != v.shape or k.dtype != v.dtype:
        raise SageError("k and v must share shape and dtype")
    B, H, N, d = k.shape
    dev = k.device
    k_i8 = torch.empty((B, H, N, d), dtype=torch.int8, device=dev)
    k_scale = torch.empty((B, H, -(-N // 64)), dtype=torch.float32, device=dev)
    k_mean = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    v_fp8 = torch.empty((B, H, -(-N // 128), d, 128), dtype=torch.uint8, device=dev)
    v_scale = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    ws = workspace if workspace is not None else _workspace(quant_workspace_bytes(B, H, N, d), dev)
    _check(lib().sage_quant_kv(k.data_ptr(), v.data_ptr(), k_i8.data_ptr(), k_scale.data_ptr(), k_mean.data_ptr(),
                               v_fp8.data_ptr(), v_scale.data_ptr(), float(v_r), B, H, N, d, _dt(k), _stream(),
                               ws.data_ptr(), ws.numel()))
    return k_i8, k_scale, k_mean, v_fp8, v_scale


def diag_quant_kv_path(path: int = 0, wait_ticks: int = 50_000) -> None:
    """Select the kernels of the K/V quantisers (0: by shape, 1: three launches, 2: single-read kernel) and the
    single-read kernel's wait bound; see include/sage.h.  For benchmarks and tests."""
    _check(lib().sage_diag_quant_kv_path(int(path), int(wait_ticks)))


def diag_mfma_rate(kind: int, iters: int = 4096, workgroups: int = 2048, repeats: int = 5) -> float:
    """Sustained rate (operations per second) of the matrix instructions the attention kernel uses, measured
    with HIP events around `sage_diag_mfma_rate` launches; kind as in include/sage.h.  A measurement aid."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    ops = ctypes.c_double(0.0)
    stream = torch.cuda.current_stream()

    def launch():
        _check(lib().sage_diag_mfma_rate(kind, iters, workgroups, sink.data_ptr(), ctypes.byref(ops), stream.cuda_stream))

    for _ in range(3):
        launch()
    best = float("inf")
    for _ in range(repeats):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        launch()
        b.record(stream)
        b.synchronize()
        best = min(best, a.elapsed_time(b) * 1e-3)
    return ops.value / best


def sage_quant_kv_static(k: torch.Tensor, v: torch.Tensor, v_r: float = 4.5, out=None):
    """sage_quant_kv through the entry point that uses the library's built-in scratch (no workspace, nothing
    allocated by the call itself).  `out` = (k_i8, k_scale, k_mean, v_fp8, v_scale) preallocated, or None."""
    _dev(k, v)
    if k.shape != v.shape or k.dtype != v.dtype:
        raise SageError("k and v must share shape and dtype")
    B, H, N, d = k.shape
    dev = k.device
    if out is None:
        out = (torch.empty((B, H, N, d), dtype=torch.int8, device=dev),
               torch.empty((B, H, -(-N // 64)), dtype=torch.float32, device=dev),
               torch.empty((B, H, d), dtype=torch.float32, device=dev),
               torch.empty((B, H, -(-N // 128), d, 128), dtype=torch.uint8, device=dev),
               torch.empty((B, H, d), dtype=torch.float32, device=dev))
    k_i8, k_scale, k_mean, v_fp8, v_scale = out
    _dev(*out)
    _check(lib().sage_quant_kv_static(k.data_ptr(), v.data_ptr(), k_i8.data_ptr(), k_scale.data_ptr(),
                                      k_mean.data_ptr(), v_fp8.data_ptr(), v_scale.data_ptr(), float(v_r), B, H, N, d,
                                      _dt(k), _stream()))
    return out


def sage_quant_v(v: torch.Tensor, v_r: float = 4.5, workspace: torch.Tensor | None = None):
    """-> (v_fp8 uint8 [B,H,ceil(N/128),d,128] in the library's tile layout, v_scale [B,H,d])."""
    _dev(v)
    B, H, N, d = v.shape
    dev = v.device
    nT = -(-N // 128)
    v_fp8 = torch.empty((B, H, nT, d, 128), dtype=torch.uint8, device=dev)
    v_scale = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    need = quant_workspace_bytes(B, H, N, d)
    ws = workspace if workspace is not None else _workspace(need, dev)
    _check(lib().sage_quant_v(v.data_ptr(), v_fp8.data_ptr(), v_scale.data_ptr(), float(v_r), B, H, N, d, _dt(v),
                              _stream(), ws.data_ptr(), ws.numel()))
    return v_fp8, v_scale


def sage_attn_fwd_quantized(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, *, causal: bool, sm_scale: float,
                            out_dtype: torch.dtype, p_r: float = 224.0, out: torch.Tensor | None = None):
    _dev(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale)
    B, H, N, d = q_i8.shape
    if out is None:
        out = torch.empty((B, H, N, d), dtype=out_dtype, device=q_i8.device)
    _dev(out)
    _check(lib().sage_attn_fwd_quantized(q_i8.data_ptr(), k_i8.data_ptr(), v_fp8.data_ptr(), q_scale.data_ptr(),
                                         k_scale.data_ptr(), v_scale.data_ptr(), out.data_ptr(), B, H, N, d,
                                         int(causal), float(sm_scale), float(p_r), _dt(out), _stream()))
    return out


def sage_attn_fwd_quantized_gqa(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale, *, causal: bool, sm_scale: float,
                                out_dtype: torch.dtype, p_r: float = 224.0, out: torch.Tensor | None = None):
    """q_i8 [B,Hq,Nq,d] against k_i8 [B,Hkv,Nk,d] / v_fp8 of the same K/V shape."""
    _dev(q_i8, k_i8, v_fp8, q_scale, k_scale, v_scale)
    B, Hq, Nq, d = q_i8.shape
    _, Hkv, Nk, _ = k_i8.shape
    if out is None:
        out = torch.empty((B, Hq, Nq, d), dtype=out_dtype, device=q_i8.device)
    _dev(out)
    _check(lib().sage_attn_fwd_quantized_gqa(q_i8.data_ptr(), k_i8.data_ptr(), v_fp8.data_ptr(), q_scale.data_ptr(),
                                             k_scale.data_ptr(), v_scale.data_ptr(), out.data_ptr(), B, Hq, Hkv, Nq,
                                             Nk, d, int(causal), float(sm_scale), float(p_r), _dt(out), _stream()))
    return out


def sage_attn_fwd_kvquantized_gqa(q, k_i8, v_fp8, k_scale, v_scale, *, causal: bool, sm_scale: float,
                                  p_r: float = 224.0, out: torch.Tensor | None = None):
    """Unquantised q [B,Hq,Nq,d] (quantised inside the kernel) against k_i8 [B,Hkv,Nk,d] / v_fp8."""
    _dev(q, k_i8, v_fp8, k_scale, v_scale)
    B, Hq, Nq, d = q.shape
    _, Hkv, Nk, _ = k_i8.shape
    if out is None:
        out = torch.empty_like(q)
    _dev(out)
    if out.dtype != q.dtype:
        raise SageError("out must have q's dtype")
    _check(lib().sage_attn_fwd_kvquantized_gqa(q.data_ptr(), k_i8.data_ptr(), v_fp8.data_ptr(), k_scale.data_ptr(),
                                               v_scale.data_ptr(), out.data_ptr(), B, Hq, Hkv, Nq, Nk, d, int(causal),
                                               float(sm_scale), float(p_r), _dt(q), _stream()))
    return out


def decode_split_keys(B: int, Hq: int, Hkv: int, Nq: int, Nk: int) -> int:
    """Keys per range that sage_attn_fwd_decode uses for split_keys = 0."""
    return int(lib().sage_decode_split_keys(B, Hq, Hkv, Nq, Nk))


def decode_workspace_bytes(B: int, Hq: int, Hkv: int, Nq: int, Nk: int, d: int, split_keys: int = 0) -> int:
    """Workspace of sage_attn_fwd_decode."""
    return int(lib().sage_decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, d, split_keys))


def sage_attn_fwd_decode(q, k_i8, v_fp8, k_scale, v_scale, *, causal: bool, sm_scale: float = 0.0,
                         p_r: float = 224.0, split_keys: int = 0, out: torch.Tensor | None = None,
                         workspace: torch.Tensor | None = None):
    """Few query rows over a long quantised key sequence: q [B,Hq,Nq,d] against k_i8 [B,Hkv,Nk,d] / v_fp8; the keys
    are evaluated in ranges of split_keys keys (0: the library's choice) and combined."""
    _dev(q, k_i8, v_fp8, k_scale, v_scale)
    B, Hq, Nq, d = q.shape
    _, Hkv, Nk, _ = k_i8.shape
    if out is None:
        out = torch.empty_like(q)
    _dev(out)
    if out.dtype != q.dtype:
        raise SageError("out must have q's dtype")
    need = decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, d, split_keys)
    ws = workspace if workspace is not None else _workspace(max(need, 256), q.device)
    _check(lib().sage_attn_fwd_decode(q.data_ptr(), k_i8.data_ptr(), v_fp8.data_ptr(), k_scale.data_ptr(),
                                      v_scale.data_ptr(), out.data_ptr(), B, Hq, Hkv, Nq, Nk, d, int(causal),
                                      float(sm_scale), float(p_r), int(split_keys), _dt(q), _stream(), ws.data_ptr(),
                                      ws.numel()))
    return out


def sage_attn_fwd_gqa(q, k, v, *, causal: bool, sm_scale: float = 0.0, out: torch.Tensor | None = None,
                      workspace: torch.Tensor | None = None):
    """Whole forward pass for q [B,Hq,Nq,d] and k, v [B,Hkv,Nk,d] (Hq % Hkv == 0)."""
    _dev(q, k, v)
    B, Hq, Nq, d = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[3] != d or k.dtype != q.dtype or v.dtype != q.dtype:
        raise SageError("k and v must share a shape [B,Hkv,Nk,d] and the dtype of q")
    _, Hkv, Nk, _ = k.shape
    if out is None:
        out = torch.empty_like(q)
    _dev(out)
    need = workspace_bytes_gqa(B, Hq, Hkv, Nq, Nk, d)
    ws = workspace if workspace is not None else _workspace(need, q.device)
    _check(lib().sage_attn_fwd_gqa(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, Hq, Hkv, Nq, Nk, d,
                                   int(causal), float(sm_scale), _stream(), _dt(q), ws.data_ptr(), ws.numel()))
    return out


def _bhn_strides(t: torch.Tensor, layout: str):
    """(B, H, N, d) and the ctypes {batch, head, token} element strides of a 4-D view."""
    if t.dim() != 4 or t.stride(3) != 1:
        raise SageError("strided tensors must be 4-D with a contiguous last (channel) dimension")
    if layout == "bhnd":
        (B, H, N, d), (sb, sh, sn) = t.shape, t.stride()[:3]
    elif layout == "bnhd":
        (B, N, H, d), (sb, sn, sh) = t.shape, t.stride()[:3]
    else:
        raise SageError(f"unknown layout {layout!r}: 'bhnd' or 'bnhd'")
    return (B, H, N, d), (ctypes.c_int64 * 3)(sb, sh, sn)


def sage_attn_fwd_strided(q, k, v, *, causal: bool, sm_scale: float = 0.0, layout: str = "bhnd",
                          out: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """Whole forward pass on views (no copies): `layout` names the order of the tensors' dimensions,
    'bhnd' ([B,H,N,d]) or 'bnhd' ([B,N,H,d]); any strides with a contiguous channel dimension are accepted
    (transposed views, slices of a packed QKV tensor).  `out` defaults to a new contiguous tensor of q's
    shape in the same dimension order."""
    for t in (q, k, v):
        if not t.is_cuda:
            raise SageError("libsage needs device tensors (no CPU path exists)")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise SageError("k and v must have the dtype of q")
    (B, Hq, Nq, d), qs = _bhn_strides(q, layout)
    (Bk, Hkv, Nk, dk), ks = _bhn_strides(k, layout)
    (Bv, Hv, Nv, dv), vs = _bhn_strides(v, layout)
    if (Bk, dk) != (B, d) or (Bv, Hv, Nv, dv) != (Bk, Hkv, Nk, dk):
        raise SageError("k and v must share a shape and q's batch and head dimension")
    if out is None:
        out = torch.empty(q.shape, dtype=q.dtype, device=q.device)
    if not out.is_cuda or out.dtype != q.dtype or out.shape != q.shape:
        raise SageError("out must be a device tensor of q's shape and dtype")
    _, os_ = _bhn_strides(out, layout)
    need = workspace_bytes_gqa(B, Hq, Hkv, Nq, Nk, d)
    ws = workspace if workspace is not None else _workspace(need, q.device)
    _check(lib().sage_attn_fwd_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, Hq, Hkv, Nq, Nk, d,
                                       ctypes.addressof(qs), ctypes.addressof(ks), ctypes.addressof(vs),
                                       ctypes.addressof(os_), int(causal), float(sm_scale), _stream(), _dt(q),
                                       ws.data_ptr(), ws.numel()))
    return out


def sage_attn_fwd(q, k, v, *, causal: bool, sm_scale: float = 0.0, out: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None):
    """Whole forward pass (quantisation + attention) with the default ranges."""
    _dev(q, k, v)
    B, H, N, d = q.shape
    if k.shape != q.shape or v.shape != q.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise SageError("q, k, v must have the same shape and dtype")
    if out is None:
        out = torch.empty_like(q)
    _dev(out)
    need = workspace_bytes(B, H, N, d)
    ws = workspace if workspace is not None else _workspace(need, q.device)
    _check(lib().sage_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, d, int(causal),
                               float(sm_scale), _stream(), _dt(q), ws.data_ptr(), ws.numel()))
    return out


# --------------------------------------------------------------------------
# the 4+8 variant (INT4 Q K^T with smoothing of Q and K)
# --------------------------------------------------------------------------
def workspace_bytes_4bit(B, Hq, Hkv, Nq, Nk, d) -> int:
    return int(lib().sage_workspace_bytes_4bit(B, Hq, Hkv, Nq, Nk, d))


def sage_quant_q4(q: torch.Tensor, codes: bool = True):
    """-> (q_mean [B,H,ceil(N/128),d], q_i4 [B,H,N,d] int8 in [-7,7], q_scale [B,H,ceil(N/128)]); the last two
    are None with codes=False."""
    _dev(q)
    B, H, N, d = q.shape
    nq = -(-N // 128)
    q_mean = torch.empty((B, H, nq, d), dtype=torch.float32, device=q.device)
    q_i4 = torch.empty((B, H, N, d), dtype=torch.int8, device=q.device) if codes else None
    q_scale = torch.empty((B, H, nq), dtype=torch.float32, device=q.device) if codes else None
    _check(lib().sage_quant_q4(q.data_ptr(), q_mean.data_ptr(), q_i4.data_ptr() if codes else None,
                               q_scale.data_ptr() if codes else None, B, H, N, d, _dt(q), _stream()))
    return q_mean, q_i4, q_scale


def sage_quant_kv4(k: torch.Tensor, v: torch.Tensor, v_r: float = 4.5, workspace: torch.Tensor | None = None):
    """sage_quant_kv with INT4 codes for K -> (k_i4, k_scale, k_mean, v_fp8, v_scale)."""
    _dev(k, v)
    if k.shape != v.shape or k.dtype != v.dtype:
        raise SageError("k and v must share shape and dtype")
    B, H, N, d = k.shape
    dev = k.device
    k_i4 = torch.empty((B, H, N, d), dtype=torch.int8, device=dev)
    k_scale = torch.empty((B, H, -(-N // 64)), dtype=torch.float32, device=dev)
    k_mean = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    v_fp8 = torch.empty((B, H, -(-N // 128), d, 128), dtype=torch.uint8, device=dev)
    v_scale = torch.empty((B, H, d), dtype=torch.float32, device=dev)
    ws = workspace if workspace is not None else _workspace(quant_workspace_bytes(B, H, N, d), dev)
    _check(lib().sage_quant_kv4(k.data_ptr(), v.data_ptr(), k_i4.data_ptr(), k_scale.data_ptr(), k_mean.data_ptr(),
                                v_fp8.data_ptr(), v_scale.data_ptr(), float(v_r), B, H, N, d, _dt(k), _stream(),
                                ws.data_ptr(), ws.numel()))
    return k_i4, k_scale, k_mean, v_fp8, v_scale


def sage_delta_s(k: torch.Tensor, k_mean: torch.Tensor, q_mean: torch.Tensor, Nq: int, *, causal: bool,
                 sm_scale: float = 0.0) -> torch.Tensor:
    """The score correction in exponent units -> [B,Hq,ceil(Nq/128),ceil(Nk/128),128] float32 (lane order)."""
    _dev(k, k_mean, q_mean)
    B, Hkv, Nk, d = k.shape
    Hq, nq = q_mean.shape[1], q_mean.shape[2]
    dsx = torch.empty((B, Hq, nq, -(-Nk // 128), 128), dtype=torch.float32, device=k.device)
    _check(lib().sage_delta_s(k.data_ptr(), k_mean.data_ptr(), q_mean.data_ptr(), dsx.data_ptr(), B, Hq, Hkv, Nq, Nk, d,
                              int(causal), float(sm_scale), _dt(k), _stream()))
    return dsx


def sage_attn_fwd_q4(q, q_mean, k_i4, v_fp8, k_scale, v_scale, dsx, *, causal: bool, sm_scale: float = 0.0,
                     p_r: float = 224.0, out: torch.Tensor | None = None):
    _dev(q, q_mean, k_i4, v_fp8, k_scale, v_scale, dsx)
    B, Hq, Nq, d = q.shape
    _, Hkv, Nk, _ = k_i4.shape
    if out is None:
        out = torch.empty_like(q)
    _dev(out)
    _check(lib().sage_attn_fwd_q4(q.data_ptr(), q_mean.data_ptr(), k_i4.data_ptr(), v_fp8.data_ptr(), k_scale.data_ptr(),
                                  v_scale.data_ptr(), dsx.data_ptr(), out.data_ptr(), B, Hq, Hkv, Nq, Nk, d, int(causal),
                                  float(sm_scale), float(p_r), _dt(q), _stream()))
    return out


def sage_attn_fwd_4bit(q, k, v, *, causal: bool, sm_scale: float = 0.0, out: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None):
    """Whole forward pass of the 4+8 variant for q [B,Hq,Nq,d] and k, v [B,Hkv,Nk,d]."""
    _dev(q, k, v)
    B, Hq, Nq, d = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[3] != d or k.dtype != q.dtype or v.dtype != q.dtype:
        raise SageError("k and v must share a shape [B,Hkv,Nk,d] and the dtype of q")
    _, Hkv, Nk, _ = k.shape
    if out is None:
        out = torch.empty_like(q)
    _dev(out)
    ws = workspace if workspace is not None else _workspace(workspace_bytes_4bit(B, Hq, Hkv, Nq, Nk, d), q.device)
    _check(lib().sage_attn_fwd_4bit(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, Hq, Hkv, Nq, Nk, d,
                                    int(causal), float(sm_scale), _stream(), _dt(q), ws.data_ptr(), ws.numel()))
    return out


def delta_s_to_key_order(dsx: torch.Tensor, Nk: int) -> torch.Tensor:
    """Undo the lane order of the score-correction buffer: [B,Hq,nQ,T,128] -> [B,Hq,nQ,Nk] (layout bookkeeping
    only).  Position 32*g + 4*t + j of a tile is key 16*t + 4*g + j."""
    B, H, nq, T, _ = dsx.shape
    x = dsx.reshape(B, H, nq, T, 4, 8, 4)            # [.., g, t, j]
    x = x.permute(0, 1, 2, 3, 5, 4, 6)               # [.., t, g, j]
    return x.reshape(B, H, nq, T * 128)[..., :Nk].contiguous()


def v_fp8_to_token_major(v_fp8: torch.Tensor, N: int) -> torch.Tensor:
    """Undo the library's V tile layout: [B,H,T,d,128] -> codes [B,H,N,d] (layout bookkeeping only).

    Byte 64*(t>>2) + 16*g + 4*(t&3) + i of a tile row is key 16*t + 4*g + i of that tile.
    """
    B, H, T, d, _ = v_fp8.shape
    x = v_fp8.reshape(B, H, T, d, 2, 4, 4, 4)       # [.., t>>2, g, t&3, i]
    x = x.permute(0, 1, 2, 4, 6, 5, 7, 3)           # [B, H, T, t>>2, t&3, g, i, d]
    return x.reshape(B, H, T * 128, d)[:, :, :N].contiguous()
