#!/usr/bin/env python3
"""Time the whole forward pass (sage_attn_fwd_gqa: K/V quantisation + attention with Q quantised in its
prologue; with --four-bit the 4+8 variant, sage_attn_fwd_4bit) on shapes the five benchmark workloads do not cover: grouped-query prefill, rectangular
(N_q != N_k) and decode-shaped calls.

    python -m paper_2505_21136_amd.shape_bench --shape B,Hq,Hkv,Nq,Nk,d[,causal[,fp16|bf16]] [--shape ...]

Inputs are seeded normal draws (K with a per-channel bias, as in the benchmark workloads), resident in HBM.
Prints one JSON line per shape: milliseconds per call (HIP events over `--steps` calls after a warm-up) and
attention TOPS = 4 * B * Hq * (visible query-key pairs) * d / t.

With --decode (shapes with few query rows over many keys) K and V are quantised once outside the timed
region (as a decode loop over a fixed cache would) and two attention-only calls are timed on them,
sage_attn_fwd_decode (query heads packed, key ranges) and sage_attn_fwd_kvquantized_gqa (the prefill kernel on the
same shape), with the rate at which each streams the quantised cache (2 * B * Hkv * Nk * d bytes per call).
"""
import argparse
import json
import sys

import torch

import paper_2505_21136_amd as sage


def visible_pairs(nq: int, nk: int, causal: bool) -> float:
    """Query-key pairs the mask leaves visible (causal: aligned to the end of both sequences)."""
    if not causal:
        return float(nq) * nk
    return float(nq) * (nk - nq) + nq * (nq + 1) / 2.0


def run(shape: str, steps: int, warm_s: float, four_bit: bool = False) -> dict:
    f = shape.split(",")
    B, Hq, Hkv, Nq, Nk, d = (int(x) for x in f[:6])
    causal = bool(int(f[6])) if len(f) > 6 else False
    dtype = {"fp16": torch.float16, "bf16": torch.bfloat16}[f[7] if len(f) > 7 else "bf16"]
    g = torch.Generator(device="cuda").manual_seed(250521136)
    q = torch.randn((B, Hq, Nq, d), generator=g, device="cuda").to(dtype)
    k = (torch.randn((B, Hkv, Nk, d), generator=g, device="cuda")
         + 3.0 * torch.randn((B, Hkv, 1, d), generator=g, device="cuda")).to(dtype)
    v = torch.randn((B, Hkv, Nk, d), generator=g, device="cuda").to(dtype)
    out = torch.empty_like(q)
    nbytes = (sage.workspace_bytes_4bit if four_bit else sage.workspace_bytes_gqa)(B, Hq, Hkv, Nq, Nk, d)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def call():
        if four_bit:
            sage.sage_attn_fwd_4bit(q, k, v, causal=causal, out=out, workspace=ws)
        else:
            sage.sage_attn_fwd_gqa(q, k, v, causal=causal, out=out, workspace=ws)

    call()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    call()
    b.record()
    b.synchronize()
    for _ in range(max(3, int(warm_s / max(a.elapsed_time(b) * 1e-3, 1e-5)))):   # let the clock settle
        call()
    a.record()
    for _ in range(steps):
        call()
    b.record()
    b.synchronize()
    ms = a.elapsed_time(b) / steps
    ops = 4.0 * B * Hq * visible_pairs(Nq, Nk, causal) * d
    return {"variant": "4+8" if four_bit else "8+8", "shape": dict(B=B, Hq=Hq, Hkv=Hkv, Nq=Nq, Nk=Nk, d=d, causal=causal, dtype=str(dtype).split(".")[-1]),
            "ms_per_call": round(ms, 4), "attention_TOPS": round(ops / (ms * 1e-3) / 1e12, 2),
            "workgroups": B * Hq * -(-Nq // 128)}


def run_decode(shape: str, steps: int, warm_s: float) -> dict:
    f = shape.split(",")
    B, Hq, Hkv, Nq, Nk, d = (int(x) for x in f[:6])
    causal = bool(int(f[6])) if len(f) > 6 else False
    dtype = {"fp16": torch.float16, "bf16": torch.bfloat16}[f[7] if len(f) > 7 else "bf16"]
    g = torch.Generator(device="cuda").manual_seed(250521136)
    q = torch.randn((B, Hq, Nq, d), generator=g, device="cuda").to(dtype)
    k = (torch.randn((B, Hkv, Nk, d), generator=g, device="cuda")
         + 3.0 * torch.randn((B, Hkv, 1, d), generator=g, device="cuda")).to(dtype)
    v = torch.randn((B, Hkv, Nk, d), generator=g, device="cuda").to(dtype)
    k_i8, k_scale, _, v_fp8, v_scale = sage.sage_quant_kv(k, v, 4.5)
    del k, v
    out = torch.empty_like(q)
    ws = torch.empty(max(256, sage.decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, d, 0)), dtype=torch.uint8,
                     device="cuda")
    sm = 1.0 / d ** 0.5

    def dec():
        sage.sage_attn_fwd_decode(q, k_i8, v_fp8, k_scale, v_scale, causal=causal, sm_scale=sm, out=out, workspace=ws)

    def pre():
        sage.sage_attn_fwd_kvquantized_gqa(q, k_i8, v_fp8, k_scale, v_scale, causal=causal, sm_scale=sm, out=out)

    res = {}
    for name, call in (("decode", dec), ("prefill_kernel", pre)):
        call()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        call()
        b.record()
        b.synchronize()
        for _ in range(max(3, int(warm_s / max(a.elapsed_time(b) * 1e-3, 1e-5)))):
            call()
        a.record()
        for _ in range(steps):
            call()
        b.record()
        b.synchronize()
        res[name] = a.elapsed_time(b) / steps
    cache_bytes = 2.0 * B * Hkv * Nk * d
    return {"shape": dict(B=B, Hq=Hq, Hkv=Hkv, Nq=Nq, Nk=Nk, d=d, causal=causal, dtype=str(dtype).split(".")[-1]),
            "split_keys": sage.decode_split_keys(B, Hq, Hkv, Nq, Nk),
            "decode_ms": round(res["decode"], 4), "prefill_kernel_ms": round(res["prefill_kernel"], 4),
            "decode_cache_GBps": round(cache_bytes / (res["decode"] * 1e-3) / 1e9, 1),
            "prefill_kernel_cache_GBps": round(cache_bytes / (res["prefill_kernel"] * 1e-3) / 1e9, 1)}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shape", action="append", required=True)
    ap.add_argument("--four-bit", action="store_true", help="time sage_attn_fwd_4bit (the 4+8 variant) instead")
    ap.add_argument("--decode", action="store_true",
                    help="time sage_attn_fwd_decode against the prefill kernel on already quantised K and V")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warm-seconds", type=float, default=0.15)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(2)
    for s in args.shape:
        if args.decode:
            print(json.dumps(run_decode(s, args.steps, args.warm_seconds)), flush=True)
        else:
            print(json.dumps(run(s, args.steps, args.warm_seconds, args.four_bit)), flush=True)


if __name__ == "__main__":
    main()
