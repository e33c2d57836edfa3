#!/usr/bin/env python3
"""Benchmark of the SageAttention2++ 8+8 forward pass on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: K smoothing + INT8 quantisation of K, FP8
quantisation of V (one joint call), fused attention with the INT8 quantisation
of Q in its prologue -- the two C-ABI stage calls that ``sage_attn_fwd`` makes,
on one stream, with HIP events between them so that the attention kernel's own
duration is measured inside the timed region.

Prints ONE JSON line (metric: attention TOPS = 4*B*H*N^2*d / t, halved when
causal), with the MFMA roofline of the attention kernel and the CPU oracle's
throughput on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published dense peaks used for the roofline
PEAK_MFMA_8BIT = 5.0e15      # INT8 and FP8 dense, op/s
PEAK_HBM = 8.0e12            # B/s

# What rocprofv3 measured for the attention kernel on a workload (summaries under profiles/): HBM traffic of one
# launch (FETCH_SIZE / WRITE_SIZE scaled by a copy kernel of known size) and, per wavefront and 128-key step,
# the vector instructions issued, how many of them are MFMA, and how many run at half rate (exp, FP8 pack).
# Only workloads that were profiled have an entry; everything derived from a missing entry is null in the
# JSON line.  `valu_busy` / `mfma_busy` are SQ_ACTIVE_INST_VALU and SQ_VALU_MFMA_BUSY_CYCLES as fractions of
# the kernel's SIMD time.
PROFILED = {
    "cfg5": dict(source="profiles/attn_kernel_cfg5_counters.md",
                 traffic=int(885132 * 1024 * 2.0 + 196608 * 1024 * 1.0),
                 valu_per_step=222.2, mfma_i8=16, mfma_f8=8, half_rate=49.2, valu_busy=0.88, mfma_busy=0.41),
    "cfg3": dict(source="profiles/attn_kernel_cfg5_counters.md (section cfg3)", traffic=None,
                 valu_per_step=211.7, mfma_i8=8, mfma_f8=4, half_rate=49.2, valu_busy=0.98, mfma_busy=0.24),
    # causal: per executed wavefront-step, prologue and epilogue of the short workgroups included
    "cfg2": dict(source="profiles/attn_kernel_cfg5_counters.md (section cfg2)",
                 traffic=int(174437 * 1024 * 2.0 + 131182 * 1024 * 1.0),
                 valu_per_step=266.9, mfma_i8=16, mfma_f8=8, half_rate=49.0, valu_busy=0.80, mfma_busy=0.32),
}


def alu_bound(prof):
    """The co-limit of the MFMA roofline: the vector-ALU issue port, which MFMA and ordinary vector
    instructions share.  Port cycles per wavefront-step from the measured instruction mix -- 4 cycles per
    full-rate instruction and per 4-pass MFMA (INT8 16x16x64), 8 per half-rate instruction and per 8-pass MFMA
    (FP8 16x16x128) -- against the MFMA pipe's own cycles for the same step (16 and 32 per instruction): their
    ratio is the fraction of the MFMA peak this instruction mix can reach at equal clock."""
    if not prof:
        return None
    n_mfma = prof["mfma_i8"] + prof["mfma_f8"]
    other = prof["valu_per_step"] - n_mfma
    port = 4.0 * (other - prof["half_rate"]) + 8.0 * prof["half_rate"] + 4.0 * prof["mfma_i8"] + 8.0 * prof["mfma_f8"]
    pipe = 16.0 * prof["mfma_i8"] + 32.0 * prof["mfma_f8"]
    return {"port_cycles_per_wavefront_step": round(port, 1), "mfma_cycles_per_wavefront_step": pipe,
            "frac_of_peak_allowed": round(pipe / port, 4), "peak_allowed": round(PEAK_MFMA_8BIT / 1e12 * pipe / port, 1),
            "unit": "TFLOP/s", "instruction_mix_from": prof["source"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed steps before the timed ones (default: at least 3 and at least 0.15 s of them -- "
                         "the clock of a GPU coming out of idle takes some tens of ms of load to settle)")
    ap.add_argument("--config", default="cfg5", help="cfg1..cfg5 (default: the d=128, N=32768 target workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU time budget of the oracle sample")
    ap.add_argument("--staged-q", action="store_true",
                    help="quantise Q with the stand-alone kernel (sage_quant_q + sage_attn_fwd_quantized) instead "
                         "of inside the attention kernel; same result bit for bit, for comparison")
    ap.add_argument("--quant-path", choices=["auto", "three-launches", "single-read"], default="auto",
                    help="kernels of the K/V quantisation stage: chosen by shape (default), always the three "
                         "launches (statistics, finalize, codes: K and V read twice), or always the single-read "
                         "kernel; same result bit for bit, for comparison")
    ap.add_argument("--no-mfma-peak", action="store_true",
                    help="skip the live measurement of the matrix-pipe rate (roofline.peak_measured)")
    ap.add_argument("--mfma-table", action="store_true",
                    help="only measure the matrix-pipe rates (INT8 16x16x64, FP8 16x16x128, FP8 16x16x32, the "
                         "attention kernel's mix) with the library's MFMA-only kernel, print them as JSON and exit")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain device copy of Q (2E bytes read, 2E written) before the timed loop: "
                         "the known-size kernel that FETCH_SIZE / WRITE_SIZE counter runs are scaled by")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path would shard over batch*heads with no "
              "exchange between the GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2505_21136_amd as sage
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(2)
    sage.lib()
    sage.diag_quant_kv_path({"auto": 0, "three-launches": 1, "single-read": 2}[args.quant_path])
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.mfma_table:
        names = ["int8_16x16x64", "fp8_16x16x128_f8f6f4", "fp8_16x16x32", "attention_mix_2xint8_1xfp8"]
        for _ in range(2):      # the first round warms the clock up
            rates = {n: round(sage.diag_mfma_rate(k, iters=8192, workgroups=2048, repeats=5) / 1e12, 1)
                     for k, n in enumerate(names)}
        print(json.dumps({"mfma_rate_TOPS": rates, "published_peak_TOPS": PEAK_MFMA_8BIT / 1e12}), flush=True)
        return
    cfg = {c.name: c for c in wl.CONFIGS}[args.config]

    t0 = time.time()
    q_h, k_h, v_h = wl.generate(cfg)
    q, k, v = q_h.to(dev), k_h.to(dev), v_h.to(dev)
    print(f"[bench] {cfg.name}: inputs generated and uploaded in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    B, H, N, d = cfg.B, cfg.H, cfg.N, cfg.d
    sm_scale = float(np.float32(cfg.sm_scale))
    out = torch.empty_like(q)
    qws = torch.empty(sage.quant_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=dev)
    # outputs of stage 1, allocated once (nothing is allocated inside the timed region)
    k_i8, k_scale, k_mean, v_fp8, v_scale = sage.sage_quant_kv(k, v, 4.5, qws)
    if args.staged_q:
        q_i8, q_scale = sage.sage_quant_q(q)
    L = sage.lib()
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    dt = 1 if cfg.dtype == "bf16" else 0

    def step(ev=None):
        rc = L.sage_quant_kv(k.data_ptr(), v.data_ptr(), k_i8.data_ptr(), k_scale.data_ptr(), k_mean.data_ptr(),
                             v_fp8.data_ptr(), v_scale.data_ptr(), 4.5, B, H, N, d, dt, sp, qws.data_ptr(), qws.numel())
        if args.staged_q:
            rc |= L.sage_quant_q(q.data_ptr(), q_i8.data_ptr(), q_scale.data_ptr(), B, H, N, d, dt, sp)
        if ev:
            ev[0].record(stream)
        if args.staged_q:
            rc |= L.sage_attn_fwd_quantized(q_i8.data_ptr(), k_i8.data_ptr(), v_fp8.data_ptr(), q_scale.data_ptr(),
                                            k_scale.data_ptr(), v_scale.data_ptr(), out.data_ptr(), B, H, N, d,
                                            int(cfg.causal), sm_scale, 224.0, dt, sp)
        else:
            rc |= L.sage_attn_fwd_kvquantized_gqa(q.data_ptr(), k_i8.data_ptr(), v_fp8.data_ptr(), k_scale.data_ptr(),
                                                  v_scale.data_ptr(), out.data_ptr(), B, H, H, N, N, d,
                                                  int(cfg.causal), sm_scale, 224.0, dt, sp)
        if ev:
            ev[1].record(stream)
        if rc != 0:
            raise RuntimeError("libsage call failed")

    if args.calib_copy:
        calib = torch.empty_like(q)
        calib.copy_(q)
        torch.cuda.synchronize()
    if args.warmup is None:
        t_w = time.perf_counter()
        for _ in range(3):
            step()
        torch.cuda.synchronize()
        more = int(0.15 / max((time.perf_counter() - t_w) / 3, 1e-5))
        for _ in range(more):  # enqueued back to back, like the timed steps
            step()
        args.warmup = 3 + more
    else:
        for _ in range(args.warmup):
            step()
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    ms_per_step = 1e3 * elapsed / args.steps
    tops = cfg.ops / (elapsed / args.steps) / 1e12
    attn_ms = sum(a.elapsed_time(b) for a, b in events) / args.steps
    attn_tops = cfg.ops / (attn_ms * 1e-3) / 1e12
    quant_ms = ms_per_step - attn_ms
    E = B * H * N * d
    # K and V: 2 bytes read + 1 byte written per element (Q is quantised inside the attention kernel)
    quant_gbs = (9.0 if args.staged_q else 6.0) * E / (quant_ms * 1e-3) / 1e9 if quant_ms > 0 else None

    prof = PROFILED.get(cfg.name)
    # the matrix-pipe rate this GPU sustains on the kernel's own instruction mix (two INT8 16x16x64 per FP8
    # 16x16x128), measured now, on the warm GPU, with the library's MFMA-only kernel
    peak_measured = None if args.no_mfma_peak else sage.diag_mfma_rate(3) / 1e12

    result = {
        "metric": "attention TOPS (4*B*H*N^2*d/s, halved when causal), quantisation + attention",
        "value": round(tops, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 (QK^T, int32 acc) + fp8 e4m3 (PV, fp32 acc); fp32 softmax",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={B} H={H} N={N} d={d} {'causal' if cfg.causal else 'non-causal'} "
                               f"{cfg.dtype}, Q {cfg.q_dist}, K bias std 3"
                               + (f", {cfg.k_outlier_channels} K outlier channels x20" if cfg.k_outlier_channels else ""),
                   "p_r": 224.0, "v_r": 4.5, "bq": 128, "bk": 64, "w": 128},
        "roofline": {
            "kernel": "attn_kernel (" + ("" if args.staged_q else "Q quantisation + ")
                      + "fused INT8 QK^T + softmax + FP8 PV)",
            "bound": "mfma",
            "achieved": round(attn_tops, 2),
            "peak": PEAK_MFMA_8BIT / 1e12,
            "unit": "TFLOP/s",
            "frac": round(attn_tops * 1e12 / PEAK_MFMA_8BIT, 4),
            "traffic": prof["traffic"] if prof else None,
            "kernel_ms": round(attn_ms, 4),
            # measured in this run: MFMA-only kernel, same instruction mix (null with --no-mfma-peak)
            "peak_measured": round(peak_measured, 1) if peak_measured else None,
            "frac_of_peak_measured": round(attn_tops / peak_measured, 4) if peak_measured else None,
            # from the rocprofv3 counters of this workload (null for a workload that was not profiled)
            "alu_bound": alu_bound(prof),
            "limiter": (f"vector-ALU issue port (softmax arithmetic shares it with MFMA issue): "
                        f"{100 * prof['valu_busy']:.0f} % busy, MFMA pipe {100 * prof['mfma_busy']:.0f} % "
                        f"[{prof['source']}]") if prof else None,
        },
        "quant_stage": {"ms": round(quant_ms, 4), "algorithmic_GBps": round(quant_gbs, 1) if quant_gbs else None,
                        "frac_of_hbm_peak": round(quant_gbs * 1e9 / PEAK_HBM, 4) if quant_gbs else None,
                        "kernels": args.quant_path},
    }

    if not args.no_cpu_baseline:
        result.update(cpu_baseline(cfg, q_h, k_h, v_h, out, args.cpu_seconds))
    print(json.dumps(result), flush=True)


def cpu_baseline(cfg, q_h, k_h, v_h, out, budget_s):
    """Time the CPU oracle (as it stands) on a bounded sample: head (0,0), quantisation of the
    whole head plus attention for evenly spaced query rows; compare the GPU output on those rows."""
    import numpy as np

    import oracle
    import workloads as wl

    qf, kf, vf = (wl.as_f32(t[0, 0]) for t in (q_h, k_h, v_h))
    sm = np.float32(cfg.sm_scale)
    N, d = cfg.N, cfg.d
    t0 = time.perf_counter()
    quant = oracle.quantize_head(qf, kf, vf)
    t_quant = time.perf_counter() - t0

    def rows_ops(r0, r1):
        if cfg.causal:
            return sum(4.0 * (r + 1) * d for r in range(r0, r1))
        return 4.0 * (r1 - r0) * N * d

    # 128-row query blocks in a spread-out order (golden-ratio stride), until the time budget is used
    nblk_total = -(-N // 128)
    stride = max(1, int(nblk_total * 0.6180339887)) | 1
    while math.gcd(stride, nblk_total) != 1:
        stride += 2
    order = [(i * stride) % nblk_total for i in range(nblk_total)]
    blocks = []
    ops = 0.0
    refs, gots = [], []
    t0 = time.perf_counter()
    for i in order:
        r0, r1 = i * 128, min(N, (i + 1) * 128)
        ref, _ = oracle.sage_attention_head(qf, kf, vf, causal=cfg.causal, sm_scale=sm, out_dtype=cfg.dtype,
                                            row0=r0, row1=r1, quant=quant)
        ops += rows_ops(r0, r1)
        refs.append(ref)
        gots.append(out[0, 0, r0:r1].float().cpu().numpy())
        blocks.append(i)
        if time.perf_counter() - t0 + t_quant > budget_s:
            break
    t_attn = time.perf_counter() - t0
    ref, got = np.concatenate(refs), np.concatenate(gots)
    # the sample's share of the head's quantisation work is charged in proportion
    share = sum(min(N, (i + 1) * 128) - i * 128 for i in blocks) / N
    t_total = t_attn + t_quant * share
    return {
        "cpu_baseline": {"value": round(ops / t_total / 1e12, 6), "unit": "TOPS", "cores": oracle.num_threads(),
                         "kind": "oracle",
                         "sample": f"head (0,0): {len(blocks)} query blocks of 128 rows against all {N} keys "
                                   f"({t_attn:.1f}s attention + {t_quant * share:.2f}s share of the head's quantisation)"},
        "accuracy": {"rows": int(ref.shape[0]), "cos_vs_oracle": round(wl.cos_sim(ref, got), 7),
                     "rel_l1_vs_oracle": float(f"{wl.rel_l1(ref, got):.3e}")},
    }


if __name__ == "__main__":
    main()
