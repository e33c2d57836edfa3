#!/usr/bin/env python3
"""CPU-only study: what does the static scale of P~ (delta_P = 1/P_r) cost or gain against Section 3.1 Eq. 2
read literally (delta_P = max(P~)/P_r per Q block x key step)?

For small versions of the five workloads (same distributions, dtype, mask and head dimension; N and the head
count reduced so that the oracle finishes in seconds) this prints, over all compared rows,
  * the distance between the two modes (16-bit outputs),
  * the accuracy of each against full-precision attention (double precision softmax(QK^T/sqrt(d))V on the
    unquantised 16-bit inputs), as cosine similarity, relative L1 and RMSE (paper, appendix "Accuracy metrics").
Calls only the oracle.  Usage:  python oracle/study_delta_p.py [--n 2048] [--heads 2]
"""
import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import workloads as wl  # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=2048, help="sequence length of the reduced workloads")
    ap.add_argument("--heads", type=int, default=2)
    args = ap.parse_args()
    print(f"| workload (N={args.n}, {args.heads} heads) | static vs block_max: relL1 | static vs full precision: "
          "cos / relL1 / rmse | block_max vs full precision: cos / relL1 / rmse |")
    print("|---|---|---|---|")
    for base in wl.CONFIGS:
        n = min(args.n, base.N)
        cfg = base.scaled(B=1, H=args.heads, N=n)
        q, k, v = wl.generate(cfg)
        sm = np.float32(cfg.sm_scale)
        outs = {"static": [], "block_max": [], "fp": []}
        for h in range(cfg.H):
            qf, kf, vf = (wl.as_f32(t[0, h]) for t in (q, k, v))
            quant = oracle.quantize_head(qf, kf, vf)
            for mode in ("static", "block_max"):
                o, _ = oracle.sage_attention_head(qf, kf, vf, causal=cfg.causal, sm_scale=sm, out_dtype=cfg.dtype,
                                                  quant=quant, delta_p=mode)
                outs[mode].append(o)
            outs["fp"].append(oracle.attn_rows_fp(qf, kf, vf, causal=cfg.causal, sm_scale=sm))
        st, bm, fp = (np.stack(outs[m]) for m in ("static", "block_max", "fp"))

        def acc(x):
            return f"{100 * wl.cos_sim(fp, x):.4f} % / {wl.rel_l1(fp, x):.5f} / {wl.rmse(fp, x):.3e}"

        print(f"| {base.name}: d={cfg.d} {cfg.dtype} {'causal' if cfg.causal else 'full'}"
              f"{', Student-t Q, K outliers' if cfg.k_outlier_channels else ''} | {wl.rel_l1(st, bm):.3e} | {acc(st)} | {acc(bm)} |",
              flush=True)


if __name__ == "__main__":
    main()
