"""Oracle-only study: what does the MXFP4 substitution (the build's format) cost against the paper's NVFP4,
what would a scale rule that never saturates change, and how does the paper's single global k (App. B) compare
with the per-row budget rule of the benchmark configurations?

Runs the CPU oracle on sampled query blocks of the synthetic Qwen3-8B-shaped workload and prints the relative
Frobenius error against fp64 exact attention and the error-gap recovery at 5 / 10 / 25 % budgets.
Test infrastructure: calls only oracle/ and the seeded input generators.

    python -m oracle.format_study [--seq 32768]
"""
from __future__ import annotations

import argparse
import math
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import thrift_oracle as O  # noqa: E402
from paper_2605_23081_amd import metrics  # noqa: E402
from paper_2605_23081_amd import workloads as W  # noqa: E402


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--seq", type=int, default=32768)
    args = ap.parse_args()
    wl = W.scaled(W.QWEN3_131K, N=args.seq)
    q, k, v = W.make_q_head(wl, 0, 0), *W.make_kv_head(wl, 0, 0)
    q, k, v = q[None, None], k[None, None], v[None, None]
    qb, dt = O.bits_of(q); kb, _ = O.bits_of(k); vb, _ = O.bits_of(v)
    Tq = wl.N // wl.Bq
    picks = sorted({Tq - 1, (3 * Tq) // 4, Tq // 2, Tq // 4, Tq // 16, 0})
    units = np.array([(0, 0, i) for i in picks], np.int32)
    rows = np.array([(0, 0, i * wl.Bq + r) for i in picks for r in range(wl.Bq)], np.int32)
    scale = 1 / math.sqrt(wl.D)
    exact = O.attn_exact(qb, kb, vb, dt, True, scale, rows)
    qm = O.block_means(qb, dt, wl.Bq); km = O.block_means(kb, dt, wl.Bk)
    print(f"workload {wl.name} N={wl.N}, head 0, query blocks {picks}; rel. Frobenius error vs fp64 exact attention")
    print(f"{'format':9s} " + " ".join(f"{'f=' + str(f):>10s}" for f in (0.0, 0.05, 0.10, 0.25, 1.0)) + "   recovery % at 5/10/25")
    Tk = wl.N // wl.Bk
    for name, fmt, global_k in (("MXFP4", 0, False), ("NVFP4", 1, False), ("MX-nosat", 2, False), ("MX-glob-k", 0, True)):
        errs = {}
        for f in (0.0, 0.05, 0.10, 0.25, 1.0):
            # App. B: one k for every row, chosen so that the causal tile fraction is closest to f
            fixed_k = O.paper_global_k(Tk, f) if global_k and 0.0 < f < 1.0 else -1
            idx, cnt = O.select_topk(qm, km, wl.Bq, wl.Bk, True, f, fixed_k)
            out = O.attn_thrift_prefill(qb, kb, vb, dt, idx, cnt, wl.Bq, wl.Bk, True, scale, units, fmt=fmt)
            errs[f] = metrics.rel_fro(out.reshape(-1, wl.D), exact)
        rec = [100 * metrics.recovery(errs[1.0], errs[0.0], errs[f]) for f in (0.05, 0.10, 0.25)]
        print(f"{name:9s} " + " ".join(f"{errs[f]:10.5f}" for f in (0.0, 0.05, 0.10, 0.25, 1.0)) + "   " + " / ".join(f"{r:.1f}" for r in rec))
    return 0


if __name__ == "__main__":
    sys.exit(main())
