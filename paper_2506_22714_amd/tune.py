"""Offline threshold / load-balance sweep (the paper's "threshold tuner", Section 4.2.2 and Section 5.3.3).

The paper argues that the utilisation threshold eta_thr depends on the architecture, not on the matrix, and finds
it once per GPU by a sweep over representative matrices (its Fig. 11).  This script is that sweep for MI355X: for one
workload it builds a plan per candidate setting, times libra_spmm / libra_sddmm, and prints a table.  It calls the
library through the binding only.

    python -m paper_2506_22714_amd.tune --workload powerlaw --N 128 --K 32
    python -m paper_2506_22714_amd.tune --workload community --what tau_sddmm
    python -m paper_2506_22714_amd.tune --workload gat --N 64 --K 64 --what ablation
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def time_us(fn, reps: int = 30, warm: int = 5):
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in ev]) * 1e3)


SWEEPS = {
    "mode": [dict(mode=0), dict(mode=1), dict(mode=2)],
    "tau_spmm": [dict(spmm_min_vec_nnz=t) for t in (1, 2, 3, 4, 6, 8, 12, 16)],
    "tau_sddmm": [dict(sddmm_min_blk_nnz=t) for t in (16, 20, 24, 32, 48, 64, 96, 128)],
    "ts": [dict(ts=t) for t in (2, 4, 8, 16, 64)],
    "cs": [dict(cs=c) for c in (32, 64, 96, 128, 192, 256, 512)],
    "sddmm_cs": [dict(sddmm_cs=c) for c in (64, 128, 256, 512, 1024)],
}

# The parts of the method switched off one at a time (the paper's ablations, Section 5.4): not part of "all".
# Flag values as in libra.h: 1 no filling of padding slots, 8 window order, 32 | 256 heaviest first without any
# die-aware order or placement.
UNBOUNDED = 1 << 20
ABLATION = [
    ("as shipped", dict()),
    ("no load balancing (Ts, Cs unbounded)", dict(ts=UNBOUNDED, cs=UNBOUNDED)),
    ("dense part not decomposed (Ts unbounded)", dict(ts=UNBOUNDED)),
    ("long rows not decomposed (Cs unbounded)", dict(cs=UNBOUNDED)),
    ("window order instead of heaviest first", dict(flags=8)),
    ("heaviest first, nothing die-aware", dict(flags=32 | 256)),
    ("padding slots not filled", dict(flags=1)),
    ("matrix cores only", dict(mode=1)),
    ("vector ALUs only", dict(mode=2)),
]


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="powerlaw")
    ap.add_argument("--small", action="store_true")
    ap.add_argument("--N", type=int, default=128)
    ap.add_argument("--K", type=int, default=32)
    ap.add_argument("--what", default="all", help="one of: all, ablation, " + ", ".join(SWEEPS))
    args = ap.parse_args()

    import torch
    from . import binding as lb
    from . import workloads as wl

    A = wl.make(args.workload, small=args.small)
    B = torch.from_numpy(wl.dense_normal(A.Kc, args.N, seed=1)).cuda()
    X = torch.from_numpy(wl.dense_normal(A.M, args.K, seed=2)).cuda()
    Y = torch.from_numpy(wl.dense_normal(A.Kc, args.K, seed=3)).cuda()
    C = torch.empty((A.M, args.N), dtype=torch.float32, device="cuda")
    out = torch.empty(A.nnz, dtype=torch.float32, device="cuda")
    rowptr, col, val = (torch.from_numpy(x).cuda() for x in (A.rowptr.astype(np.int32), A.col.astype(np.int32), A.val))
    print(f"# {args.workload}: M={A.M} nnz={A.nnz} N={args.N} K={args.K}")
    print(f"# {'setting':34s} {'spmm us':>9s} {'dense':>6s} {'tasks':>8s} | {'sddmm us':>9s} {'dense':>6s} {'tasks':>8s}")
    if args.what == "ablation":
        for label, kw in ABLATION:
            p = lb.Plan.from_device_csr(A.M, A.Kc, rowptr, col, val, resident=True, keep_host_copy=False, **kw)
            st = p.stats()
            t_spmm, t_sddmm = time_us(lambda: p.spmm(B, out=C)), time_us(lambda: p.sddmm(X, Y, out=out))
            print(f"  {label:42s} {t_spmm:9.1f} {st['spmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['spmm_tasks']:8d} | "
                  f"{t_sddmm:9.1f} {st['sddmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['sddmm_tasks']:8d}", flush=True)
            p.close()
        return 0
    names = list(SWEEPS) if args.what == "all" else [args.what]
    for name in names:
        for kw in SWEEPS[name]:
            # a plan per setting, built on the GPU straight into device memory
            p = lb.Plan.from_device_csr(A.M, A.Kc, rowptr, col, val, resident=True, keep_host_copy=False, **kw)
            st = p.stats()
            t_spmm = time_us(lambda: p.spmm(B, out=C)) if name not in ("tau_sddmm", "sddmm_cs") else float("nan")
            t_sddmm = time_us(lambda: p.sddmm(X, Y, out=out)) if name not in ("tau_spmm", "cs") else float("nan")
            print(f"  {json.dumps(kw):34s} {t_spmm:9.1f} {st['spmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['spmm_tasks']:8d} | "
                  f"{t_sddmm:9.1f} {st['sddmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['sddmm_tasks']:8d}", flush=True)
            p.close()
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
