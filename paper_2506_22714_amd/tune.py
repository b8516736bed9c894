"""Offline threshold / load-balance sweep (the paper's "threshold tuner", Section 4.2.2 and Section 5.3.3).

The paper argues that the utilisation threshold eta_thr depends on the architecture, not on the matrix, and finds
it once per GPU by a sweep over representative matrices (its Fig. 11).  This script is that sweep for MI355X: for one
workload it builds a plan per candidate setting, times libra_spmm / libra_sddmm, and prints a table.  It calls the
library through the binding only.

    python -m paper_2506_22714_amd.tune --workload powerlaw --N 128 --K 32
    python -m paper_2506_22714_amd.tune --workload community --what tau_sddmm
    python -m paper_2506_22714_amd.tune --workload gat --N 64 --K 64 --what ablation
    python -m paper_2506_22714_amd.tune --workload powerlaw --what row_order       # rows permuted before planning
    python -m paper_2506_22714_amd.tune --emit tuned.json          # the tuner: best settings per width class, as a table
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
    "sddmm_ts": [dict(sddmm_ts=t) for t in (1, 2, 4, 8, 16)],
    "cs": [dict(cs=c) for c in (32, 64, 96, 128, 192, 256, 512)],
    "sddmm_cs": [dict(sddmm_cs=c) for c in (64, 128, 256, 512, 1024)],
    "sddmm_share": [dict(sddmm_min_blk_nnz=32, sddmm_min_dense_pct=c) for c in (0, 25, 50, 75, 100)],
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


# ---------------------------------------------------------------------------------------------------------------
# The tuner proper: per (value type, feature-width class) the setting with the best geometric mean over the workloads,
# found by coordinate descent from the library's defaults, written as a table that Plan.from_* can apply (tuned=...).
# ---------------------------------------------------------------------------------------------------------------
SPMM_AXES = [("spmm_min_vec_nnz", (2, 3, 4, 6)), ("ts", (8, 16, 32, 64)), ("cs", (64, 96, 128, 192, 256))]
SDDMM_AXES = [("sddmm_min_blk_nnz", (16, 32, 64, 128, 257)), ("sddmm_cs", (64, 128, 256)), ("sddmm_ts", (2, 4, 8, 16)),
              ("sddmm_min_dense_pct", (0, 50))]       # 0: the share rule is off
SPMM_START = dict(spmm_min_vec_nnz=3, ts=16, cs=128)
SDDMM_START = dict(sddmm_min_blk_nnz=64, sddmm_cs=128, sddmm_ts=4, sddmm_min_dense_pct=0)
N_CLASSES = {"n32": 32, "n64": 64, "n128": 128}      # class name -> the width the class is tuned at
K_CLASSES = {"k32": 32, "k64": 64, "k128": 128}
TUNER_WORKLOADS = ("powerlaw", "community", "gat", "irregular")


def permute_rows(A, order):
    """The matrix with row order[k] as its row k (columns untouched): what a plan-time row reordering would hand the planner.
    C = A B then comes out in the permuted row order."""
    from . import workloads as wl
    deg = np.diff(A.rowptr).astype(np.int64)[order]
    rp = np.zeros(A.M + 1, dtype=np.int64)
    np.cumsum(deg, out=rp[1:])
    idx = np.repeat(A.rowptr[:-1].astype(np.int64)[order] - rp[:-1], deg) + np.arange(rp[-1])
    return wl.Csr(A.M, A.Kc, rp.astype(np.int32), A.col[idx], A.val[idx])


def row_orders(A) -> dict:
    """Row orders tried by `--what row_order`: as given; by descending length (long rows share windows, so their common
    columns become vectors with several nonzeros); by descending length inside classes of 16 consecutive windows only
    (the same idea without moving rows far)."""
    deg = np.diff(A.rowptr)
    ident = np.arange(A.M)
    block = 256
    local = np.concatenate([s + np.argsort(-deg[s:s + block], kind="stable") for s in range(0, A.M, block)])
    return {"as given": ident, "descending length": np.argsort(-deg, kind="stable"), "descending length inside 256 rows": local}


def n_class(N: int) -> str:
    return "n32" if N <= 32 else "n64" if N <= 64 else "n128"


def k_class(K: int) -> str:
    return "k32" if K <= 32 else "k64" if K <= 64 else "k128"


def geomean(xs) -> float:
    return float(np.exp(np.mean(np.log(np.asarray(xs, dtype=np.float64)))))


def coordinate_descent(axes, start: dict, cost, rounds: int = 2, log=print):
    """Minimise cost(setting) over the grid `axes`, one axis at a time, starting from `start`; every evaluated setting
    is kept.  Returns (best setting, its cost, {setting as sorted tuple: cost})."""
    seen = {}

    def ev(setting):
        key = tuple(sorted(setting.items()))
        if key not in seen:
            seen[key] = cost(setting)
            log(f"    {json.dumps(setting):70s} {seen[key]:10.2f}")
        return seen[key]

    best, best_cost = dict(start), ev(start)
    for _ in range(rounds):
        moved = False
        for name, values in axes:
            for v in values:
                cand = dict(best, **{name: v})
                c = ev(cand)
                if c < best_cost * 0.995:           # a change has to be worth half a percent
                    best, best_cost, moved = cand, c, True
        if not moved:
            break
    return best, best_cost, seen


def load_table(path_or_dict):
    if isinstance(path_or_dict, dict):
        table = path_or_dict
    else:
        with open(path_or_dict) as f:
            table = json.load(f)
    if table.get("format") != "libra-tuned-1" or "spmm" not in table or "sddmm" not in table:
        raise ValueError("not a table written by `python -m paper_2506_22714_amd.tune --emit`")
    return table


def tuned_options(table, dtype: str = "f16", N: int | None = None, K: int | None = None) -> dict:
    """Plan options for a value type and the feature widths the plan will be used with (the SpMM options come from the
    class of N, the SDDMM options from the class of K; a width that is not given leaves its options at their defaults).
    bfloat16 uses the float16 entries; a value type without entries
    falls back to float16."""
    table = load_table(table)
    allowed = {n for n, _ in SPMM_AXES} | {n for n, _ in SDDMM_AXES}
    out = {}
    for op, cls in (("spmm", n_class(N) if N else None), ("sddmm", k_class(K) if K else None)):
        if cls is None:
            continue
        per_type = table[op].get("f16" if dtype == "bf16" else dtype) or table[op]["f16"]
        for name, v in per_type[cls]["options"].items():
            if name not in allowed or not isinstance(v, int) or v < (0 if name == "sddmm_min_dense_pct" else 1):
                raise ValueError(f"bad entry {name}={v!r} in the tuned table")
            out[name] = v
    return out


def emit_table(path: str, small: bool, dtypes, log=print) -> dict:
    import torch
    from . import binding as lb
    from . import workloads as wl

    table = {"format": "libra-tuned-1", "device": torch.cuda.get_device_name(0), "small_workloads": bool(small),
             "workloads": list(TUNER_WORKLOADS), "objective": "geometric mean of the median call time (us) over the workloads",
             "spmm": {}, "sddmm": {}}
    mats = {name: wl.make(name, small=small) for name in TUNER_WORKLOADS}
    dev = {name: tuple(torch.from_numpy(x).cuda() for x in (A.rowptr.astype(np.int32), A.col.astype(np.int32))) for name, A in mats.items()}
    for dt in dtypes:
        np_dt, code = (np.float32, lb.F32) if dt == "f32" else (np.float16, lb.F16)
        vals = {name: torch.from_numpy(A.val.astype(np_dt)).cuda() for name, A in mats.items()}

        def plan(name, **kw):
            A = mats[name]
            return lb.Plan.from_device_csr(A.M, A.Kc, dev[name][0], dev[name][1], vals[name], resident=True, keep_host_copy=False, **kw)

        table["spmm"][dt], table["sddmm"][dt] = {}, {}
        for cls, N in N_CLASSES.items():
            log(f"  spmm {dt} {cls} (N={N})")
            Bs = {name: torch.from_numpy(wl.dense_normal(A.Kc, N, seed=1, dtype=np_dt)).cuda() for name, A in mats.items()}
            Cs = {name: torch.empty((A.M, N), dtype=torch.float32, device="cuda") for name, A in mats.items()}

            def cost(setting):
                ts = []
                for name in TUNER_WORKLOADS:
                    p = plan(name, flags=lb.FLAG_NO_SDDMM, **setting)
                    ts.append(time_us(lambda: p.spmm(Bs[name], out=Cs[name]), reps=15, warm=3))
                    p.close()
                return geomean(ts)

            best, c, seen = coordinate_descent(SPMM_AXES, SPMM_START, cost, log=log)
            table["spmm"][dt][cls] = {"options": best, "geomean_us": round(c, 2), "defaults_geomean_us": round(seen[tuple(sorted(SPMM_START.items()))], 2),
                                      "settings_tried": len(seen)}
            del Bs, Cs
        for cls, K in K_CLASSES.items():
            log(f"  sddmm {dt} {cls} (K={K})")
            Xs = {name: torch.from_numpy(wl.dense_normal(A.M, K, seed=2, dtype=np_dt)).cuda() for name, A in mats.items()}
            Ys = {name: torch.from_numpy(wl.dense_normal(A.Kc, K, seed=3, dtype=np_dt)).cuda() for name, A in mats.items()}
            outs = {name: torch.empty(A.nnz, dtype=torch.float32, device="cuda") for name, A in mats.items()}

            def cost(setting):
                ts = []
                for name in TUNER_WORKLOADS:
                    p = plan(name, flags=lb.FLAG_NO_SPMM, **setting)
                    ts.append(time_us(lambda: p.sddmm(Xs[name], Ys[name], out=outs[name]), reps=15, warm=3))
                    p.close()
                return geomean(ts)

            best, c, seen = coordinate_descent(SDDMM_AXES, SDDMM_START, cost, log=log)
            table["sddmm"][dt][cls] = {"options": best, "geomean_us": round(c, 2), "defaults_geomean_us": round(seen[tuple(sorted(SDDMM_START.items()))], 2),
                                       "settings_tried": len(seen)}
            del Xs, Ys, outs
    with open(path, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    return table


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="powerlaw")
    ap.add_argument("--small", action="store_true")
    ap.add_argument("--N", type=int, default=128)
    ap.add_argument("--K", type=int, default=32)
    ap.add_argument("--what", default="all", help="one of: all, ablation, row_order, " + ", ".join(SWEEPS))
    ap.add_argument("--emit", metavar="TABLE.json", help="run the tuner over the four workloads and write the table of best "
                    "settings per value type and feature-width class (apply it with Plan.from_csr(..., tuned=TABLE.json, N=, K=))")
    ap.add_argument("--dtypes", default="f16", help="value types to tune, comma separated (f16, f32; bf16 uses the f16 entries)")
    args = ap.parse_args()
    if args.emit:
        t = emit_table(args.emit, args.small, [d for d in args.dtypes.split(",") if d])
        for op in ("spmm", "sddmm"):
            for dt, per in t[op].items():
                for cls, e in per.items():
                    print(f"{op:6s} {dt:4s} {cls:5s} {json.dumps(e['options']):60s} {e['geomean_us']:9.2f} us (defaults {e['defaults_geomean_us']:.2f})")
        return 0

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
    if args.what == "row_order":
        # plan-time row reordering: rows with similar columns in one window give vectors with more nonzeros, i.e. fewer
        # fetched rows (Eq. 2) - at the price of windows of long rows only
        for label, order in row_orders(A).items():
            P = permute_rows(A, order)
            rp, cl, vl = (torch.from_numpy(x).cuda() for x in (P.rowptr, P.col.astype(np.int32), P.val))
            for kw in (dict(ts=32), dict(ts=32, spmm_min_vec_nnz=2)):
                p = lb.Plan.from_device_csr(P.M, P.Kc, rp, cl, vl, resident=True, keep_host_copy=False, **kw)
                st = p.stats()
                t_spmm, t_sddmm = time_us(lambda: p.spmm(B, out=C)), time_us(lambda: p.sddmm(X, Y, out=out))
                print(f"  {label + ' ' + json.dumps(kw):62s} {t_spmm:9.1f} {st['spmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['spmm_tasks']:8d} | "
                      f"{t_sddmm:9.1f} {st['sddmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['sddmm_tasks']:8d}  fetched rows {st['spmm_gather_rows']}", flush=True)
                p.close()
        return 0
    names = list(SWEEPS) if args.what == "all" else [args.what]
    for name in names:
        for kw in SWEEPS[name]:
            # a plan per setting, built on the GPU straight into device memory
            p = lb.Plan.from_device_csr(A.M, A.Kc, rowptr, col, val, resident=True, keep_host_copy=False, **kw)
            st = p.stats()
            t_spmm = time_us(lambda: p.spmm(B, out=C)) if name not in ("tau_sddmm", "sddmm_cs", "sddmm_share") else float("nan")
            t_sddmm = time_us(lambda: p.sddmm(X, Y, out=out)) if name not in ("tau_spmm", "cs") else float("nan")
            print(f"  {json.dumps(kw):34s} {t_spmm:9.1f} {st['spmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['spmm_tasks']:8d} | "
                  f"{t_sddmm:9.1f} {st['sddmm_dense_nnz'] / max(A.nnz, 1):6.3f} {st['sddmm_tasks']:8d}", flush=True)
            p.close()
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
