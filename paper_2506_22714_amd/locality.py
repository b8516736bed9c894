"""Which fetches of a plan miss the L2s: a replay of the SpMM task table through a model of the eight dies.

An analysis aid, not part of the compute path.  Workgroup b of a launch runs on die b mod 8 and every die has an L2 of
its own, so where the planner puts a task in the table decides which L2 sees its row fetches (Eq. 2 counts them: one
row of the dense operand per dense vector and per residual nonzero).  The model keeps, per die, an LRU set of operand
rows of a given capacity; the die's tasks start in table order, `slots` of them are resident at a time and each advances
`batch` fetches per round, which is how one-wave tasks with a fixed number of fetches in flight share a die.  With 3 MiB
of rows per die, 512 resident tasks and 32 fetches per round the model reproduces the fetch traffic that the counters
measure for the power-law plan at N = 128 (208 MB per call); it is then asked what-ifs about task placement.

    python -m paper_2506_22714_amd.locality --workload powerlaw --N 128

runs on the host only (the host planner builds the plan).
"""
from __future__ import annotations

import argparse
import json
from collections import OrderedDict

import numpy as np

N_DIES = 8


def task_columns(export: dict):
    """Per task of an exported SpMM sub-plan, in table order: the operand rows it fetches (block columns, then residual entries)."""
    tasks, bc, rc = export["tasks"], export["blk_cols"], export["res_col"]
    out = []
    for t in tasks:
        parts = []
        if t["blk_end"] > t["blk_begin"]:
            c = bc[t["blk_begin"]:t["blk_end"]].reshape(-1)
            parts.append(c[c >= 0])
        parts.append(rc[t["res_begin"]:t["res_end"]])
        out.append(np.concatenate(parts))
    return out


def replay(cols_per_task, kinds, capacity_rows: int, slots: int = 512, batch: int = 32) -> dict:
    """Fetches and misses per task kind; task i runs on die i mod 8."""
    acc = {}
    miss = {}
    distinct = 0
    for d in range(N_DIES):
        queue = list(range(d, len(cols_per_task), N_DIES))
        cache: OrderedDict = OrderedDict()
        seen = set()
        resident = []
        nxt = 0
        while nxt < len(queue) or resident:
            while len(resident) < slots and nxt < len(queue):
                i = queue[nxt]
                resident.append([cols_per_task[i].tolist(), 0, int(kinds[i])])
                nxt += 1
            still = []
            for r in resident:
                c, pos, kind = r
                for x in c[pos:pos + batch]:
                    acc[kind] = acc.get(kind, 0) + 1
                    if x in cache:
                        cache.move_to_end(x)
                    else:
                        miss[kind] = miss.get(kind, 0) + 1
                        cache[x] = True
                        if len(cache) > capacity_rows:
                            cache.popitem(last=False)
                    seen.add(x)
                r[1] = pos + batch
                if r[1] < len(c):
                    still.append(r)
            resident = still
        distinct += len(seen)
    return {"fetches": acc, "misses": miss, "distinct_rows_summed_over_dies": distinct}


def main(argv=None) -> int:
    from . import binding as lb
    from . import workloads as wl
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workload", default="powerlaw")
    ap.add_argument("--small", action="store_true", help="the reduced instance of the workload")
    ap.add_argument("--N", type=int, default=128, help="feature columns (a row of the 16-bit operand is 2 N bytes)")
    ap.add_argument("--cache-mib", type=float, nargs="+", default=[2.0, 3.0, 4.0], help="operand rows an L2 keeps, in MiB")
    ap.add_argument("--options", default='{"ts": 32, "cs": 128, "spmm_min_vec_nnz": 3}', help="plan options (JSON)")
    args = ap.parse_args(argv)
    A = wl.make(args.workload, small=args.small)
    p = lb.Plan(A.M, A.Kc, A.rowptr.astype(np.int32), A.col.astype(np.int32), A.val, **json.loads(args.options))
    e = p.export(0)
    cols = task_columns(e)
    kinds = e["tasks"]["kind"]
    row_bytes = 2 * args.N
    total = sum(len(c) for c in cols)
    print(f"# {args.workload}: nnz {A.nnz}, {len(cols)} tasks, {total} row fetches of {row_bytes} bytes, "
          f"{len(np.unique(np.concatenate(cols)))} distinct rows")
    print("# capacity MiB | fetches window / segment tasks | misses window / segment tasks | missed MB | rows distinct per die, summed")
    for mib in list(args.cache_mib) + [float("inf")]:
        cap = int(mib * (1 << 20) // row_bytes) if np.isfinite(mib) else 1 << 62
        r = replay(cols, kinds, cap)
        f, m = r["fetches"], r["misses"]
        print(f"  {mib:8} | {f.get(0, 0):9d} / {f.get(1, 0):9d} | {m.get(0, 0):9d} / {m.get(1, 0):9d} | "
              f"{sum(m.values()) * row_bytes / 1e6:8.1f} | {r['distinct_rows_summed_over_dies']}", flush=True)
    p.close()
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
