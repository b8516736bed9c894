#!/usr/bin/env python3
"""Benchmark of the SpMM + SDDMM hot path on one MI355X.

A step is one pass of the whole path on the power-law workload: SpMM with
N=128 followed by SDDMM with K=32, both on the same plan (the plan is built
and uploaded once, outside the timed region, as the method prescribes).
Prints ONE JSON line.

  value      effective GFLOP/s of the step, (2*nnz*N + 2*nnz*K) / t
  roofline   the dominant kernel (the SpMM task kernel, N=128): algorithmic
             bytes of one SpMM / average duration of libra_spmm measured with
             events on the launch stream over 40 further steps right after
             the timed ones (the same number at any --steps); also the rate of
             its row fetches against a bare gather of the same rows
  cpu_baseline  the CPU oracle timed on the host cores on the same workload
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per libra_spmm call as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by the reading of a
# 1 GiB copy (--copy-calibration).  They live in a tracked file together with a digest of the kernel sources they were
# measured with (--traffic-from writes it); the bench line quotes them only while the sources are unchanged and the run
# uses exactly the measured configuration, and says null otherwise.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_measured.json")
SOURCE_DIRS = (os.path.join(ROOT, "paper_2506_22714_amd", "csrc"), os.path.join(ROOT, "include"))


def source_digest() -> str:
    """sha256 over the library's sources (names and contents, sorted): what a traffic measurement is valid for."""
    import hashlib
    h = hashlib.sha256()
    for d in SOURCE_DIRS:
        for fn in sorted(os.listdir(d)):
            if fn.endswith((".hip", ".cpp", ".h")):
                h.update(fn.encode())
                with open(os.path.join(d, fn), "rb") as f:
                    h.update(f.read())
    return h.hexdigest()


def measured_traffic(key: str):
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None
    if t.get("source_sha256") != source_digest():
        return None
    e = t.get("entries", {}).get(key)
    return int(e["bytes"]) if e else None


def _counter_means(directory: str, counter: str) -> dict:
    """kernel name -> mean reading of `counter` over the dispatches in a rocprofv3 --pmc csv under `directory`."""
    import csv
    import glob
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no counter csv under {directory}")
    acc: dict = {}
    for fn in files:
        with open(fn) as f:
            for r in csv.DictReader(f):
                if r["Counter_Name"] == counter:
                    acc.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}


def record_traffic(directory: str, key: str) -> int:
    """Reads <dir>/fetch, <dir>/write (counter runs of this bench) and <dir>/cal_fetch, <dir>/cal_write (counter runs of
    --copy-calibration) and writes TRAFFIC_FILE.  No GPU needed."""
    copy_bytes = float(1 << 30)
    out = {"source_sha256": source_digest(), "unit": "bytes per libra_spmm call (task kernel + the kernel that clears multi-writer rows)",
           "commands": ["rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir>/fetch -o pmc -- python3 bench.py --no-cpu-baseline --no-probes --steps 5 --warmup 2",
                        "rocprofv3 --pmc WRITE_SIZE ... -d <dir>/write ... (same program)",
                        "rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE ... -d <dir>/cal_fetch|cal_write ... -- python3 bench.py --copy-calibration",
                        "python3 bench.py --traffic-from <dir>"],
           "entries": {}}
    entry = {}
    for what, counter in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
        cal = _counter_means(os.path.join(directory, "cal_" + what), counter)
        cal_kib = max(cal.values())                                   # the copy kernel is the only large one in that run
        scale = copy_bytes / (cal_kib * 1024.0)
        run = _counter_means(os.path.join(directory, what), counter)
        kib = sum(v for k, v in run.items() if "spmm_task_kernel" in k or "zero_rows_kernel" in k)
        entry[what + "_kib_raw"] = round(kib, 1)
        entry[what + "_scale"] = round(scale, 4)
        entry[what + "_bytes"] = int(kib * 1024.0 * scale)
    entry["bytes"] = entry["fetch_bytes"] + entry["write_bytes"]
    out["entries"][key] = entry
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(out["entries"]))
    return 0


def spmm_algorithmic_bytes(A, N: int, kref: int, es: int = 2) -> int:
    """Every array of the method once: col + val, rowptr, referenced rows of B, C (es = bytes per stored value)."""
    return A.nnz * (4 + es) + 4 * (A.M + 1) + kref * N * es + A.M * N * 4


def sddmm_algorithmic_bytes(A, K: int, mref: int, kref: int, es: int = 2) -> int:
    return A.nnz * (4 + es + 4) + 4 * (A.M + 1) + (mref + kref) * K * es


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="powerlaw", choices=["powerlaw", "tiny", "community", "irregular", "gat"])
    ap.add_argument("--N", type=int, default=0)
    ap.add_argument("--K", type=int, default=0)
    ap.add_argument("--small", action="store_true", help="reduced instance (smoke runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", type=int, default=0)
    ap.add_argument("--tau-spmm", type=int, default=0)
    ap.add_argument("--tau-sddmm", type=int, default=0)
    ap.add_argument("--ts", type=int, default=0)
    ap.add_argument("--cs", type=int, default=0)
    ap.add_argument("--natural-order", action="store_true")
    ap.add_argument("--xcd-order", action="store_true", help="group tasks of neighbouring windows on one accelerator die")
    ap.add_argument("--no-xcd-order", action="store_true", help="never do that (default: the planner decides from the matrix)")
    ap.add_argument("--segments-by-cost", action="store_true", help="row segments in heaviest-first order instead of one column range per die")
    ap.add_argument("--two-kernels", action="store_true", help="SpMM as two launches (dense blocks, then residual nonzeros)")
    ap.add_argument("--host-plan", action="store_true",
                    help="run the compute calls on the host-built, uploaded plan (default: on the plan the device planner "
                         "wrote; the two plans are identical and both planners are timed either way)")
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16", "f32"], help="storage type of A's values and the dense operands")
    ap.add_argument("--no-tuned", action="store_true", help="library defaults instead of the tuner's table (paper_2506_22714_amd/tuned_gfx950.json)")
    ap.add_argument("--no-probes", action="store_true", help="skip the cold calls, the copy rate and the bare-gather probe (counter runs)")
    ap.add_argument("--traffic-from", metavar="DIR", help="no GPU: read rocprofv3 counter csvs under DIR and write profiles/traffic_measured.json")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a 1 GiB device copy (5 times): the known-size kernel that scales the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.traffic_from:
        return record_traffic(args.traffic_from, f"{args.workload}:N={args.N or 128}:{args.dtype}")
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2506_22714_amd import binding as lb
    from paper_2506_22714_amd import workloads as wl

    if not os.path.exists(lb.LIB_PATH):
        from paper_2506_22714_amd.build import build_library
        build_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_each_way": src.numel() * 4, "launches": 5}))
        return 0

    defaults = {"powerlaw": (128, 32), "tiny": (32, 32), "community": (128, 32), "irregular": (32, 32), "gat": (64, 64)}
    N = args.N or defaults[args.workload][0]
    K = args.K or defaults[args.workload][1]
    A = wl.make(args.workload, small=args.small)
    B = wl.dense_normal(A.Kc, N, seed=wl.BASE_SEED + 201)
    X = wl.dense_normal(A.M, K, seed=wl.BASE_SEED + 202)
    Y = wl.dense_normal(A.Kc, K, seed=wl.BASE_SEED + 203)

    bf16, f32 = args.dtype == "bf16", args.dtype == "f32"
    es = 4 if f32 else 2
    if f32:
        B, X, Y = (a.astype(np.float32) for a in (B, X, Y))
    val = wl.to_bf16_bits(A.val.astype(np.float32)) if bf16 else A.val.astype(np.float32) if f32 else None
    # thresholds and load-balance limits: the tuner's table for this value type and these widths, unless switched off or
    # given on the command line (explicit options win)
    tuned_path = os.path.join(ROOT, "paper_2506_22714_amd", "tuned_gfx950.json")
    tuned = None if args.no_tuned or not os.path.exists(tuned_path) else tuned_path
    opts = dict(tuned=tuned, N=N, K=K, mode=args.mode, spmm_min_vec_nnz=args.tau_spmm, sddmm_min_blk_nnz=args.tau_sddmm, ts=args.ts, cs=args.cs,
                flags=(lb.FLAG_NATURAL_ORDER if args.natural_order else 0) | (lb.FLAG_XCD_ORDER if args.xcd_order else 0)
                | (lb.FLAG_NO_XCD_ORDER if args.no_xcd_order else 0) | (lb.FLAG_SEGMENTS_BY_COST if args.segments_by_cost else 0)
                | (lb.FLAG_TWO_KERNELS if args.two_kernels else 0))
    # the plan is built once per matrix, outside the timed region, by both planners: on the host (+ upload) and on the
    # device (the plan's device copy written directly, no host copy kept)
    t0 = time.perf_counter()
    host_plan = lb.Plan.from_csr(A, val=val, val_dtype=lb.BF16 if bf16 else None, **opts)
    plan_s = time.perf_counter() - t0
    t0 = time.perf_counter()
    host_plan.upload()
    torch.cuda.synchronize()
    upload_s = time.perf_counter() - t0
    rp_d, col_d = torch.from_numpy(A.rowptr.astype(np.int32)).cuda(), torch.from_numpy(A.col.astype(np.int32)).cuda()
    val_d = (torch.from_numpy(val.view(np.int16)).cuda().view(torch.bfloat16) if bf16 else torch.from_numpy(A.val if val is None else val).cuda())
    dev_s = []
    dev_plan = None
    for _ in range(3):                      # the first call pays for module loading and the allocator
        if dev_plan is not None:
            dev_plan.close()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dev_plan = lb.Plan.from_device_csr(A.M, A.Kc, rp_d, col_d, val_d, resident=True, keep_host_copy=False, **opts)
        torch.cuda.synchronize()
        dev_s.append(time.perf_counter() - t0)
    hs, ds = host_plan.stats(), dev_plan.stats()
    assert all(hs[k] == ds[k] for k in hs if k not in ("plan_seconds", "device_seconds")), "the two planners disagree"
    plan = host_plan if args.host_plan else dev_plan
    (dev_plan if args.host_plan else host_plan).close()
    st = plan.stats()

    if bf16:
        B, X, Y = (wl.to_bf16_bits(a.astype(np.float32)) for a in (B, X, Y))
        Bd, Xd, Yd = (torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16) for a in (B, X, Y))
    else:
        Bd, Xd, Yd = (torch.from_numpy(a).cuda() for a in (B, X, Y))
    Cd = torch.empty((A.M, N), dtype=torch.float32, device="cuda")
    od = torch.empty(A.nnz, dtype=torch.float32, device="cuda")

    def step():
        plan.spmm(Bd, out=Cd)
        plan.sddmm(Xd, Yd, out=od)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps
    # Per-operator durations: a fixed number of further steps, the same at any --steps, with events on the launch stream
    # around each call (an event record keeps the next kernel from starting until the previous one has retired, about 5 us
    # of idle GPU each on this machine, so these steps stay out of the timed region).
    n_ev = 48
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_ev)]
    for e in ev:
        e[0].record()
        plan.spmm(Bd, out=Cd)
        e[1].record()
        plan.sddmm(Xd, Yd, out=od)
        e[2].record()
    torch.cuda.synchronize()
    spmm_ms = np.array([e[0].elapsed_time(e[1]) for e in ev[8:]])
    sddmm_ms = np.array([e[1].elapsed_time(e[2]) for e in ev[8:]])

    # Cold calls (a 1 GiB buffer is streamed between calls, which evicts L2 and the 256 MB Infinity Cache) and the
    # streaming-copy rate of this machine; both after the timed region, so they do not disturb it.
    gather = None
    if not args.no_probes and not f32:
        # the row fetches of the SpMM call and nothing else: rows col[p] of B in CSR order, 256 indices per wave
        sink = torch.zeros(1, dtype=torch.float32, device="cuda")
        rb = N * 2
        if rb in (64, 128, 256) and Bd.is_contiguous():
            stream = torch.cuda.current_stream().cuda_stream

            def probe_us(call):
                gev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(12)]
                for e in gev:
                    e[0].record()
                    call()
                    e[1].record()
                torch.cuda.synchronize()
                return float(np.median([e[0].elapsed_time(e[1]) for e in gev[2:]])) * 1e3

            g_us = probe_us(lambda: lb.libra_probe_gather(Bd.data_ptr(), A.Kc, rb, col_d.data_ptr(), A.nnz, sink.data_ptr(), stream))
            gather = {"rows": A.nnz, "row_bytes": rb, "median_us": round(g_us, 2), "GBs": round(A.nnz * rb / g_us / 1e3, 1)}
            # the same number of fetches from the first 4 MiB of the operand only (every fetch hits in an L2): what the
            # L2 -> L1 path alone allows
            hit_rows = max(1, min(A.Kc, (4 << 20) // rb))
            col_hit = col_d % hit_rows
            h_us = probe_us(lambda: lb.libra_probe_gather(Bd.data_ptr(), A.Kc, rb, col_hit.data_ptr(), A.nnz, sink.data_ptr(), stream))
            gather["all_l2_hits_us"] = round(h_us, 2)
            del col_hit
            # ... and with the most referenced rows (96 KB of them) resident in LDS, persistent workgroups
            if A.Kc * rb < (1 << 32) - 16:
                n_hub = min(A.Kc, (96 << 10) // rb)
                popularity = np.bincount(A.col, minlength=A.Kc)
                hub_rows = np.argsort(-popularity, kind="stable")[:n_hub].astype(np.int32)
                slot = np.full(A.Kc, -1, dtype=np.int64)
                slot[hub_rows] = np.arange(n_hub)
                s_of = slot[A.col]
                enc = torch.from_numpy(np.where(s_of >= 0, -1 - s_of, A.col).astype(np.int32)).cuda()
                hub_d = torch.from_numpy(hub_rows).cuda()
                p_us = probe_us(lambda: lb.libra_probe_gather_hub(Bd.data_ptr(), A.Kc, rb, col_d.data_ptr(), A.nnz, hub_d.data_ptr(), 0, sink.data_ptr(), stream))
                l_us = probe_us(lambda: lb.libra_probe_gather_hub(Bd.data_ptr(), A.Kc, rb, enc.data_ptr(), A.nnz, hub_d.data_ptr(), n_hub, sink.data_ptr(), stream))
                gather["hub_rows_in_lds"] = {"rows_in_lds": int(n_hub), "share_of_fetches": round(float((s_of >= 0).mean()), 4),
                                             "persistent_no_hub_us": round(p_us, 2), "persistent_hub_us": round(l_us, 2)}
                del enc, hub_d
    scratch = torch.zeros(1 << 28 if not args.no_probes else 1 << 10, dtype=torch.float32, device="cuda")
    n_cold = 15 if not args.no_probes else 3
    cev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_cold)]
    for i in range(n_cold):
        scratch.add_(1.0)
        cev[i][0].record()
        plan.spmm(Bd, out=Cd)
        cev[i][1].record()
        scratch.add_(1.0)
        cev[i][2].record()
        plan.sddmm(Xd, Yd, out=od)
        cev[i][3].record()
    torch.cuda.synchronize()
    spmm_cold = np.array([e[0].elapsed_time(e[1]) for e in cev[2:]])
    sddmm_cold = np.array([e[2].elapsed_time(e[3]) for e in cev[2:]])
    dst = torch.empty_like(scratch)
    kev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(8)]
    for i in range(8):
        kev[i][0].record()
        dst.copy_(scratch)
        kev[i][1].record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * scratch.numel() * 4 / (float(np.median([e[0].elapsed_time(e[1]) for e in kev[2:]])) * 1e-3) / 1e9
    del scratch, dst

    flops_spmm = 2.0 * A.nnz * N
    flops_sddmm = 2.0 * A.nnz * K
    value = (flops_spmm + flops_sddmm) / (ms_per_step * 1e-3) / 1e9

    kref = int(np.unique(A.col).size)
    mref = int((np.diff(A.rowptr) > 0).sum())
    bytes_spmm = spmm_algorithmic_bytes(A, N, kref, es)
    bytes_sddmm = sddmm_algorithmic_bytes(A, K, mref, kref, es)
    spmm_avg_s = float(spmm_ms.mean()) * 1e-3
    achieved = bytes_spmm / spmm_avg_s / 1e9
    default_cfg = (not args.small and args.dtype == "f16" and args.mode == 0 and not (args.tau_spmm or args.tau_sddmm or args.ts or args.cs)
                   and not args.natural_order and not args.xcd_order and not args.no_xcd_order
                   and not args.segments_by_cost and not args.two_kernels)
    traffic = measured_traffic(f"{args.workload}:N={N}:{args.dtype}") if default_cfg and not args.no_tuned else None
    spmm_fetch_gbs = st["spmm_gather_rows"] * N * es / spmm_avg_s / 1e9          # rows of B the plan fetches (Eq. 2) per second

    out = {
        "metric": "SpMM/SDDMM effective GFLOP/s (2*nnz*N + 2*nnz*K per step)",
        "value": round(value, 1),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": f"{args.dtype} (f32 accumulate)",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}{'-small' if args.small else ''}: M={A.M} nnz={A.nnz} SpMM N={N} + SDDMM K={K}",
                   "M": A.M, "nnz": A.nnz, "N": N, "K": K, "mode": args.mode,
                   "options": "tuner table" if tuned else "library defaults"},
        "roofline": {"bound": "hbm", "kernel": f"spmm_task_kernel<{args.dtype},{min(N, 256)}>", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "algorithmic_bytes": bytes_spmm, "avg_us": round(spmm_avg_s * 1e6, 2),
                     "frac_of_measured_copy": round(achieved / copy_gbs, 4), "measured_copy_GBs": round(copy_gbs, 1),
                     "modelled_gather_GBs": round((st["spmm_gather_rows"] * N * 2 + A.nnz * 6 + A.M * N * 4)
                                                  / spmm_avg_s / 1e9, 1),
                     "row_fetch_GBs": round(spmm_fetch_gbs, 1),
                     "frac_of_measured_gather": round(spmm_fetch_gbs / gather["GBs"], 4) if gather else None},
        "gather_probe": gather,
        "spmm": {"gflops": round(flops_spmm / spmm_avg_s / 1e9, 1), "median_us": round(float(np.median(spmm_ms)) * 1e3, 2),
                 "min_us": round(float(spmm_ms.min()) * 1e3, 2), "cold_median_us": round(float(np.median(spmm_cold)) * 1e3, 2),
                 "bytes": bytes_spmm},
        "sddmm": {"gflops": round(flops_sddmm / (float(sddmm_ms.mean()) * 1e-3) / 1e9, 1),
                  "median_us": round(float(np.median(sddmm_ms)) * 1e3, 2), "min_us": round(float(sddmm_ms.min()) * 1e3, 2),
                  "cold_median_us": round(float(np.median(sddmm_cold)) * 1e3, 2), "bytes": bytes_sddmm,
                  "hbm_frac": round(bytes_sddmm / (float(sddmm_ms.mean()) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "plan": {"used": "host planner + upload" if args.host_plan else "device planner (resident)",
                 "host_plan_s": round(plan_s, 4), "host_upload_s": round(upload_s, 4),
                 "device_plan_s": round(min(dev_s[1:]), 5), "device_passes_s": round(ds["device_seconds"], 5),
                 "spmm_dense_share": round(st["spmm_dense_nnz"] / max(A.nnz, 1), 4),
                 "sddmm_dense_share": round(st["sddmm_dense_nnz"] / max(A.nnz, 1), 4),
                 "nnz1_vector_ratio": round(st["n_vectors_nnz1"] / max(st["n_vectors"], 1), 4),
                 "spmm_tasks": st["spmm_tasks"], "spmm_chunk_tasks": st["spmm_chunk_tasks"],
                 "spmm_gather_rows": st["spmm_gather_rows"], "neighbour_share": round(st["neighbour_share"], 3),
                 "xcd_order": st["xcd_order"]},
    }

    if args.workload == "gat" and N == K and args.dtype == "f16":
        # the attention head of this configuration as a whole: scores (SDDMM) -> row softmax -> new values into the SpMM
        # arrays -> aggregation (SpMM with B = Y); outside the timed region, the plan's values are restored afterwards
        alpha = torch.empty(A.nnz, dtype=torch.float16, device="cuda")
        scale = 1.0 / float(np.sqrt(K))

        def timed(fn, reps=12):
            for _ in range(3):
                fn()
            es = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(reps)]
            for e in es:
                e[0].record()
                fn()
                e[1].record()
            torch.cuda.synchronize()
            return round(float(np.median([e[0].elapsed_time(e[1]) for e in es])) * 1e3, 1)

        def head():
            plan.sddmm(Xd, Yd, out=od)
            plan.edge_softmax(od, scale, out=alpha)
            plan.set_values(alpha, lb.OP_SPMM)
            plan.spmm(Yd, out=Cd)

        out["attention_head"] = {"softmax_us": timed(lambda: plan.edge_softmax(od, scale, out=alpha)),
                                 "new_values_us": timed(lambda: plan.set_values(alpha, lb.OP_SPMM)),
                                 "head_us": timed(head)}
        plan.set_values(torch.from_numpy(A.val).cuda(), lb.OP_SPMM)

    if not args.no_cpu_baseline:
        import oracle
        nt = oracle.max_threads()
        t0 = time.perf_counter()
        oracle.spmm(A.rowptr, A.col, A.val if val is None else val, B, want_scale=False, bf16=bf16)
        t_sp = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.sddmm(A.rowptr, A.col, A.val if val is None else val, X, Y, want_scale=False, bf16=bf16)
        t_sd = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.spmm(A.rowptr, A.col, A.val if val is None else val, B, want_scale=False, bf16=bf16, nthreads=1)
        oracle.sddmm(A.rowptr, A.col, A.val if val is None else val, X, Y, want_scale=False, bf16=bf16, nthreads=1)
        t_one = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round((flops_spmm + flops_sddmm) / (t_sp + t_sd) / 1e9, 2), "unit": "GFLOP/s",
                               "cores": nt, "kind": "oracle",
                               "sample": f"the whole workload once (SpMM {t_sp:.2f} s + SDDMM {t_sd:.2f} s)",
                               "one_thread_value": round((flops_spmm + flops_sddmm) / t_one / 1e9, 2)}
    print(json.dumps(out))
    plan.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
