"""The threshold tuner (Section 4.2.2: the utilisation threshold depends on the architecture and is found once per GPU by a
sweep over representative matrices; Section 5.3.3): the search, the table it writes, and how a plan takes its options
from the table."""
import json

import numpy as np
import pytest

from paper_2506_22714_amd import binding as lb
from paper_2506_22714_amd import tune
from paper_2506_22714_amd import workloads as wl


def _table(spmm_opts, sddmm_opts):
    entry = lambda o: {"options": o, "geomean_us": 1.0, "defaults_geomean_us": 2.0, "settings_tried": 3}
    return {"format": "libra-tuned-1", "device": "test", "small_workloads": True, "workloads": [], "objective": "",
            "spmm": {"f16": {c: entry(spmm_opts[c]) for c in tune.N_CLASSES}},
            "sddmm": {"f16": {c: entry(sddmm_opts[c]) for c in tune.K_CLASSES}}}


def test_coordinate_descent_finds_the_grid_minimum_and_counts_each_setting_once():
    calls = []

    def cost(s):
        calls.append(dict(s))
        return 10.0 + (s["a"] - 3) ** 2 + 0.5 * (s["b"] - 20) ** 2 / 100 + (0.3 if s["a"] == 4 and s["b"] == 30 else 0)

    best, c, seen = tune.coordinate_descent([("a", (1, 2, 3, 4)), ("b", (10, 20, 30))], dict(a=1, b=10), cost, log=lambda *_: None)
    assert best == dict(a=3, b=20) and c == 10.0
    assert len(calls) == len(seen) == len({tuple(sorted(s.items())) for s in calls})        # nothing is timed twice
    # a change worth less than half a percent does not move the setting
    best, c, _ = tune.coordinate_descent([("a", (1, 2))], dict(a=1), lambda s: 100.0 - 0.2 * (s["a"] == 2), log=lambda *_: None)
    assert best == dict(a=1)


def test_width_classes():
    assert [tune.n_class(n) for n in (16, 32, 33, 64, 96, 128, 512)] == ["n32", "n32", "n64", "n64", "n128", "n128", "n128"]
    assert [tune.k_class(k) for k in (32, 64, 128)] == ["k32", "k64", "k128"]
    assert tune.geomean([2.0, 8.0]) == pytest.approx(4.0)


def test_table_is_parsed_checked_and_applied_to_a_plan(tmp_path):
    t = _table({"n32": dict(spmm_min_vec_nnz=2, ts=8, cs=64), "n64": dict(spmm_min_vec_nnz=4, ts=16, cs=128),
                "n128": dict(spmm_min_vec_nnz=6, ts=32, cs=256)},
               {"k32": dict(sddmm_min_blk_nnz=257, sddmm_cs=64, sddmm_ts=8), "k64": dict(sddmm_min_blk_nnz=32, sddmm_cs=128, sddmm_ts=2),
                "k128": dict(sddmm_min_blk_nnz=16, sddmm_cs=256, sddmm_ts=4)})
    path = tmp_path / "tuned.json"
    path.write_text(json.dumps(t))
    assert tune.tuned_options(str(path), "f16", N=128, K=32) == dict(spmm_min_vec_nnz=6, ts=32, cs=256, sddmm_min_blk_nnz=257, sddmm_cs=64, sddmm_ts=8)
    assert tune.tuned_options(t, "bf16", N=48) == dict(spmm_min_vec_nnz=4, ts=16, cs=128)        # bfloat16 -> float16 entries; no K: no SDDMM options
    assert tune.tuned_options(t, "f32", K=64) == dict(sddmm_min_blk_nnz=32, sddmm_cs=128, sddmm_ts=2)       # a type without entries falls back
    with pytest.raises(ValueError):
        tune.load_table({"format": "something else"})
    bad = json.loads(json.dumps(t))
    bad["spmm"]["f16"]["n128"]["options"]["flags"] = 3
    with pytest.raises(ValueError):
        tune.tuned_options(bad, "f16", N=128)
    # a plan built with the table equals the plan built with the same options spelled out; explicit options win
    A = wl.community(n_blocks=8, seed=4)
    a = lb.Plan.from_csr(A, tuned=str(path), N=128, K=64)
    b = lb.Plan.from_csr(A, spmm_min_vec_nnz=6, ts=32, cs=256, sddmm_min_blk_nnz=32, sddmm_cs=128, sddmm_ts=2)
    c = lb.Plan.from_csr(A, tuned=t, N=128, K=64, spmm_min_vec_nnz=2)
    d = lb.Plan.from_csr(A, spmm_min_vec_nnz=2, ts=32, cs=256, sddmm_min_blk_nnz=32, sddmm_cs=128, sddmm_ts=2)
    for x, y in ((a, b), (c, d)):
        for which in (0, 1):
            ex, ey = x.export(which), y.export(which)
            assert all(np.array_equal(ex[k], ey[k]) for k in ex)
    assert a.stats()["spmm_dense_nnz"] < c.stats()["spmm_dense_nnz"]
    for p in (a, b, c, d):
        p.close()


@pytest.mark.gpu
def test_tuner_emits_a_table_whose_plans_pass_parity(tmp_path):
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import oracle
    path = str(tmp_path / "tuned_small.json")
    lines = []
    table = tune.emit_table(path, small=True, dtypes=["f16"], log=lines.append)
    assert tune.load_table(path) == json.loads(json.dumps(table))
    for op, classes in (("spmm", tune.N_CLASSES), ("sddmm", tune.K_CLASSES)):
        for cls in classes:
            e = table[op]["f16"][cls]
            assert e["geomean_us"] <= e["defaults_geomean_us"] and e["settings_tried"] >= 5, (op, cls, e)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    for name, N, K in (("powerlaw", 128, 32), ("community", 64, 64), ("gat", 32, 128)):
        A = wl.make(name, small=True)
        B, X, Y = wl.dense_normal(A.Kc, N, seed=11), wl.dense_normal(A.M, K, seed=12), wl.dense_normal(A.Kc, K, seed=13)
        for planner in ("host", "device"):
            if planner == "host":
                p = lb.Plan.from_csr(A, tuned=path, N=N, K=K).upload()
            else:
                p = lb.Plan.from_device_csr(A.M, A.Kc, dev(A.rowptr.astype(np.int32)), dev(A.col.astype(np.int32)), dev(A.val),
                                            resident=True, tuned=table, N=N, K=K)
            C = p.spmm(dev(B)).cpu().numpy()
            out = p.sddmm(dev(X), dev(Y)).cpu().numpy()
            ref, S = oracle.spmm(A.rowptr, A.col, A.val, B)
            deg = np.diff(A.rowptr).astype(np.float64)
            assert oracle.graded_error(C, ref, S, deg[:, None]) <= min(1e-2, 16 * np.sqrt(max(deg.max(), 1)) * 2.0 ** -24)
            ref, S = oracle.sddmm(A.rowptr, A.col, A.val, X, Y)
            assert oracle.graded_error(out, ref, S, K) <= min(1e-2, 16 * np.sqrt(K) * 2.0 ** -24)
            p.close()
