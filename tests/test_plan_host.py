"""Host-side tests of the product library (no GPU): it loads, exports every
symbol the header declares, validates its input, and its planner output is
bit-identical to the reference planner's."""
import os
import re

import numpy as np
import pytest

from oracle import planner_ref as pr
from paper_2506_22714_amd import binding as lb
from paper_2506_22714_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol(built_library):
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(libra_[a-z_]+)\s*\(", text))
    assert {"libra_plan", "libra_spmm", "libra_sddmm", "libra_plan_upload", "libra_edge_softmax"} <= names
    for n in sorted(names):
        assert hasattr(built_library, n), n
    assert lb.libra_version() == 1
    assert "NULL" in lb.strerror(-1) and lb.strerror(0) == "ok"


# ----------------------------------------------------------------- validation
def _plan_rc(M, Kc, rowptr, col, val, opts=None, dtype=None):
    import ctypes as C
    h = C.c_void_p()
    rowptr = None if rowptr is None else np.ascontiguousarray(rowptr, dtype=np.int32)
    col = None if col is None else np.ascontiguousarray(col, dtype=np.int32)
    val = None if val is None else np.ascontiguousarray(val)
    rc = lb.lib().libra_plan(M, Kc, lb._np_ptr(rowptr), lb._np_ptr(col), lb._np_ptr(val),
                             lb.F16 if dtype is None else dtype, C.byref(opts) if opts else None, C.byref(h))
    if rc == 0:
        lb.libra_plan_destroy(h)
    return rc


def test_invalid_inputs_are_rejected_with_codes():
    rp = np.array([0, 2, 3], dtype=np.int32)
    col = np.array([0, 2, 1], dtype=np.int32)
    val = np.ones(3, dtype=np.float16)
    assert _plan_rc(2, 3, rp, col, val) == 0
    assert _plan_rc(2, 3, None, col, val) == lb.ERR["NULL"]
    assert _plan_rc(2, 3, rp, None, val) == lb.ERR["NULL"]
    assert _plan_rc(0, 3, rp, col, val) == lb.ERR["SHAPE"]
    assert _plan_rc(2, 0, rp, col, val) == lb.ERR["SHAPE"]
    assert _plan_rc(2, 3, np.array([1, 2, 3]), col, val) == lb.ERR["ROWPTR"]
    assert _plan_rc(2, 3, np.array([0, 3, 2]), col, val) == lb.ERR["ROWPTR"]
    assert _plan_rc(2, 2, rp, col, val) == lb.ERR["COLUMN"]
    assert _plan_rc(2, 3, rp, np.array([0, -1, 1]), val) == lb.ERR["COLUMN"]
    assert _plan_rc(2, 3, rp, np.array([2, 0, 1]), val) == lb.ERR["UNSORTED"]
    assert _plan_rc(2, 3, rp, np.array([1, 1, 1]), val) == lb.ERR["UNSORTED"]       # duplicate
    assert _plan_rc(2, 3, rp, col, val, dtype=7) == lb.ERR["DTYPE"]
    assert _plan_rc(2, 3, rp, col, val.view(np.uint16), dtype=lb.BF16) == 0
    assert _plan_rc(2, 3, rp, col, val, opts=lb.PlanOpts(window_rows=33)) == lb.ERR["OPTION"]
    assert _plan_rc(2, 3, rp, col, val, opts=lb.PlanOpts(mode=5)) == lb.ERR["OPTION"]
    assert _plan_rc(2, 3, rp, col, val, opts=lb.PlanOpts(sddmm_min_dense_pct=101)) == lb.ERR["OPTION"]
    assert _plan_rc(2, 3, rp, col, val, opts=lb.PlanOpts(sddmm_min_dense_pct=-1)) == lb.ERR["OPTION"]
    bad = lb.PlanOpts()
    bad.struct_size = 8
    assert _plan_rc(2, 3, rp, col, val, opts=bad) == lb.ERR["OPTION"]
    # an empty matrix (no nonzeros) is valid
    assert _plan_rc(3, 3, np.zeros(4, dtype=np.int32), None, None) == 0


def test_gather_probes_check_their_arguments_before_any_launch():
    """The measurement aids refuse bad arguments on the host: nothing here reaches the GPU."""
    import ctypes as C
    L = lb.lib()
    null, some = C.c_void_p(0), C.c_void_p(256)           # `some`: a non-null, 16-byte aligned value that is never dereferenced
    assert L.libra_probe_gather(null, 10, 256, some, 5, some, null) == lb.ERR["NULL"]
    assert L.libra_probe_gather(some, 10, 96, some, 5, some, null) == lb.ERR["UNSUPPORTED"]
    assert L.libra_probe_gather(some, 0, 256, some, 5, some, null) == lb.ERR["SHAPE"]
    assert L.libra_probe_gather_hub(null, 10, 256, some, 5, some, 2, some, null) == lb.ERR["NULL"]
    assert L.libra_probe_gather_hub(some, 10, 256, some, 5, null, 2, some, null) == lb.ERR["NULL"]          # hub rows announced, none given
    assert L.libra_probe_gather_hub(some, 10, 256, some, 0, some, 2, some, null) == lb.ERR["SHAPE"]
    assert L.libra_probe_gather_hub(some, 10, 256, some, 5, some, -1, some, null) == lb.ERR["SHAPE"]
    assert L.libra_probe_gather_hub(some, 10, 48, some, 5, some, 2, some, null) == lb.ERR["UNSUPPORTED"]
    assert L.libra_probe_gather_hub(C.c_void_p(264), 10, 256, some, 5, some, 2, some, null) == lb.ERR["BUFFER"]
    assert L.libra_probe_gather_hub(some, 10, 256, some, 5, some, 513, some, null) == lb.ERR["TOO_LARGE"]    # 513 rows of 256 bytes > 128 KB of LDS
    assert L.libra_probe_gather_hub(some, 1 << 24, 256, some, 5, some, 2, some, null) == lb.ERR["TOO_LARGE"]  # table of 4 GiB


def test_compute_calls_without_device_copy_fail_cleanly():
    A = wl.random_pattern(40, 40, 0.1, seed=1)
    p = lb.Plan.from_csr(A)
    with pytest.raises(lb.LibraError) as e:
        lb.libra_spmm(p.handle, 256, 32, 32, 512, 32)
    assert e.value.code == lb.ERR["NOT_UPLOADED"]
    with pytest.raises(lb.LibraError) as e:
        lb.libra_spmm(p.handle, 0, 32, 32, 512, 32)
    assert e.value.code == lb.ERR["NULL"]
    with pytest.raises(lb.LibraError) as e:
        lb.libra_plan_upload(p.handle, 128, 10)
    assert e.value.code == lb.ERR["BUFFER"]
    p2 = lb.Plan.from_csr(A, flags=lb.FLAG_NO_SDDMM)
    with pytest.raises(lb.LibraError) as e:
        lb.libra_sddmm(p2.handle, 256, 256, 32, 256)
    assert e.value.code == lb.ERR["NOT_BUILT"]
    with pytest.raises(lb.LibraError) as e:
        p2.export(1)
    assert e.value.code == lb.ERR["NOT_BUILT"]
    assert lb.libra_plan_device_bytes(p.handle) > 0


# ------------------------------------------------- plan == reference planner
def is_empty_task(t):
    """Filler of the die-aware order: no blocks, no entries, no output rows."""
    return t["blk_begin"] == t["blk_end"] and t["res_begin"] == t["res_end"] and t["atomic_mask"] == 0 and t["store_mask"] == 0


def canon_tasks(tasks):
    tasks = [t for t in tasks if not is_empty_task(t)]
    return sorted((int(t["kind"]), int(t["id"]), int(t["blk_begin"]), int(t["blk_end"]), int(t["res_begin"]),
                   int(t["res_end"]), int(t["scalar_mask"]), int(t["atomic_mask"]), int(t["store_mask"])) for t in tasks)


def check_subplan(A: wl.Csr, ex: dict, ref: pr.SubPlan, spmm: bool):
    assert list(ex["win_blkptr"]) == ref.win_blkptr
    assert ex["n_blocks"] == len(ref.blocks)
    if ref.blocks:
        assert np.array_equal(ex["blk_cols"], np.array([b.cols for b in ref.blocks], dtype=np.int32))
        assert np.array_equal(ex["blk_bitmap"], np.array([b.bitmap for b in ref.blocks], dtype=np.uint64))
    assert list(ex["blk_valptr"]) == list(np.cumsum([0] + [b.nnz for b in ref.blocks]))
    ref_dense_perm = [p for b in ref.blocks for p in b.perm]
    assert list(ex["dense_perm"]) == ref_dense_perm
    assert list(ex["res_perm"]) == ref.res_perm
    # every nonzero exactly once, on exactly one path
    allp = np.concatenate([ex["dense_perm"], ex["res_perm"]])
    assert np.array_equal(np.sort(allp), np.arange(A.nnz))
    label = np.zeros(A.nnz, dtype=np.int8)
    label[ex["dense_perm"]] = 1
    assert np.array_equal(label, ref.label)
    # values and columns travel with their nonzero
    assert np.array_equal(ex["dense_val"], A.val[ex["dense_perm"]])
    assert np.array_equal(ex["res_val"], A.val[ex["res_perm"]])
    assert np.array_equal(ex["res_col"], A.col[ex["res_perm"]])
    # bitmap popcounts equal block nnz
    pc = [sum(bin(int(w)).count("1") for w in row) for row in ex["blk_bitmap"]]
    assert pc == list(np.diff(ex["blk_valptr"]))
    rows = np.repeat(np.arange(A.M), np.diff(A.rowptr))
    assert np.array_equal(ex["res_row"], rows[ex["res_perm"]]) and list(ex["res_row"]) == ref.res_row
    if spmm:
        assert list(ex["win_resptr"]) == ref.win_resptr
        assert sorted(ex["zero_rows"]) == ref.zero_rows
    else:
        assert np.all(np.diff(ex["res_perm"]) > 0)
    # tasks that do nothing (the die-aware order adds some; a window whose rows are all decomposed is one) are not compared
    assert canon_tasks(ex["tasks"]) == sorted(t for t in ref.tasks if not (t[2] == t[3] and t[4] == t[5] and t[7] == 0 and t[8] == 0))


CASES = [
    dict(),                                                     # defaults
    dict(spmm_min_vec_nnz=3, sddmm_min_blk_nnz=20, ts=2, cs=7, sddmm_cs=33, sddmm_ts=3),
    dict(mode=lb.MODE_DENSE_ONLY, ts=3, sddmm_ts=1),
    dict(mode=lb.MODE_SCALAR_ONLY, cs=5),
    dict(flags=lb.FLAG_NO_FILL_PADDING, ts=1, cs=3),
    dict(window_rows=4, block_cols=4, spmm_min_vec_nnz=2, sddmm_min_blk_nnz=4, ts=2, cs=5, short_len=2),
    dict(window_rows=8, block_cols=16, sddmm_min_blk_nnz=24, spmm_min_vec_nnz=3, ts=4, cs=16),
    dict(window_rows=32, block_cols=64, ts=1, cs=9),
    dict(flags=lb.FLAG_NATURAL_ORDER, ts=2, cs=6),
    dict(sddmm_min_blk_nnz=20, sddmm_min_dense_pct=30),         # the dense-share rule: fires on some of the matrices
    dict(sddmm_min_blk_nnz=20, sddmm_min_dense_pct=85),
]


def ref_opts(kw: dict) -> pr.Opts:
    fl = kw.get("flags", 0)
    return pr.Opts(mode=kw.get("mode", 0), W=kw.get("window_rows", 16), KB=kw.get("block_cols", 16),
                   tau_spmm=kw.get("spmm_min_vec_nnz", 3), tau_sddmm=kw.get("sddmm_min_blk_nnz", 64),
                   Ts=kw.get("ts", 16), Cs=kw.get("cs", 128), short_len=kw.get("short_len", 3),
                   fill_padding=not (fl & lb.FLAG_NO_FILL_PADDING), sddmm_Cs=kw.get("sddmm_cs", 128),
                   sddmm_Ts=kw.get("sddmm_ts", 4), sddmm_min_dense_pct=kw.get("sddmm_min_dense_pct", 0))


def matrices():
    yield "random", wl.random_pattern(203, 150, 0.08, seed=5, empty_rows=0.15)
    yield "community", wl.community(n_blocks=6, seed=2)
    yield "rmat", wl.rmat(scale=9, avg_degree=8, seed=3)
    yield "longrows", wl.with_long_rows(wl.random_pattern(90, 400, 0.03, seed=7), [3, 17, 18, 64], 300, seed=8)
    yield "single_row", wl.random_pattern(1, 50, 0.5, seed=9)
    # more window ranges than windows can fill near the tail: M not a multiple of the window height
    yield "ragged_tail", wl.random_pattern(1000, 300, 0.03, seed=10, empty_rows=0.3)


@pytest.mark.parametrize("case", range(len(CASES)))
def test_planner_matches_reference_bit_for_bit(case):
    kw = CASES[case]
    for name, A in matrices():
        p = lb.Plan.from_csr(A, threads=8, **kw)
        o = ref_opts(kw)
        check_subplan(A, p.export(0), pr.plan_spmm(A.M, A.rowptr, A.col, o), spmm=True)
        check_subplan(A, p.export(1), pr.plan_sddmm(A.M, A.rowptr, A.col, o), spmm=False)
        st = p.stats()
        ref = pr.plan_spmm(A.M, A.rowptr, A.col, o)
        assert st["n_vectors"] == ref.stats["n_vectors"] and st["n_vectors_nnz1"] == ref.stats["n_vectors_nnz1"]
        assert st["spmm_dense_vectors"] == ref.stats["n_dense_vectors"] and st["spmm_pad_slots"] == ref.stats["n_pad_slots"]
        assert (st["spmm_short_rows"], st["spmm_long_rows"], st["spmm_split_rows"]) == (ref.n_short_rows, ref.n_long_rows, ref.n_split_rows)
        # Eq. 2 summed over the plan: rows of B fetched = dense vectors + residual nonzeros <= nnz
        assert st["spmm_gather_rows"] == st["spmm_dense_vectors"] + st["spmm_res_nnz"] <= max(A.nnz, st["spmm_gather_rows"])
        p.close()


def test_plan_does_not_depend_on_thread_count_and_orders_heaviest_first():
    A = wl.rmat(scale=11, avg_degree=8, seed=4)
    plain = lb.FLAG_NO_XCD_ORDER | lb.FLAG_SEGMENTS_BY_COST
    e1 = lb.Plan.from_csr(A, threads=1, cs=16, ts=2, flags=plain).export(0)
    e7 = lb.Plan.from_csr(A, threads=7, cs=16, ts=2, flags=plain).export(0)
    for k in e1:
        assert np.array_equal(e1[k], e7[k]), k
    a1, a7 = (lb.Plan.from_csr(A, threads=t, cs=16, ts=2).export(0) for t in (1, 7))       # order decided from the matrix
    assert np.array_equal(a1["tasks"], a7["tasks"])
    cost = e1["tasks"]["cost"].astype(np.int64)
    assert np.all(np.diff(cost) <= 0)
    nat = lb.Plan.from_csr(A, cs=16, ts=2, flags=lb.FLAG_NATURAL_ORDER).export(0)
    assert canon_tasks(nat["tasks"]) == canon_tasks(e1["tasks"])
    win = nat["tasks"]["id"][nat["tasks"]["kind"] == lb.TASK_WINDOW]
    assert np.all(np.diff(win) >= 0)


def test_fp32_values_plan_like_16_bit_values_and_are_carried_whole():
    """The split rule looks at the pattern only: fp32 values give the same blocks, bitmaps and tasks as fp16 ones (the dense
    tiles then run on the fp32 matrix instruction), and every value arrives unrounded on its path."""
    A = wl.make("community", small=True)
    v32 = (A.val.astype(np.float32) * np.float32(1.0009765625) + np.float32(1e-4)).astype(np.float32)   # not fp16 numbers
    p16, p32 = lb.Plan.from_csr(A), lb.Plan.from_csr(A, val=v32)
    st = p32.stats()
    assert st["spmm_dense_nnz"] > 0 and st["sddmm_dense_nnz"] > 0 and st["spmm_res_nnz"] > 0
    for which in (0, 1):
        a, b = p16.export(which), p32.export(which)
        for k in ("tasks", "blk_cols", "blk_bitmap", "blk_valptr", "dense_perm", "res_perm", "res_row", "res_col"):
            assert np.array_equal(a[k], b[k]), (which, k)
        assert b["dense_val"].dtype == np.float32 and b["res_val"].dtype == np.float32
        assert np.array_equal(b["dense_val"], v32[b["dense_perm"]]) and np.array_equal(b["res_val"], v32[b["res_perm"]])
    sc = lb.Plan.from_csr(A, val=v32, mode=lb.MODE_SCALAR_ONLY).stats()
    assert sc["spmm_dense_nnz"] == 0 and sc["sddmm_dense_nnz"] == 0 and sc["spmm_res_nnz"] == A.nnz


def test_bfloat16_plan_has_the_same_structure_and_carries_the_bits():
    """The storage type only changes how the 16 value bits are read: same pattern, same plan, bits copied."""
    A = wl.make("powerlaw", small=True)
    bits = wl.to_bf16_bits(np.linspace(-3.0, 3.0, A.nnz, dtype=np.float32) + 0.01)
    pf = lb.Plan.from_csr(A, val=bits.view(np.float16))
    pb = lb.Plan.from_csr(A, val=bits, val_dtype=lb.BF16)
    for which in (0, 1):
        ef, eb = pf.export(which), pb.export(which)
        for k in ("blk_cols", "blk_bitmap", "blk_valptr", "dense_perm", "res_row", "res_col", "res_perm", "zero_rows"):
            assert np.array_equal(ef[k], eb[k]), k
        assert np.array_equal(ef["tasks"], eb["tasks"])
        assert np.array_equal(eb["dense_val"], bits[eb["dense_perm"]])
        assert np.array_equal(eb["res_val"], bits[eb["res_perm"]])
    pf.close()
    pb.close()


def test_xcd_order_keeps_the_tasks_and_puts_neighbouring_windows_on_one_die():
    A = wl.community(n_blocks=64, seed=3)
    for which in (0, 1):
        base = lb.Plan.from_csr(A, flags=lb.FLAG_NO_XCD_ORDER).export(which)["tasks"]
        auto = lb.Plan.from_csr(A)
        assert auto.stats()["xcd_order"] == 1 and auto.stats()["neighbour_share"] < 0.6      # diagonal blocks: decided from the matrix
        grp = auto.export(which)["tasks"]
        assert np.array_equal(grp, lb.Plan.from_csr(A, flags=lb.FLAG_XCD_ORDER).export(which)["tasks"])
        empty = np.array([bool(is_empty_task(t)) for t in grp])
        assert canon_tasks(grp[~empty]) == canon_tasks(base)           # same work, a few empty tasks added
        assert empty.sum() <= 8 * 64 and not empty[-1]
        # the four windows of a group sit in one residue class modulo 8 (= one die), next to each other
        pos = {}
        for k, t in enumerate(grp):
            if not empty[k] and t["kind"] == lb.TASK_WINDOW:
                pos.setdefault(int(t["id"]) // 4, []).append(k)
        for g, ks in pos.items():
            assert len({k % 8 for k in ks}) == 1, g
            assert max(ks) - min(ks) == 8 * (len(ks) - 1), g


def test_segments_by_column_keeps_the_tasks_and_gives_each_die_one_column_range():
    A = wl.rmat(scale=12, avg_degree=24, seed=6)
    base = lb.Plan.from_csr(A, cs=16, flags=lb.FLAG_NO_XCD_ORDER | lb.FLAG_SEGMENTS_BY_COST)
    plan = lb.Plan.from_csr(A, cs=16, flags=lb.FLAG_NO_XCD_ORDER)
    asked = lb.Plan.from_csr(A, cs=16, flags=lb.FLAG_NO_XCD_ORDER | lb.FLAG_SEGMENTS_BY_COLUMN)
    assert np.array_equal(asked.export(0)["tasks"], plan.export(0)["tasks"])          # the flag names the default
    ex = plan.export(0)
    t = ex["tasks"]
    assert canon_tasks(t) == canon_tasks(base.export(0)["tasks"])
    assert sum(bool(is_empty_task(x)) for x in t) <= 8
    first_col = np.array([ex["res_col"][x["res_begin"]] if x["kind"] == lb.TASK_CHUNK else -1 for x in t])
    seg = t["kind"] == lb.TASK_CHUNK
    assert seg.sum() > 200
    med = [np.median(first_col[q::8][seg[q::8]]) for q in range(8)]
    assert all(med[q] < med[q + 1] for q in range(7))              # column ranges ascend from die to die
    for q in range(7):                              # (light tasks moved to level the queues may stray)
        assert (first_col[q::8][seg[q::8]] > med[q + 1]).mean() <= 0.2
    for q in range(8):                              # and a die meets its segments in ascending column order
        c = first_col[q::8][seg[q::8]]
        assert (np.diff(c) < 0).sum() <= 0.1 * c.size


def test_binding_rejects_operands_of_the_wrong_size_before_any_launch():
    """The C ABI takes pointers; the wrapper is the only place that sees the sizes behind them.  Every mismatch raises
    ValueError before a kernel could read or write past an operand's end (no GPU is needed to see that)."""
    torch = pytest.importorskip("torch")
    A = wl.random_pattern(40, 56, 0.2, seed=3)
    p = lb.Plan.from_csr(A)
    h = torch.float16
    ok_B = torch.zeros((A.Kc, 32), dtype=h)

    def rejected(call, what):
        with pytest.raises(ValueError, match=what):
            call()

    # well-formed operands pass every size check and stop at the last one: they are not on a GPU
    rejected(lambda: p.spmm(ok_B), "B: must be a GPU tensor")
    rejected(lambda: p.spmm(torch.zeros((A.Kc - 1, 32), dtype=h)), "B: shape")
    rejected(lambda: p.spmm(torch.zeros((A.Kc, 32), dtype=torch.float32)), "B: dtype")
    rejected(lambda: p.spmm(torch.zeros((A.Kc * 32,), dtype=h)), "B: shape")
    rejected(lambda: p.spmm(torch.zeros((32, A.Kc), dtype=h).t()), "B: rows must be contiguous")
    rejected(lambda: p.spmm(ok_B, out=torch.zeros((A.M - 1, 32))), "B: must be a GPU")      # B is checked first
    rejected(lambda: p.sddmm(torch.zeros((A.M + 1, 32), dtype=h), torch.zeros((A.Kc, 32), dtype=h)), "X: shape")
    rejected(lambda: p.sddmm(torch.zeros((A.M, 32), dtype=h), torch.zeros((A.Kc - 1, 32), dtype=h)), "X: must be a GPU")
    rejected(lambda: p.edge_softmax(torch.zeros(A.nnz - 1), 1.0), "scores: .* elements")
    rejected(lambda: p.edge_softmax(torch.zeros(A.nnz, dtype=torch.float64), 1.0), "scores: dtype")
    rejected(lambda: p.edge_softmax_backward(torch.zeros(A.nnz + 1, dtype=h), torch.zeros(A.nnz), 1.0), "alpha: .* elements")
    rejected(lambda: p.edge_softmax_backward(torch.zeros(A.nnz, dtype=torch.int32), torch.zeros(A.nnz), 1.0), "alpha: dtype")
    rejected(lambda: p.set_values(torch.zeros(A.nnz - 1, dtype=h)), "vals: .* elements")
    rejected(lambda: p.set_values(torch.zeros(A.nnz, dtype=torch.float32)), "vals: dtype")
    rejected(lambda: lb.Plan.from_device_csr(A.M, A.Kc, torch.zeros(A.M, dtype=torch.int32), torch.zeros(3, dtype=torch.int32),
                                             torch.zeros(3, dtype=h)), "rowptr: .* elements")
    rejected(lambda: lb.transpose_csr(A.M, A.Kc, torch.zeros(A.M + 1, dtype=torch.int64), torch.zeros(3, dtype=torch.int32)), "rowptr: expected")
    p.close()


def test_locality_model_counts_fetches_and_compulsory_misses():
    """The L2 replay of a plan's task table: every fetch of Eq. 2 is counted once, an unbounded cache misses exactly the
    distinct rows of each die, and a smaller cache never misses less."""
    from paper_2506_22714_amd import locality
    A = wl.make("powerlaw", small=True)
    p = lb.Plan.from_csr(A, ts=32, cs=128, spmm_min_vec_nnz=3)
    e = p.export(0)
    cols = locality.task_columns(e)
    st = p.stats()
    assert sum(len(c) for c in cols) == st["spmm_gather_rows"]
    per_die = sum(len(np.unique(np.concatenate([cols[i] for i in range(d, len(cols), 8)] + [np.zeros(0, np.int32)]))) for d in range(8))
    big = locality.replay(cols, e["tasks"]["kind"], 1 << 40)
    assert sum(big["fetches"].values()) == st["spmm_gather_rows"]
    assert sum(big["misses"].values()) == per_die == big["distinct_rows_summed_over_dies"]
    small = locality.replay(cols, e["tasks"]["kind"], 64)
    tiny = locality.replay(cols, e["tasks"]["kind"], 1)
    assert sum(big["misses"].values()) <= sum(small["misses"].values()) <= sum(tiny["misses"].values()) <= st["spmm_gather_rows"]
    p.close()
