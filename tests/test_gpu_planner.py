"""The device planner (the paper's GPU preprocessing, Section 4.5) against the host planner: the exported
plans must be identical array by array, for every option the kernels' window shape allows.  The host planner
itself is checked against the reference planner in the CPU tests, so equality here carries that parity over."""
import time

import numpy as np
import pytest

from paper_2506_22714_amd import binding as lb
from paper_2506_22714_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    lb.lib()


def dev_val(val, dtype_code):
    if dtype_code == lb.BF16:
        return torch.from_numpy(np.ascontiguousarray(val).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(val)).cuda()


def device_plan(A, val=None, val_dtype=None, **kw):
    v = A.val if val is None else val
    code = val_dtype if val_dtype is not None else (lb.F16 if v.dtype == np.float16 else lb.F32)
    return lb.Plan.from_device_csr(A.M, A.Kc, torch.from_numpy(A.rowptr.astype(np.int32)).cuda(),
                                   torch.from_numpy(A.col.astype(np.int32)).cuda(), dev_val(v, code), **kw)


TIMES = ("plan_seconds", "device_seconds")


def assert_same_plan(ph, pd, flags=0):
    sh, sd = ph.stats(), pd.stats()
    for k in sh:
        if k not in TIMES:
            assert sh[k] == sd[k], (k, sh[k], sd[k])
    assert sd["device_seconds"] > 0 and sh["device_seconds"] == 0
    for which in (0, 1):
        if flags & (lb.FLAG_NO_SPMM if which == 0 else lb.FLAG_NO_SDDMM):
            continue
        eh, ed = ph.export(which), pd.export(which)
        assert eh.keys() == ed.keys()
        for k in eh:
            assert np.array_equal(eh[k], ed[k]), (which, k)


CASES = [
    dict(),
    dict(spmm_min_vec_nnz=3, sddmm_min_blk_nnz=20, ts=2, cs=7, sddmm_cs=33, sddmm_ts=3),
    dict(spmm_min_vec_nnz=2, sddmm_min_blk_nnz=17, ts=1, cs=2, short_len=4),
    dict(mode=lb.MODE_DENSE_ONLY, ts=3, sddmm_ts=1),
    dict(mode=lb.MODE_SCALAR_ONLY, cs=5),
    dict(flags=lb.FLAG_NO_FILL_PADDING, ts=1, cs=3),
    dict(flags=lb.FLAG_NATURAL_ORDER, ts=2, cs=6),
    dict(flags=lb.FLAG_NO_SDDMM | lb.FLAG_XCD_ORDER, spmm_min_vec_nnz=1),
    dict(flags=lb.FLAG_NO_SPMM | lb.FLAG_NO_XCD_ORDER, sddmm_min_blk_nnz=64),
    dict(spmm_min_vec_nnz=16, sddmm_min_blk_nnz=200),
    dict(sddmm_min_blk_nnz=20, sddmm_min_dense_pct=30),
    dict(sddmm_min_blk_nnz=20, sddmm_min_dense_pct=85),
]


def matrices():
    yield "random", wl.random_pattern(203, 150, 0.08, seed=5, empty_rows=0.15)
    yield "community", wl.community(n_blocks=6, seed=2)
    yield "rmat", wl.rmat(scale=9, avg_degree=8, seed=3)
    yield "longrows", wl.with_long_rows(wl.random_pattern(90, 400, 0.03, seed=7), [3, 17, 18, 64], 300, seed=8)
    yield "single_row", wl.random_pattern(1, 50, 0.5, seed=9)
    yield "ragged_tail", wl.random_pattern(1000, 300, 0.03, seed=10, empty_rows=0.3)
    yield "dense_rows", wl.random_pattern(40, 700, 0.6, seed=11)          # windows with many blocks
    yield "leading_empty_windows", wl.with_long_rows(wl.random_pattern(100, 64, 0.0, seed=12), [70, 99], 40, seed=13)


@pytest.mark.parametrize("case", range(len(CASES)))
def test_device_planner_equals_host_planner(case):
    kw = CASES[case]
    for name, A in matrices():
        print("case", case, name, flush=True)
        ph = lb.Plan.from_csr(A, **kw)
        pd = device_plan(A, **kw)
        assert_same_plan(ph, pd, kw.get("flags", 0))
        ph.close()
        pd.close()


@pytest.mark.parametrize("case", range(len(CASES)))
def test_device_planner_equals_reference_planner(case):
    """The device-built plan against the reference planner written from the paper (not against the host planner, with
    which it shares the code that orders the task tables): same blocks, bitmaps, residual arrays, tasks, cleared rows."""
    from test_plan_host import check_subplan, ref_opts
    from oracle import planner_ref as pr
    kw = CASES[case]
    fl = kw.get("flags", 0)
    for name, A in matrices():
        if A.nnz > 20000:
            continue                    # the reference planner walks Python dictionaries
        print("case", case, name, flush=True)
        pd = device_plan(A, **kw)
        o = ref_opts(kw)
        if not fl & lb.FLAG_NO_SPMM:
            check_subplan(A, pd.export(0), pr.plan_spmm(A.M, A.rowptr, A.col, o), spmm=True)
        if not fl & lb.FLAG_NO_SDDMM:
            check_subplan(A, pd.export(1), pr.plan_sddmm(A.M, A.rowptr, A.col, o), spmm=False)
        pd.close()


def test_device_planner_random_options():
    rng = np.random.default_rng(20250622)
    for it in range(40):
        M, Kc = int(rng.integers(1, 400)), int(rng.integers(1, 500))
        A = wl.random_pattern(M, Kc, float(rng.uniform(0, 0.4)), seed=int(rng.integers(1 << 30)), empty_rows=0.2)
        if M > 3 and Kc > 30 and it % 2:
            A = wl.with_long_rows(A, [M // 2], min(Kc, 200), seed=it)
        kw = dict(mode=int(rng.integers(0, 3)), spmm_min_vec_nnz=int(rng.integers(1, 8)), sddmm_min_blk_nnz=int(rng.integers(1, 80)),
                  ts=int(rng.integers(1, 6)), cs=int(rng.integers(1, 40)), short_len=int(rng.integers(1, 5)),
                  sddmm_cs=int(rng.integers(1, 60)), sddmm_ts=int(rng.integers(1, 9)), flags=int(rng.choice([0, 1, 8, 9, 16, 32, 256, 288])),
                  sddmm_min_dense_pct=int(rng.choice([0, 0, 25, 60, 100])))
        print("random case", it, M, Kc, A.nnz, kw, flush=True)
        ph = lb.Plan.from_csr(A, **kw)
        pd = device_plan(A, **kw)
        assert_same_plan(ph, pd)
        ph.close()
        pd.close()


def test_device_planner_value_types_and_results():
    A = wl.make("powerlaw", small=True)
    # fp32 values: forced onto the scalar path, 4-byte values travel
    v32 = A.val.astype(np.float32) * 1.25
    assert_same_plan(lb.Plan.from_csr(A, val=v32), device_plan(A, val=v32))
    # bfloat16 bit patterns
    vb = wl.to_bf16_bits(np.linspace(-2, 2, A.nnz, dtype=np.float32) + 0.3)
    assert_same_plan(lb.Plan.from_csr(A, val=vb, val_dtype=lb.BF16), device_plan(A, val=vb, val_dtype=lb.BF16))
    # a device-built plan runs like a host-built one
    B = wl.dense_normal(A.Kc, 64, seed=3)
    ph = lb.Plan.from_csr(A).upload()
    pd = device_plan(A).upload()
    Bd = torch.from_numpy(B).cuda()
    Ch, Cd = ph.spmm(Bd), pd.spmm(Bd)
    one_writer = torch.ones(A.M, dtype=torch.bool, device="cuda")
    one_writer[torch.from_numpy(ph.export(0)["zero_rows"]).cuda().long()] = False
    assert torch.equal(Ch[one_writer], Cd[one_writer])
    assert torch.allclose(Ch, Cd, rtol=1e-4, atol=1e-3)


def _run_all(p, A, B, X, Y):
    """Every compute call on a ready plan; SpMM rows with several writers are returned separately."""
    C1 = p.spmm(B)
    out = torch.full((p.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    p.sddmm(X, Y, out=out)
    alpha = p.edge_softmax(out, 0.25)
    p.set_values(alpha)
    C2 = p.spmm(B)
    out2 = p.sddmm(X, Y)
    torch.cuda.synchronize()
    return C1, out, alpha, C2, out2


@pytest.mark.parametrize("keep_host_copy", [True, False])
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_resident_device_plan_computes_like_an_uploaded_host_plan(dtype, keep_host_copy):
    """The plan's device copy written by the planner itself (no host round trip) against libra_plan + libra_plan_upload."""
    A = wl.make("powerlaw", small=True)
    N, K = 64, 32
    if dtype == "f32":
        val, code, tdt = A.val.astype(np.float32) * 0.75, lb.F32, torch.float32
        mk = lambda r, c, seed: torch.from_numpy(wl.dense_normal(r, c, seed=seed, dtype=np.float32)).cuda()
    elif dtype == "bf16":
        val, code, tdt = wl.to_bf16_bits(A.val.astype(np.float32) * 0.75), lb.BF16, torch.bfloat16
        mk = lambda r, c, seed: torch.from_numpy(wl.dense_normal(r, c, seed=seed, dtype=np.float32)).cuda().to(torch.bfloat16)
    else:
        val, code, tdt = A.val, lb.F16, torch.float16
        mk = lambda r, c, seed: torch.from_numpy(wl.dense_normal(r, c, seed=seed)).cuda()
    B, X, Y = mk(A.Kc, N, 1), mk(A.M, K, 2), mk(A.Kc, K, 3)
    kw = dict(cs=40, ts=2)
    ph = lb.Plan.from_csr(A, val=val, val_dtype=code, **kw).upload()
    pd = lb.Plan.from_device_csr(A.M, A.Kc, torch.from_numpy(A.rowptr.astype(np.int32)).cuda(), torch.from_numpy(A.col.astype(np.int32)).cuda(),
                                 dev_val(val, code), resident=True, keep_host_copy=keep_host_copy, **kw)
    assert lb.libra_plan_device_bytes(pd.handle) == lb.libra_plan_device_bytes(ph.handle) <= pd._buf.numel()
    if keep_host_copy:
        assert_same_plan(ph, pd)
    else:
        for call in (lambda: pd.export(0), lambda: pd.upload()):
            with pytest.raises(lb.LibraError) as e:
                call()
            assert e.value.code == lb.ERR["NOT_BUILT"]
        sh, sd = ph.stats(), pd.stats()
        assert all(sh[k] == sd[k] for k in sh if k not in TIMES)
    one_writer = torch.ones(A.M, dtype=torch.bool, device="cuda")
    one_writer[torch.from_numpy(ph.export(0)["zero_rows"]).cuda().long()] = False
    assert 0 < int(one_writer.sum()) < A.M
    rh, rd = _run_all(ph, A, B, X, Y), _run_all(pd, A, B, X, Y)
    for k in (1, 2, 4):                                     # SDDMM, softmax: one writer per output
        assert torch.equal(rh[k], rd[k]), k
    for k in (0, 3):
        assert torch.equal(rh[k][one_writer], rd[k][one_writer]), k
        assert torch.allclose(rh[k], rd[k], rtol=1e-3, atol=1e-3), k


def test_device_planner_rejects_what_the_host_planner_rejects():
    A = wl.random_pattern(64, 64, 0.2, seed=3)
    rp = torch.from_numpy(A.rowptr.astype(np.int32)).cuda()
    col = torch.from_numpy(A.col.astype(np.int32)).cuda()
    val = torch.from_numpy(A.val).cuda()

    def rc(M=A.M, Kc=A.Kc, rowptr=rp, c=col, **kw):
        try:
            lb.Plan.from_device_csr(M, Kc, rowptr, c, val, **kw).close()
            return 0
        except lb.LibraError as e:
            return e.code

    assert rc() == 0
    bad = col.clone(); bad[5] = A.Kc
    assert rc(c=bad) == lb.ERR["COLUMN"]
    bad = col.clone(); bad[3] = -1
    assert rc(c=bad) == lb.ERR["COLUMN"]
    s, e = int(A.rowptr[10]), int(A.rowptr[11])
    assert e - s >= 2
    bad = col.clone(); bad[s + 1] = bad[s]
    assert rc(c=bad) == lb.ERR["UNSORTED"]
    badrp = rp.clone(); badrp[7] = badrp[8] + 1
    assert rc(rowptr=badrp) == lb.ERR["ROWPTR"]
    assert rc(window_rows=8) == lb.ERR["UNSUPPORTED"]
    assert rc(mode=7) == lb.ERR["OPTION"]
    # a matrix without nonzeros
    z = torch.zeros(9, dtype=torch.int32, device="cuda")
    p = lb.Plan.from_device_csr(8, 5, z, col[:0], val[:0])
    assert p.stats()["nnz"] == 0 and p.stats()["spmm_tasks"] == 1
    p.close()


@pytest.mark.parametrize("name", ["powerlaw", "community", "gat", "irregular"])
def test_device_planner_full_configs(name):
    A = wl.make(name)
    t0 = time.perf_counter()
    ph = lb.Plan.from_csr(A)
    t_host = time.perf_counter() - t0
    rp, col, val = (torch.from_numpy(x).cuda() for x in (A.rowptr.astype(np.int32), A.col.astype(np.int32), A.val))
    lb.Plan.from_device_csr(A.M, A.Kc, rp, col, val).close()           # warm-up (module load, allocator)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pd = lb.Plan.from_device_csr(A.M, A.Kc, rp, col, val)
    t_dev = time.perf_counter() - t0
    print(f"{name}: host planner {t_host:.3f} s, device planner {t_dev:.3f} s "
          f"(device passes {pd.stats()['device_seconds']:.4f} s)", flush=True)
    assert_same_plan(ph, pd)
    # plan + device copy: host planner + upload against the resident device plan without a host copy
    t0 = time.perf_counter()
    ph.upload()
    torch.cuda.synchronize()
    t_up = time.perf_counter() - t0
    lb.Plan.from_device_csr(A.M, A.Kc, rp, col, val, resident=True, keep_host_copy=False).close()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pr = lb.Plan.from_device_csr(A.M, A.Kc, rp, col, val, resident=True, keep_host_copy=False)
    torch.cuda.synchronize()
    t_res = time.perf_counter() - t0
    print(f"{name}: ready to compute: host plan + upload {t_host + t_up:.3f} s, resident device plan {t_res:.4f} s", flush=True)
    B = torch.from_numpy(wl.dense_normal(A.Kc, 32, seed=5)).cuda()
    one_writer = torch.ones(A.M, dtype=torch.bool, device="cuda")
    one_writer[torch.from_numpy(ph.export(0)["zero_rows"]).cuda().long()] = False
    assert torch.equal(ph.spmm(B)[one_writer], pr.spmm(B)[one_writer])
