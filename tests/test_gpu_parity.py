"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.

Tolerances (graded error, see oracle.graded_error):
  fp16 inputs, fp32 accumulate ... <= 1e-2   (the stated bar)
  fp32 VALU-only mode ............ <= 1e-5   (the stated bar)
and, because products of fp16 numbers are exact in fp32 and only the fp32
accumulation rounds, a derived bound 16*sqrt(d)*2^-24 (d = summed terms) that a
correct kernel also meets on these inputs; it catches small dropped terms the
1e-2 bar would let through.
"""
import functools
import os

import numpy as np
import pytest

import oracle
from paper_2506_22714_amd import binding as lb
from paper_2506_22714_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL_F16 = 1e-2
TOL_F32 = 1e-5


def derived_tol(d):
    return 16.0 * np.sqrt(max(float(d), 1.0)) * 2.0 ** -24


@pytest.fixture(scope="module", autouse=True)
def need_gpu_and_library():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if not os.path.exists(lb.LIB_PATH):
        from paper_2506_22714_amd.build import build_library
        build_library()
    lb.lib()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_spmm(A, B, val=None, ldb=None, ldc=None, **opts):
    p = lb.Plan.from_csr(A, val=val, flags=opts.pop("flags", 0) | lb.FLAG_NO_SDDMM, **opts).upload()
    N = B.shape[1]
    if ldb is None and ldc is None:
        C = p.spmm(dev(B))
    else:
        Bp = torch.zeros((B.shape[0], ldb or N), dtype=dev(B).dtype, device="cuda")
        Bp[:, :N] = dev(B)
        Cp = torch.full((A.M, ldc or N), 7.0, dtype=torch.float32, device="cuda")
        p.spmm(Bp[:, :N], out=Cp[:, :N])
        assert torch.all(Cp[:, N:] == 7.0)          # nothing written outside the N columns
        C = Cp[:, :N]
    torch.cuda.synchronize()
    out = C.cpu().numpy()
    st = p.stats()
    p.close()
    return out, st


def gpu_sddmm(A, X, Y, val=None, **opts):
    p = lb.Plan.from_csr(A, val=val, flags=opts.pop("flags", 0) | lb.FLAG_NO_SPMM, **opts).upload()
    out = torch.full((p.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    p.sddmm(dev(X), dev(Y), out=out)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    st = p.stats()
    p.close()
    return res, st


def bound(tol, d):
    """The stated bar, tightened to the derived bound where that is smaller."""
    return min(tol, derived_tol(d))


def check_spmm(A, B, C, tol, val=None, rows=None, C_is_subset=False):
    v = A.val if val is None else val
    ref, S = oracle.spmm(A.rowptr, A.col, v, B, rows=rows)
    deg = np.diff(A.rowptr).astype(np.float64)
    if rows is not None:
        deg = deg[rows]
        if not C_is_subset:
            C = C[rows]
    assert np.all(np.isfinite(C))
    err = oracle.graded_error(C, ref, S, deg[:, None])
    lim = bound(tol, deg.max() if deg.size else 1)
    assert err <= lim, f"graded error {err:.3e} > {lim:.3e}"
    return err


def check_spmm_all_rows(A, B, C_dev, tol, val=None, chunk=1 << 17, bf16=False):
    """Every row of a device result against the oracle, walked in chunks of rows so that the double-precision
    reference of a large C never exists whole; returns the largest graded error."""
    v = A.val if val is None else val
    deg_all = np.diff(A.rowptr).astype(np.float64)
    worst = 0.0
    for r0 in range(0, A.M, chunk):
        rows = np.arange(r0, min(A.M, r0 + chunk), dtype=np.int64)
        ref, S = oracle.spmm(A.rowptr, A.col, v, B, rows=rows, bf16=bf16)
        got = C_dev[r0:r0 + rows.size].cpu().numpy()
        assert np.all(np.isfinite(got)), f"rows {r0}.."
        deg = deg_all[rows]
        err = oracle.graded_error(got, ref, S, deg[:, None])
        lim = bound(tol, deg.max() if deg.size else 1)
        assert err <= lim, f"rows {r0}..{r0 + rows.size}: graded error {err:.3e} > {lim:.3e}"
        worst = max(worst, err)
    return worst


def check_sddmm(A, X, Y, out, tol, val=None, idx=None):
    v = A.val if val is None else val
    ref, S = oracle.sddmm(A.rowptr, A.col, v, X, Y, idx=idx)
    got = out if idx is None else out[idx]
    assert np.all(np.isfinite(got))
    err = oracle.graded_error(got, ref, S, X.shape[1])
    lim = bound(tol, X.shape[1])
    assert err <= lim, f"graded error {err:.3e} > {lim:.3e}"
    return err


def mixed_matrix(M=1000, Kc=900, seed=1):
    """Ragged tail (M % 16 != 0), empty rows, a few very long rows (row splitting)
    and a band of dense columns (windows with more blocks than Ts)."""
    A = wl.random_pattern(M, Kc, 0.02, seed=seed, empty_rows=0.2)
    A = wl.with_long_rows(A, [5, 6, 333, M - 1], 700, seed=seed + 1)
    D = np.zeros((M, Kc), dtype=np.float32)
    for i in range(A.M):
        s, e = A.rowptr[i], A.rowptr[i + 1]
        D[i, A.col[s:e]] = A.val[s:e]
    rng = np.random.default_rng(seed + 2)
    c0, c1 = Kc // 3, min(Kc, Kc // 3 + 200)
    band = rng.random((64, c1 - c0)) < 0.5
    D[100:164, c0:c1] = np.where(band, wl.uniform_values(rng, band.size).reshape(band.shape), D[100:164, c0:c1])
    return wl.from_dense(D)


# ---------------------------------------------------------------- config 1
@pytest.mark.parametrize("mode", [lb.MODE_HYBRID, lb.MODE_DENSE_ONLY, lb.MODE_SCALAR_ONLY])
def test_tiny_config_spmm_and_sddmm(mode):
    A = wl.tiny()
    B = wl.dense_normal(A.Kc, 32, seed=wl.BASE_SEED + 101)
    C, st = gpu_spmm(A, B, mode=mode)
    check_spmm(A, B, C, TOL_F16)
    X = wl.dense_normal(A.M, 32, seed=wl.BASE_SEED + 102)
    Y = wl.dense_normal(A.Kc, 32, seed=wl.BASE_SEED + 103)
    out, st = gpu_sddmm(A, X, Y, mode=mode)
    check_sddmm(A, X, Y, out, TOL_F16)


@pytest.mark.parametrize("mode", [lb.MODE_HYBRID, lb.MODE_DENSE_ONLY, lb.MODE_SCALAR_ONLY])
def test_tiny_config_fp32_mode(mode):
    A = wl.tiny()
    v32 = A.val.astype(np.float32)
    B = wl.dense_normal(A.Kc, 32, seed=wl.BASE_SEED + 101, dtype=np.float32)
    kw = dict(mode=mode, spmm_min_vec_nnz=2, sddmm_min_blk_nnz=17)          # both paths in use in the hybrid mode
    C, st = gpu_spmm(A, B, val=v32, **kw)
    assert (st["spmm_dense_nnz"] > 0) == (mode != lb.MODE_SCALAR_ONLY) and (st["spmm_res_nnz"] > 0) == (mode != lb.MODE_DENSE_ONLY)
    check_spmm(A, B, C, TOL_F32, val=v32)
    X = wl.dense_normal(A.M, 32, seed=wl.BASE_SEED + 102, dtype=np.float32)
    Y = wl.dense_normal(A.Kc, 32, seed=wl.BASE_SEED + 103, dtype=np.float32)
    out, st = gpu_sddmm(A, X, Y, val=v32, **kw)
    assert (st["sddmm_dense_nnz"] > 0) == (mode != lb.MODE_SCALAR_ONLY)
    check_sddmm(A, X, Y, out, TOL_F32, val=v32)


# ------------------------------------------------------- shapes and splitting
@pytest.mark.parametrize("N", [32, 64, 96, 128, 160, 256, 384, 512])
def test_spmm_feature_widths_on_mixed_matrix(N):
    A = mixed_matrix()
    B = wl.dense_normal(A.Kc, N, seed=N)
    # with the die-aware window order the 128-column pieces of a wide operand share one launch, without it they run in turn
    for flags in (lb.FLAG_XCD_ORDER, lb.FLAG_NO_XCD_ORDER):
        C, st = gpu_spmm(A, B, ts=2, cs=48, flags=flags)
        assert st["xcd_order"] == (flags == lb.FLAG_XCD_ORDER)
        assert st["spmm_split_rows"] >= 4 and st["spmm_chunk_tasks"] > 8 and st["spmm_zero_rows"] > 0
        assert st["spmm_dense_nnz"] > 0 and st["spmm_res_nnz"] > 0
        check_spmm(A, B, C, TOL_F16)


@pytest.mark.parametrize("N", [16, 48, 128])
def test_spmm_fp32_mode_widths(N):
    A = mixed_matrix(M=500, Kc=450, seed=4)
    v32 = A.val.astype(np.float32)
    B = wl.dense_normal(A.Kc, N, seed=N, dtype=np.float32)
    for mode in (lb.MODE_HYBRID, lb.MODE_DENSE_ONLY, lb.MODE_SCALAR_ONLY):
        C, st = gpu_spmm(A, B, val=v32, cs=64, ts=2, mode=mode)
        assert (st["spmm_dense_nnz"] > 0) == (mode != lb.MODE_SCALAR_ONLY)
        check_spmm(A, B, C, TOL_F32, val=v32)


@pytest.mark.parametrize("K", [32, 64, 128])
def test_sddmm_feature_widths_on_mixed_matrix(K):
    A = mixed_matrix(seed=3)
    X = wl.dense_normal(A.M, K, seed=K)
    Y = wl.dense_normal(A.Kc, K, seed=K + 1)
    out, st = gpu_sddmm(A, X, Y, ts=2, sddmm_cs=100, sddmm_min_blk_nnz=24)
    assert st["sddmm_dense_nnz"] > 0 and st["sddmm_res_nnz"] > 0
    check_sddmm(A, X, Y, out, TOL_F16)
    v32 = A.val.astype(np.float32)
    for mode in (lb.MODE_HYBRID, lb.MODE_DENSE_ONLY, lb.MODE_SCALAR_ONLY):
        out32, st32 = gpu_sddmm(A, X.astype(np.float32), Y.astype(np.float32), val=v32, ts=2, sddmm_min_blk_nnz=24, mode=mode)
        assert (st32["sddmm_dense_nnz"] > 0) == (mode != lb.MODE_SCALAR_ONLY)
        check_sddmm(A, X.astype(np.float32), Y.astype(np.float32), out32, TOL_F32, val=v32)


def test_mode_equivalence_over_thresholds():
    """Matrix-unit-only, scalar-only and hybrid at several thresholds compute the same product (Section 5.3.2)."""
    A = wl.community(n_blocks=12, seed=9)
    B = wl.dense_normal(A.Kc, 64, seed=5)
    X = wl.dense_normal(A.M, 32, seed=6)
    Y = wl.dense_normal(A.Kc, 32, seed=7)
    shares = []
    for kw in (dict(mode=lb.MODE_SCALAR_ONLY), dict(mode=lb.MODE_DENSE_ONLY), dict(spmm_min_vec_nnz=2, sddmm_min_blk_nnz=16),
               dict(spmm_min_vec_nnz=4, sddmm_min_blk_nnz=48), dict(spmm_min_vec_nnz=8, sddmm_min_blk_nnz=96, flags=lb.FLAG_NO_FILL_PADDING)):
        C, st = gpu_spmm(A, B, **dict(kw))
        check_spmm(A, B, C, TOL_F16)
        out, st2 = gpu_sddmm(A, X, Y, **dict(kw))
        check_sddmm(A, X, Y, out, TOL_F16)
        shares.append((st["spmm_dense_nnz"], st2["sddmm_dense_nnz"]))
    assert shares[0] == (0, 0) and shares[1] == (A.nnz, A.nnz)
    assert len(set(shares)) == len(shares)          # the thresholds really changed the split


def test_strided_operands_and_untouched_padding():
    A = mixed_matrix(M=300, Kc=260, seed=8)
    B = wl.dense_normal(A.Kc, 64, seed=2)
    C, _ = gpu_spmm(A, B, ldb=72, ldc=100, cs=32)
    check_spmm(A, B, C, TOL_F16)


def test_non_atomic_rows_are_bitwise_repeatable_and_exact_on_integers():
    A = mixed_matrix(M=400, Kc=300, seed=11)
    A.val = np.random.default_rng(0).integers(1, 4, size=A.nnz).astype(np.float16)
    B = wl.dense_small_int(A.Kc, 128, seed=3)
    C1, _ = gpu_spmm(A, B, cs=64)
    C2, _ = gpu_spmm(A, B, cs=64)
    ref, _ = oracle.spmm(A.rowptr, A.col, A.val, B)
    # small integers: every partial sum is exact in fp32, so any summation order gives the oracle's bits
    assert np.array_equal(C1.astype(np.float64), ref) and np.array_equal(C1, C2)


# ------------------------------------------------------------------ edge cases
def test_degenerate_matrices():
    B = wl.dense_normal(40, 32, seed=1)
    # no nonzeros at all: C must be all zeros whatever it held before
    E = wl.Csr(33, 40, np.zeros(34, dtype=np.int32), np.zeros(0, dtype=np.int32), np.zeros(0, dtype=np.float16))
    C, _ = gpu_spmm(E, B, ldc=32)
    assert C.shape == (33, 32) and not C.any()
    out, _ = gpu_sddmm(E, wl.dense_normal(33, 32, seed=2), wl.dense_normal(40, 32, seed=3))
    assert out.size == 0
    # one row, one nonzero; one full dense row; M = 1
    one = wl.from_dense(np.eye(1, 40, 7))
    C, _ = gpu_spmm(one, B)
    assert np.array_equal(C[0], B[7].astype(np.float32))
    full = wl.from_dense(np.ones((17, 40)))
    C, _ = gpu_spmm(full, B)
    check_spmm(full, B, C, TOL_F16)
    out, _ = gpu_sddmm(full, wl.dense_normal(17, 32, seed=2), wl.dense_normal(40, 32, seed=3))
    check_sddmm(full, wl.dense_normal(17, 32, seed=2), wl.dense_normal(40, 32, seed=3), out, TOL_F16)


def test_fp16_subnormal_inputs_are_not_flushed():
    A = wl.random_pattern(64, 64, 0.3, seed=5)
    A.val = np.full(A.nnz, 1024.0, dtype=np.float16)
    B = np.full((64, 32), 2.0 ** -24, dtype=np.float16)        # smallest fp16 subnormal
    for mode in (lb.MODE_DENSE_ONLY, lb.MODE_SCALAR_ONLY):
        C, _ = gpu_spmm(A, B, mode=mode)
        ref, _ = oracle.spmm(A.rowptr, A.col, A.val, B)
        assert np.array_equal(C.astype(np.float64), ref)


def test_unsupported_requests_return_codes():
    A = wl.random_pattern(64, 64, 0.1, seed=2)
    p = lb.Plan.from_csr(A).upload()
    B = torch.zeros((64, 40), dtype=torch.float16, device="cuda")
    with pytest.raises(lb.LibraError) as e:
        p.spmm(B)
    assert e.value.code == lb.ERR["UNSUPPORTED"]
    X = torch.zeros((64, 48), dtype=torch.float16, device="cuda")
    with pytest.raises(lb.LibraError) as e:
        p.sddmm(X, X)
    assert e.value.code == lb.ERR["UNSUPPORTED"]
    p8 = lb.Plan.from_csr(A, window_rows=8).upload()
    with pytest.raises(lb.LibraError) as e:
        p8.spmm(torch.zeros((64, 32), dtype=torch.float16, device="cuda"))
    assert e.value.code == lb.ERR["UNSUPPORTED"]
    # residual entries keep their column in 27 bits: a wider matrix plans, and is refused when it is uploaded
    rowptr = np.array([0, 2] + [2] * 15, dtype=np.int32)
    col = np.array([5, (1 << 27) + 3], dtype=np.int32)
    for dt in (np.float16, np.float32):
        wide = lb.Plan(16, (1 << 27) + 8, rowptr, col, np.ones(2, dtype=dt))
        with pytest.raises(lb.LibraError) as e:
            wide.upload()
        assert e.value.code == lb.ERR["UNSUPPORTED"]
        lb.Plan(16, 1 << 27, rowptr, np.array([5, (1 << 27) - 1], dtype=np.int32), np.ones(2, dtype=dt)).upload().close()


# ---------------------------------------------- softmax glue and new values
def test_new_values_for_one_operator_leave_the_other_alone():
    """Refreshing only the SpMM arrays (what an attention layer needs) changes libra_spmm and not libra_sddmm, and the
    other way round; both against the oracle with the values each operator should see."""
    A = wl.make("powerlaw", small=True)
    N = K = 32
    B, X, Y = wl.dense_normal(A.Kc, N, seed=31), wl.dense_normal(A.M, K, seed=32), wl.dense_normal(A.Kc, K, seed=33)
    rng = np.random.default_rng(34)
    v1, v2 = wl.uniform_values(rng, A.nnz), wl.uniform_values(rng, A.nnz)
    p = lb.Plan.from_csr(A).upload()                     # both operators start from A.val
    p.set_values(dev(v1), lb.OP_SPMM)
    check_spmm(A, B, p.spmm(dev(B)).cpu().numpy(), TOL_F16, val=v1)
    check_sddmm(A, X, Y, p.sddmm(dev(X), dev(Y)).cpu().numpy(), TOL_F16)
    p.set_values(dev(v2), lb.OP_SDDMM)
    check_spmm(A, B, p.spmm(dev(B)).cpu().numpy(), TOL_F16, val=v1)
    check_sddmm(A, X, Y, p.sddmm(dev(X), dev(Y)).cpu().numpy(), TOL_F16, val=v2)
    for bad in (0, 4, 7):
        with pytest.raises(lb.LibraError) as e:
            p.set_values(dev(v1), bad)
        assert e.value.code == lb.ERR["OPTION"]
    p.close()


def test_edge_softmax_at_every_row_length_class_boundary():
    """Rows of exactly the lengths at which the softmax kernels change shape (16 lanes per row up to 64 nonzeros; one wave,
    512 scores per round, up to 2048; one workgroup, 4096 per round, beyond), with scores that grow along the row so that
    the running maximum is replaced in every round.  Forward against the oracle, backward against the textbook formula."""
    lengths = [0, 1, 2, 15, 16, 17, 63, 64, 65, 127, 511, 512, 513, 1023, 1025, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8193, 12001]
    Kc = 16384
    rng = np.random.default_rng(77)
    cols = [np.sort(rng.choice(Kc, size=n, replace=False)).astype(np.int32) for n in lengths]
    rowptr = np.zeros(len(lengths) + 1, dtype=np.int32)
    np.cumsum(lengths, out=rowptr[1:])
    A = wl.Csr(len(lengths), Kc, rowptr, np.concatenate(cols).astype(np.int32), np.ones(int(rowptr[-1]), dtype=np.float16))
    rows = np.repeat(np.arange(A.M), lengths)
    pos = np.arange(A.nnz) - rowptr[rows]
    scores = (20.0 * pos / np.maximum(np.asarray(lengths)[rows] - 1, 1) - 10.0 + rng.standard_normal(A.nnz)).astype(np.float32)
    dalpha = rng.standard_normal(A.nnz).astype(np.float32)
    scale = 1.3
    p = lb.Plan.from_csr(A).upload()
    ref = oracle.edge_softmax(A.rowptr, scores.astype(np.float64), scale)
    a32 = p.edge_softmax(dev(scores), scale, out=torch.empty(A.nnz, dtype=torch.float32, device="cuda"))
    got = a32.cpu().numpy().astype(np.float64)
    # fp32 exponentials of arguments down to -26 against a double reference: relative error of exp and of the sum
    assert np.max(np.abs(got - ref) / ref) < 2e-5
    sums = np.bincount(rows, weights=got, minlength=A.M)
    assert np.all(np.abs(sums[np.asarray(lengths) > 0] - 1.0) < 1e-5)
    a16 = p.edge_softmax(dev(scores), scale).cpu().numpy().astype(np.float64)
    assert np.max(np.abs(a16 - ref) / np.maximum(ref, 2.0 ** -14)) < 1e-3
    # the arrays need no more than their element alignment: views that start one element into a larger buffer are 4-byte
    # (scores, fp32 output) or 2-byte (fp16 output) aligned only and must give the same results to the same bars
    sbuf = torch.zeros(A.nnz + 1, dtype=torch.float32, device="cuda")
    sbuf[1:] = dev(scores)
    for dt in (torch.float32, torch.float16):
        obuf = torch.full((A.nnz + 1,), float("nan"), dtype=dt, device="cuda")
        assert sbuf[1:].data_ptr() % 16 != 0 and obuf[1:].data_ptr() % 16 != 0
        odd = p.edge_softmax(sbuf[1:], scale, out=obuf[1:]).cpu().numpy().astype(np.float64)
        even = p.edge_softmax(dev(scores), scale, out=torch.empty(A.nnz, dtype=dt, device="cuda"))
        assert even.data_ptr() % 16 == 0 and bool(torch.isnan(obuf[0]))           # nothing written in front of the view
        for got_x in (odd, even.cpu().numpy().astype(np.float64)):
            if dt == torch.float32:
                assert np.max(np.abs(got_x - ref) / ref) < 2e-5
            else:
                assert np.max(np.abs(got_x - ref) / np.maximum(ref, 2.0 ** -14)) < 1e-3
    ds = p.edge_softmax_backward(a32, dev(dalpha), scale).cpu().numpy().astype(np.float64)
    dot = np.bincount(rows, weights=got * dalpha, minlength=A.M)
    sabs = np.bincount(rows, weights=np.abs(got * dalpha), minlength=A.M)
    want = scale * got * (dalpha - dot[rows])
    tol = 32 * np.sqrt(max(lengths)) * 2.0 ** -24
    assert np.max(np.abs(ds - want) / (scale * got * (np.abs(dalpha) + sabs[rows]) + 1e-30)) <= tol
    p.close()


def test_edge_softmax_and_set_values_attention_head():
    A = wl.make("gat", small=True)
    K = 64
    X = wl.dense_normal(A.M, K, seed=21)
    Y = wl.dense_normal(A.Kc, K, seed=22)
    scale = 1.0 / np.sqrt(K)
    s_ref, a_ref, C_ref, S_ref = oracle.attention_head(A.rowptr, A.col, A.val, X, Y, Y, scale)
    p = lb.Plan.from_csr(A).upload()
    Yd = dev(Y)
    scores = p.sddmm(dev(X), Yd)
    alpha = p.edge_softmax(scores, scale)
    p.set_values(alpha)
    C = p.spmm(Yd)
    torch.cuda.synchronize()
    # scores and alpha step by step
    check_sddmm(A, X, Y, scores.cpu().numpy(), TOL_F16)
    a = alpha.cpu().numpy().astype(np.float64)
    deg = np.diff(A.rowptr)
    rows = np.repeat(np.arange(A.M), deg)
    assert np.max(np.abs(a - a_ref.astype(np.float64)) / np.maximum(a_ref.astype(np.float64), 2.0 ** -14)) < 4e-3
    sums = np.bincount(rows, weights=a, minlength=A.M)
    assert np.all(np.abs(sums[deg > 0] - 1.0) <= 2.0 ** -11 * np.maximum(deg[deg > 0], 4))
    # whole head against the oracle's head (alpha differs by at most an fp16 ulp, inside the 1e-2 bar)
    err = oracle.graded_error(C.cpu().numpy(), C_ref, S_ref, np.maximum(deg, 1)[:, None])
    assert err <= TOL_F16
    # and the SpMM step alone, fed the GPU's own alpha, to the derived bound
    check_spmm(A, Y, C.cpu().numpy(), TOL_F16, val=alpha.cpu().numpy())
    # fp32 softmax output path
    a32 = p.edge_softmax(scores, scale, out=torch.empty(p.nnz, dtype=torch.float32, device="cuda")).cpu().numpy()
    ref32 = oracle.edge_softmax(A.rowptr, scores.cpu().numpy().astype(np.float64), scale)
    assert np.max(np.abs(a32 - ref32) / ref32) < 1e-5


def test_die_aware_task_order_changes_no_result():
    """The order of the task table (and the empty tasks the die-aware order adds) is invisible in the results."""
    A = wl.make("community", small=True)
    B = wl.dense_normal(A.Kc, 128, seed=31)
    X = wl.dense_normal(A.M, 32, seed=32)
    Y = wl.dense_normal(A.Kc, 32, seed=33)
    res = []
    for fl in (lb.FLAG_NO_XCD_ORDER, lb.FLAG_XCD_ORDER, 0):
        p = lb.Plan.from_csr(A, flags=fl).upload()
        C = p.spmm(dev(B))
        out = torch.full((p.nnz,), float("nan"), dtype=torch.float32, device="cuda")
        p.sddmm(dev(X), dev(Y), out=out)
        torch.cuda.synchronize()
        st = p.stats()
        res.append((C.cpu().numpy(), out.cpu().numpy(), st))
        p.close()
    assert res[0][2]["xcd_order"] == 0 and res[1][2]["xcd_order"] == 1 and res[2][2]["xcd_order"] == 1
    assert res[1][2]["spmm_tasks"] >= res[0][2]["spmm_tasks"]
    assert res[0][2]["spmm_zero_rows"] == 0          # no row is decomposed here: every row has one writer, sums have one order
    for k in (1, 2):
        assert np.array_equal(res[0][0], res[k][0]) and np.array_equal(res[0][1], res[k][1])
    check_spmm(A, B, res[1][0], TOL_F16)
    check_sddmm(A, X, Y, res[1][1], TOL_F16)


@pytest.mark.parametrize("N", [64, 128])
def test_two_kernel_schedule_matches_the_fused_task(N):
    """Dense blocks and residual nonzeros as two launches (the paper's sequential schedule): same result up to the order
    of the fp32 additions."""
    A = mixed_matrix(seed=9)
    B = wl.dense_normal(A.Kc, N, seed=60 + N)
    fused, st = gpu_spmm(A, B, ts=2, cs=48)
    assert 0 < st["spmm_dense_nnz"] < A.nnz and st["spmm_chunk_tasks"] > 0
    two, _ = gpu_spmm(A, B, ts=2, cs=48, flags=lb.FLAG_TWO_KERNELS)
    check_spmm(A, B, two, TOL_F16)
    assert np.allclose(two, fused, rtol=1e-5, atol=1e-4)
    Bi = wl.dense_small_int(A.Kc, N, seed=61)               # exact arithmetic: any order gives the same bits
    Ai = wl.Csr(A.M, A.Kc, A.rowptr, A.col, np.sign(A.val).astype(np.float16))
    f2, _ = gpu_spmm(Ai, Bi, ts=2, cs=48)
    t2, _ = gpu_spmm(Ai, Bi, ts=2, cs=48, flags=lb.FLAG_TWO_KERNELS)
    assert np.array_equal(f2, t2)


def test_one_plan_on_two_streams():
    """A plan is read-only during compute calls and has no hidden workspace: calls on different streams may overlap."""
    A = wl.make("powerlaw", small=True)
    p = lb.Plan.from_csr(A, cs=32).upload()
    assert p.stats()["spmm_zero_rows"] > 0                      # rows with several writers are in play
    Bs = [dev(wl.dense_normal(A.Kc, 64, seed=40 + i)) for i in range(2)]
    X, Y = dev(wl.dense_normal(A.M, 32, seed=50)), dev(wl.dense_normal(A.Kc, 32, seed=51))
    ref = [p.spmm(B) for B in Bs]
    ref_out = p.sddmm(X, Y)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(2)]            # default priority
    got = [None, None]
    outs = [None, None]
    for rep in range(5):
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                got[i] = p.spmm(Bs[i])
                outs[i] = p.sddmm(X, Y)
        torch.cuda.synchronize()
        one_writer = torch.ones(A.M, dtype=torch.bool, device="cuda")
        one_writer[torch.from_numpy(p.export(0)["zero_rows"]).cuda().long()] = False
        for i in range(2):
            assert torch.equal(got[i][one_writer], ref[i][one_writer])
            assert torch.allclose(got[i], ref[i], rtol=1e-4, atol=1e-3)
            assert torch.equal(outs[i], ref_out)
    p.close()


def test_compute_calls_can_be_captured_in_a_graph():
    """The compute calls only launch kernels on the caller's stream (rows with several writers are cleared by a kernel, not
    by a memset; nothing is allocated), so a step can be captured once and replayed: every replay, with eager work between
    the replays, gives the eager result."""
    A = wl.make("powerlaw", small=True)
    p = lb.Plan.from_csr(A, cs=32).upload()
    assert p.stats()["spmm_zero_rows"] > 0
    B = dev(wl.dense_small_int(A.Kc, 64, seed=60))              # integer-valued inputs: every order of additions is exact
    X, Y = dev(wl.dense_small_int(A.M, 32, seed=61)), dev(wl.dense_small_int(A.Kc, 32, seed=62))
    p.set_values(dev(np.ones(A.nnz, dtype=np.float16)))
    C_ref, out_ref = p.spmm(B), p.sddmm(X, Y)
    C, out = torch.empty_like(C_ref), torch.empty_like(out_ref)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()                                   # default priority
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        p.spmm(B, out=C)                                         # warm-up on the capture stream
        p.sddmm(X, Y, out=out)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            p.spmm(B, out=C)
            p.sddmm(X, Y, out=out)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        C.fill_(float("nan"))
        out.fill_(float("nan"))
        scratch = p.spmm(B)                                      # eager work of the same library between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(C, C_ref) and torch.equal(out, out_ref), rep
        assert torch.equal(scratch, C_ref)
    p.close()


# ------------------------------------------------------------- bfloat16
def dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_inputs(A, widths, seed):
    vb = wl.to_bf16_bits(A.val.astype(np.float32) * 1.37)          # values that are not exact in 8 bits before rounding
    mats = [wl.to_bf16_bits(wl.dense_normal(r, c, seed=seed + i, dtype=np.float32)) for i, (r, c) in enumerate(widths)]
    return vb, mats


@pytest.mark.parametrize("N", [32, 128, 256])
def test_bf16_spmm_matches_oracle(N):
    """bfloat16 storage on both paths (products of bfloat16 numbers are exact in fp32, so the derived bound holds)."""
    A = mixed_matrix()
    vb, (B,) = bf16_inputs(A, [(A.Kc, N)], seed=300 + N)
    for mode in (lb.MODE_HYBRID, lb.MODE_SCALAR_ONLY, lb.MODE_DENSE_ONLY):
        p = lb.Plan.from_csr(A, val=vb, val_dtype=lb.BF16, mode=mode, flags=lb.FLAG_NO_SDDMM).upload()
        C = p.spmm(dev_bf16(B))
        torch.cuda.synchronize()
        st = p.stats()
        p.close()
        if mode == lb.MODE_HYBRID:
            assert 0 < st["spmm_dense_nnz"] < A.nnz
        ref, S = oracle.spmm(A.rowptr, A.col, vb, B, bf16=True)
        deg = np.diff(A.rowptr).astype(np.float64)
        err = oracle.graded_error(C.cpu().numpy(), ref, S, deg[:, None])
        assert err <= bound(TOL_F16, deg.max()), (mode, err)


@pytest.mark.parametrize("K", [32, 64, 128])
def test_bf16_sddmm_matches_oracle(K):
    A = mixed_matrix(seed=5)
    vb, (X, Y) = bf16_inputs(A, [(A.M, K), (A.Kc, K)], seed=400 + K)
    for mode in (lb.MODE_HYBRID, lb.MODE_SCALAR_ONLY):
        p = lb.Plan.from_csr(A, val=vb, val_dtype=lb.BF16, mode=mode, flags=lb.FLAG_NO_SPMM).upload()
        out = torch.full((p.nnz,), float("nan"), dtype=torch.float32, device="cuda")
        p.sddmm(dev_bf16(X), dev_bf16(Y), out=out)
        torch.cuda.synchronize()
        st = p.stats()
        p.close()
        if mode == lb.MODE_HYBRID:
            assert 0 < st["sddmm_dense_nnz"] < A.nnz
        ref, S = oracle.sddmm(A.rowptr, A.col, vb, X, Y, bf16=True)
        got = out.cpu().numpy()
        assert np.all(np.isfinite(got))
        err = oracle.graded_error(got, ref, S, K)
        assert err <= bound(TOL_F16, K), (mode, err)


def test_bf16_attention_head():
    """SDDMM -> softmax with bfloat16 output -> new values -> SpMM, all in bfloat16 storage."""
    A = wl.make("gat", small=True)
    K = 64
    vb, (X, Y) = bf16_inputs(A, [(A.M, K), (A.Kc, K)], seed=77)
    vb = wl.to_bf16_bits(np.ones(A.nnz, dtype=np.float32))
    scale = 1.0 / np.sqrt(K)
    p = lb.Plan.from_csr(A, val=vb, val_dtype=lb.BF16).upload()
    Yd = dev_bf16(Y)
    scores = p.sddmm(dev_bf16(X), Yd)
    alpha = p.edge_softmax(scores, scale)
    assert alpha.dtype == torch.bfloat16
    p.set_values(alpha)
    C = p.spmm(Yd)
    torch.cuda.synchronize()
    s_ref, S = oracle.sddmm(A.rowptr, A.col, vb, X, Y, bf16=True)
    assert oracle.graded_error(scores.cpu().numpy(), s_ref, S, K) <= bound(TOL_F16, K)
    a_ref = oracle.edge_softmax(A.rowptr, scores.cpu().numpy().astype(np.float64), scale)
    a_bits = alpha.view(torch.int16).cpu().numpy().view(np.uint16)
    a = oracle.widen(a_bits, bf16=True)
    assert np.max(np.abs(a - a_ref) / a_ref) <= 2.0 ** -8 * 1.01        # one rounding to 8 significant bits
    # round-to-nearest-even, not truncation: the mean signed error is far below half an ulp
    assert abs(np.mean((a - a_ref) / a_ref)) < 2.0 ** -12
    deg = np.diff(A.rowptr).astype(np.float64)
    ref, S2 = oracle.spmm(A.rowptr, A.col, a_bits, Y, bf16=True)
    err = oracle.graded_error(C.cpu().numpy(), ref, S2, np.maximum(deg, 1)[:, None])
    assert err <= bound(TOL_F16, deg.max())


# ------------------------------------------- reduced instances of configs 2-4
@pytest.mark.parametrize("name,N,K", [("powerlaw", 128, 32), ("community", 64, 64), ("irregular", 32, 32)])
def test_small_instances_of_the_configs(name, N, K):
    A = wl.make(name, small=True)
    B = wl.dense_normal(A.Kc, N, seed=31)
    C, st = gpu_spmm(A, B)
    check_spmm(A, B, C, TOL_F16)
    X = wl.dense_normal(A.M, K, seed=32)
    Y = wl.dense_normal(A.Kc, K, seed=33)
    out, _ = gpu_sddmm(A, X, Y)
    check_sddmm(A, X, Y, out, TOL_F16)


# ------------------------------------- full-size configs, sampled against the oracle
@functools.lru_cache(maxsize=1)
def _full(name):
    return wl.make(name)


def _sample_rows(A, n, seed):
    rng = np.random.default_rng(seed)
    deg = np.diff(A.rowptr)
    heavy = np.argsort(deg)[-32:]
    return np.unique(np.concatenate([rng.integers(0, A.M, size=n), heavy, [0, A.M - 1]])).astype(np.int64)


def _plan_invariants(p, A):
    """Properties that hold at any size: every nonzero on exactly one path, values in place."""
    for which in (0, 1):
        try:
            ex = p.export(which)
        except lb.LibraError:
            continue
        seen = np.zeros(A.nnz, dtype=np.uint8)
        np.add.at(seen, ex["dense_perm"], 1)
        np.add.at(seen, ex["res_perm"], 1)
        assert seen.min() == 1 and seen.max() == 1
        assert np.array_equal(ex["dense_val"], A.val[ex["dense_perm"]])
        assert np.array_equal(ex["res_col"], A.col[ex["res_perm"]])


def test_full_powerlaw_config_as_benchmarked():
    A = _full("powerlaw")
    N, K = 128, 32
    B = wl.dense_normal(A.Kc, N, seed=wl.BASE_SEED + 201)
    _plan_invariants(lb.Plan.from_csr(A), A)
    # the benchmark runs on the plan the device planner writes straight into device memory
    p = lb.Plan.from_device_csr(A.M, A.Kc, dev(A.rowptr.astype(np.int32)), dev(A.col.astype(np.int32)), dev(A.val),
                                resident=True, keep_host_copy=False)
    C = p.spmm(dev(B))
    torch.cuda.synchronize()
    check_spmm_all_rows(A, B, C, TOL_F16)        # all 131,072 x 128 outputs, element by element
    X = wl.dense_normal(A.M, K, seed=wl.BASE_SEED + 202)
    Y = wl.dense_normal(A.Kc, K, seed=wl.BASE_SEED + 203)
    out = p.sddmm(dev(X), dev(Y)).cpu().numpy()
    check_sddmm(A, X, Y, out, TOL_F16)           # all 3.7 M outputs
    p.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_full_powerlaw_config_other_value_types_all_outputs(dtype):
    """Config 2 at full size in the two other storage types (the fp32 mode to its own bar of 1e-5): every output of both
    operators, on the plan the device planner writes."""
    A = _full("powerlaw")
    N, K = 128, 32
    B32 = wl.dense_normal(A.Kc, N, seed=wl.BASE_SEED + 211, dtype=np.float32)
    X32 = wl.dense_normal(A.M, K, seed=wl.BASE_SEED + 212, dtype=np.float32)
    Y32 = wl.dense_normal(A.Kc, K, seed=wl.BASE_SEED + 213, dtype=np.float32)
    v32 = wl.uniform_values(np.random.default_rng(214), A.nnz).astype(np.float32) * 1.37      # not exact in 8 bits
    rp, col = dev(A.rowptr.astype(np.int32)), dev(A.col.astype(np.int32))
    if dtype == "bf16":
        val, B, X, Y = (wl.to_bf16_bits(a) for a in (v32, B32, X32, Y32))
        p = lb.Plan.from_device_csr(A.M, A.Kc, rp, col, dev_bf16(val), resident=True, keep_host_copy=False)
        Bd, Xd, Yd, tol, bf = dev_bf16(B), dev_bf16(X), dev_bf16(Y), TOL_F16, True
    else:
        val, B, X, Y = v32, B32, X32, Y32
        p = lb.Plan.from_device_csr(A.M, A.Kc, rp, col, dev(val), resident=True, keep_host_copy=False)
        Bd, Xd, Yd, tol, bf = dev(B), dev(X), dev(Y), TOL_F32, False
    st = p.stats()
    assert 0 < st["spmm_dense_nnz"] < A.nnz and st["spmm_zero_rows"] > 0
    C = p.spmm(Bd)
    torch.cuda.synchronize()
    check_spmm_all_rows(A, B, C, tol, val=val, bf16=bf)
    out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    p.sddmm(Xd, Yd, out=out)
    ref, S = oracle.sddmm(A.rowptr, A.col, val, X, Y, bf16=bf)
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    assert oracle.graded_error(got, ref, S, K) <= bound(tol, K)
    p.close()


@pytest.mark.parametrize("N", [64, 128, 256])
def test_full_community_config_spmm_all_rows(N):
    """Config 3 at each of its three widths (N = 256 writes a 1 GiB C in one launch of two column pieces per task):
    every output against the oracle."""
    A = _full("community")
    p = lb.Plan.from_csr(A, flags=lb.FLAG_NO_SDDMM).upload()
    if N == 64:
        _plan_invariants(p, A)
    B = wl.dense_normal(A.Kc, N, seed=wl.BASE_SEED + 300 + N)
    C = p.spmm(dev(B))
    torch.cuda.synchronize()
    err = check_spmm_all_rows(A, B, C, TOL_F16)
    print(f"community N={N}: graded error {err:.2e} over all rows", flush=True)
    p.close()


@pytest.mark.parametrize("K", [32, 64])
def test_full_community_config_sddmm_all_outputs(K):
    A = _full("community")
    p = lb.Plan.from_csr(A, flags=lb.FLAG_NO_SPMM).upload()
    st = p.stats()
    assert 0 < st["sddmm_dense_nnz"] < A.nnz                    # both paths carry a share of this matrix
    X = wl.dense_normal(A.M, K, seed=wl.BASE_SEED + 310 + K)
    Y = wl.dense_normal(A.Kc, K, seed=wl.BASE_SEED + 311 + K)
    out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    p.sddmm(dev(X), dev(Y), out=out)
    check_sddmm(A, X, Y, out.cpu().numpy(), TOL_F16)            # all 22.2 M outputs
    p.close()


def test_full_irregular_config_all_outputs():
    """Config 4: 2.4 M rows, shifted-Zipf degrees up to 100 000 (row splitting, atomics), N = K = 32; every output of both
    operators against the oracle."""
    A = _full("irregular")
    p = lb.Plan.from_csr(A).upload()
    st = p.stats()
    assert st["spmm_split_rows"] > 1000 and st["spmm_chunk_tasks"] > 100_000
    _plan_invariants(p, A)
    B = wl.dense_normal(A.Kc, 32, seed=wl.BASE_SEED + 401)
    C = p.spmm(dev(B))
    torch.cuda.synchronize()
    # rows of up to 1e5 terms accumulated in chunks with atomics: the stated bar over all rows ...
    deg = np.diff(A.rowptr).astype(np.float64)
    worst = 0.0
    for r0 in range(0, A.M, 1 << 18):
        rows = np.arange(r0, min(A.M, r0 + (1 << 18)), dtype=np.int64)
        ref, S = oracle.spmm(A.rowptr, A.col, A.val, B, rows=rows)
        got = C[r0:r0 + rows.size].cpu().numpy()
        d = np.maximum(deg[rows], 1)[:, None]
        per = np.abs(got - ref) / np.maximum(np.abs(ref), S / np.sqrt(d))
        assert np.all(np.isfinite(got))
        worst = max(worst, float(per.max()))
        # ... and the derived bound row by row (a row of d terms may err by 16 sqrt(d) 2^-24 of its natural size)
        assert np.all(per.max(axis=1) <= 16.0 * np.sqrt(d[:, 0]) * 2.0 ** -24), f"rows {r0}.."
    assert worst <= TOL_F16, worst
    del C
    X = wl.dense_normal(A.M, 32, seed=wl.BASE_SEED + 402)
    Y = wl.dense_normal(A.Kc, 32, seed=wl.BASE_SEED + 403)
    out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    p.sddmm(dev(X), dev(Y), out=out)
    check_sddmm(A, X, Y, out.cpu().numpy(), TOL_F16)            # all 119.6 M outputs
    p.close()


def test_full_gat_config_all_four_heads():
    """Config 5: the four attention heads on the 2^20-node R-MAT graph, each SDDMM K=64 -> softmax -> new values -> SpMM
    N=64 on the one plan (built once, Section 4.1); every step of every head against the oracle on all of its outputs."""
    A = _full("gat")
    K = 64
    scale = 1.0 / np.sqrt(K)
    p = lb.Plan.from_csr(A).upload()
    _plan_invariants(p, A)
    deg = np.diff(A.rowptr)
    rows_of = np.repeat(np.arange(A.M), deg)
    ones = torch.from_numpy(A.val).cuda()
    for head in range(4):
        X = wl.dense_normal(A.M, K, seed=wl.BASE_SEED + 501 + 10 * head)
        Y = wl.dense_normal(A.Kc, K, seed=wl.BASE_SEED + 502 + 10 * head)
        Yd = dev(Y)
        p.set_values(ones, lb.OP_SDDMM)                         # the scores are taken on the graph itself (unit values)
        scores = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
        p.sddmm(dev(X), Yd, out=scores)
        alpha = p.edge_softmax(scores, scale)
        p.set_values(alpha, lb.OP_SPMM)
        C = p.spmm(Yd)
        torch.cuda.synchronize()
        sc = scores.cpu().numpy()
        al = alpha.cpu().numpy()
        check_sddmm(A, X, Y, sc, TOL_F16)                       # all 60.7 M scores
        # softmax of the GPU's own scores, all rows: the oracle's row softmax in double, one rounding to fp16
        want = oracle.edge_softmax(A.rowptr, sc.astype(np.float64), scale)
        assert np.max(np.abs(al.astype(np.float64) - want) / np.maximum(want, 2.0 ** -14)) < 4e-3
        sums = np.bincount(rows_of, weights=al.astype(np.float64), minlength=A.M)
        assert np.all(np.abs(sums[deg > 0] - 1.0) <= 2.0 ** -11 * np.maximum(deg[deg > 0], 4))
        # SpMM with the GPU's alpha as values, all rows
        err = check_spmm_all_rows(A, Y, C, TOL_F16, val=al)
        print(f"head {head}: SpMM graded error {err:.2e} over all rows", flush=True)
        del C, scores, alpha
    p.close()


def test_set_values_entry_point_refreshes_both_operators():
    """libra_plan_set_values itself (one call for both sub-plans), on a plan that uses both paths of both operators."""
    A = wl.make("community", small=True)
    B, X, Y = wl.dense_normal(A.Kc, 64, seed=41), wl.dense_normal(A.M, 32, seed=42), wl.dense_normal(A.Kc, 32, seed=43)
    v2 = wl.uniform_values(np.random.default_rng(44), A.nnz)
    p = lb.Plan.from_csr(A).upload()
    st = p.stats()
    assert 0 < st["spmm_dense_nnz"] < A.nnz and 0 < st["sddmm_dense_nnz"] < A.nnz
    lb.libra_plan_set_values(p.handle, dev(v2).data_ptr(), lb.F16, torch.cuda.current_stream().cuda_stream)
    check_spmm(A, B, p.spmm(dev(B)).cpu().numpy(), TOL_F16, val=v2)
    check_sddmm(A, X, Y, p.sddmm(dev(X), dev(Y)).cpu().numpy(), TOL_F16, val=v2)
    p.set_values(dev(A.val), one_call=True)                     # the wrapper's route to the same entry point
    check_spmm(A, B, p.spmm(dev(B)).cpu().numpy(), TOL_F16)
    check_sddmm(A, X, Y, p.sddmm(dev(X), dev(Y)).cpu().numpy(), TOL_F16)
    with pytest.raises(lb.LibraError) as e:
        lb.libra_plan_set_values(p.handle, dev(v2).data_ptr(), lb.F32, 0)
    assert e.value.code == lb.ERR["DTYPE"]
    p.close()


# ---------------------------------------------- seeded sweep over shapes, value types, modes, orders and both planners
def test_seeded_sweep_of_shapes_types_modes_and_planners():
    """Small matrices of drawn shape and density (some with a long row), drawn feature widths, value type, mode and
    order flags, planned on the host and on the device; SpMM and SDDMM against the oracle, then again after new values."""
    rng = np.random.default_rng(20250622)
    for it in range(24):
        M, Kc = int(rng.integers(1, 700)), int(rng.integers(8, 600))
        density = float(rng.choice([0.002, 0.01, 0.05, 0.2, 0.5]))
        A = wl.random_pattern(M, Kc, density, seed=int(rng.integers(1 << 30)), empty_rows=float(rng.choice([0, 0.3])))
        if M > 8 and Kc > 300 and rng.random() < 0.5:
            A = wl.with_long_rows(A, [int(rng.integers(0, M))], int(rng.integers(100, Kc)), seed=it)
        f32 = bool(rng.random() < 0.3)
        N = int(rng.choice([1, 2, 3, 4, 8])) * (16 if f32 else 32)
        K = int(rng.choice([32, 64, 128]))
        mode = int(rng.choice([lb.MODE_HYBRID, lb.MODE_HYBRID, lb.MODE_DENSE_ONLY, lb.MODE_SCALAR_ONLY]))
        flags = int(rng.choice([0, lb.FLAG_XCD_ORDER, lb.FLAG_NO_XCD_ORDER, lb.FLAG_SEGMENTS_BY_COST, lb.FLAG_TWO_KERNELS]))
        dt, tol = (np.float32, TOL_F32) if f32 else (np.float16, TOL_F16)
        share = (0, 40, 80)[it % 3]             # the dense-share rule of the SDDMM sub-plan: off, and two thresholds
        val = A.val.astype(dt)
        B, X, Y = (wl.dense_normal(r, c, seed=it + s).astype(dt) for r, c, s in ((A.Kc, N, 100), (A.M, K, 200), (A.Kc, K, 300)))
        new_val = wl.uniform_values(np.random.default_rng(it), A.nnz).astype(dt)
        for planner in ("host", "device"):
            if planner == "device" and A.nnz == 0:
                continue
            if planner == "host":
                p = lb.Plan(A.M, A.Kc, A.rowptr, A.col, val, mode=mode, flags=flags, sddmm_min_dense_pct=share).upload()
            else:
                rp, col, v = (dev(x) for x in (A.rowptr.astype(np.int32), A.col.astype(np.int32), val))
                p = lb.Plan.from_device_csr(A.M, A.Kc, rp, col, v, resident=True, keep_host_copy=False, mode=mode, flags=flags, sddmm_min_dense_pct=share)
            where = f"case {it} ({planner} planner): M={M} Kc={Kc} nnz={A.nnz} f32={f32} N={N} K={K} mode={mode} flags={flags} share={share}"
            out = torch.full((A.nnz,), float("nan"), dtype=torch.float32, device="cuda")
            for values in (val, new_val):
                if values is new_val:
                    if A.nnz == 0:
                        break
                    p.set_values(dev(new_val))
                try:
                    check_spmm(A, B, p.spmm(dev(B)).cpu().numpy(), tol, val=values)
                    if A.nnz:
                        p.sddmm(dev(X), dev(Y), out=out)
                        check_sddmm(A, X, Y, out.cpu().numpy(), tol, val=values)
                except AssertionError as e:
                    raise AssertionError(f"{where}: {e}") from e
            p.close()
