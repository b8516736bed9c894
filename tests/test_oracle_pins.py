"""Pins for the CPU oracle: it is checked against things other than itself -
numpy / scipy library routines on the plain definition, closed forms and
invariants - so that a dropped term, a wrong index or a transposed operand
fails at least one test.  CPU only."""
import numpy as np
import pytest
import scipy.sparse as sps
import scipy.special

import oracle
from paper_2506_22714_amd import workloads as wl


def dense_of(A: wl.Csr) -> np.ndarray:
    D = np.zeros((A.M, A.Kc), dtype=np.float64)
    for i in range(A.M):
        s, e = A.rowptr[i], A.rowptr[i + 1]
        D[i, A.col[s:e]] = A.val[s:e].astype(np.float64)
    return D


# ---------------------------------------------------------------- conversions
def test_half_widening_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = oracle.widen(bits.view(np.float16))
    both_nan = np.isnan(want) & np.isnan(got)
    assert np.array_equal(want[~both_nan], got[~both_nan])
    assert both_nan.sum() == 2 * 1023
    # signed zero and subnormals keep their sign / exact value
    assert np.signbit(oracle.half_to_double(0x8000))
    assert oracle.half_to_double(0x0001) == 2.0 ** -24
    assert oracle.half_to_double(0x7BFF) == 65504.0


def test_bf16_widening():
    rng = np.random.default_rng(0)
    f = rng.standard_normal(1000).astype(np.float32)
    bits = (f.view(np.uint32) >> 16).astype(np.uint16)
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = oracle.widen(bits, bf16=True)
    assert np.array_equal(want, got)


# ---------------------------------------------------------------------- SpMM
@pytest.mark.parametrize("M,Kc,N,density", [(37, 53, 8, 0.2), (64, 64, 32, 0.1), (200, 120, 24, 0.05), (5, 300, 3, 0.5)])
def test_spmm_matches_dense_brute_force(M, Kc, N, density):
    A = wl.random_pattern(M, Kc, density, seed=M * 7 + Kc, empty_rows=0.2)
    B = wl.dense_normal(Kc, N, seed=11)
    C, S = oracle.spmm(A.rowptr, A.col, A.val, B)
    D = dense_of(A)
    want = D @ B.astype(np.float64)
    np.testing.assert_allclose(C, want, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S, np.abs(D) @ np.abs(B.astype(np.float64)), rtol=1e-13, atol=1e-13)


def test_spmm_identity_and_permutation():
    n, N = 97, 16
    B = wl.dense_normal(n, N, seed=3)
    I = wl.from_dense(np.eye(n))
    C, _ = oracle.spmm(I.rowptr, I.col, I.val, B)
    assert np.array_equal(C, B.astype(np.float64))
    perm = np.random.default_rng(5).permutation(n)
    P = np.zeros((n, n))
    P[np.arange(n), perm] = 1.0
    Pc = wl.from_dense(P)
    C, _ = oracle.spmm(Pc.rowptr, Pc.col, Pc.val, B)
    assert np.array_equal(C, B.astype(np.float64)[perm])


def test_spmm_ones_gives_row_sums_and_empty_rows_zero():
    A = wl.random_pattern(80, 60, 0.15, seed=9, empty_rows=0.3)
    B = np.ones((60, 5), dtype=np.float16)
    C, _ = oracle.spmm(A.rowptr, A.col, A.val, B)
    rs = np.array([A.val[A.rowptr[i]:A.rowptr[i + 1]].astype(np.float64).sum() for i in range(A.M)])
    np.testing.assert_allclose(C, np.repeat(rs[:, None], 5, axis=1), rtol=0, atol=1e-15)
    empty = np.flatnonzero(np.diff(A.rowptr) == 0)
    assert empty.size > 0 and np.all(C[empty] == 0.0)


def test_spmm_linearity_exact_on_small_integers():
    A = wl.random_pattern(50, 70, 0.2, seed=21)
    A.val = np.random.default_rng(1).integers(-3, 4, size=A.nnz).astype(np.float16)
    B1 = wl.dense_small_int(70, 12, seed=1)
    B2 = wl.dense_small_int(70, 12, seed=2)
    Bc = (2 * B1.astype(np.float32) + 0.5 * B2.astype(np.float32)).astype(np.float16)
    assert np.array_equal(Bc.astype(np.float32), 2 * B1.astype(np.float32) + 0.5 * B2.astype(np.float32))
    C1, _ = oracle.spmm(A.rowptr, A.col, A.val, B1)
    C2, _ = oracle.spmm(A.rowptr, A.col, A.val, B2)
    Cc, _ = oracle.spmm(A.rowptr, A.col, A.val, Bc)
    assert np.array_equal(Cc, 2 * C1 + 0.5 * C2)


def test_spmm_scipy_cross_check_on_tiny_config():
    A = wl.tiny()
    assert A.nnz == 32768 and np.all(np.diff(A.rowptr) == 16)
    B = wl.dense_normal(A.Kc, 32, seed=wl.BASE_SEED + 101)
    C, _ = oracle.spmm(A.rowptr, A.col, A.val, B)
    sp = sps.csr_matrix((A.val.astype(np.float64), A.col, A.rowptr), shape=(A.M, A.Kc))
    np.testing.assert_allclose(C, sp @ B.astype(np.float64), rtol=1e-12, atol=1e-12)


def test_spmm_row_subset_and_fp32_inputs():
    A = wl.random_pattern(120, 90, 0.1, seed=4)
    B = wl.dense_normal(90, 10, seed=6, dtype=np.float32)
    Cfull, Sfull = oracle.spmm(A.rowptr, A.col, A.val.astype(np.float32), B)
    rows = np.array([119, 0, 57, 57, 3], dtype=np.int64)
    Csub, Ssub = oracle.spmm(A.rowptr, A.col, A.val.astype(np.float32), B, rows=rows)
    assert np.array_equal(Csub, Cfull[rows]) and np.array_equal(Ssub, Sfull[rows])
    np.testing.assert_allclose(Cfull, dense_of(A) @ B.astype(np.float64), rtol=1e-13, atol=1e-13)


def test_spmm_threads_do_not_change_bits():
    A = wl.random_pattern(300, 200, 0.1, seed=8)
    B = wl.dense_normal(200, 16, seed=2)
    C1, _ = oracle.spmm(A.rowptr, A.col, A.val, B, nthreads=1)
    C4, _ = oracle.spmm(A.rowptr, A.col, A.val, B, nthreads=4)
    assert np.array_equal(C1, C4)


# --------------------------------------------------------------------- SDDMM
@pytest.mark.parametrize("M,Kc,K,density", [(33, 47, 8, 0.2), (64, 80, 32, 0.1), (10, 200, 64, 0.3)])
def test_sddmm_matches_dense_brute_force(M, Kc, K, density):
    A = wl.random_pattern(M, Kc, density, seed=M + Kc, empty_rows=0.1)
    X = wl.dense_normal(M, K, seed=1)
    Y = wl.dense_normal(Kc, K, seed=2)
    out, S = oracle.sddmm(A.rowptr, A.col, A.val, X, Y)
    full = dense_of(A) * (X.astype(np.float64) @ Y.astype(np.float64).T)
    fullS = np.abs(dense_of(A)) * (np.abs(X.astype(np.float64)) @ np.abs(Y.astype(np.float64)).T)
    rows = np.repeat(np.arange(M), np.diff(A.rowptr))
    np.testing.assert_allclose(out, full[rows, A.col], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S, fullS[rows, A.col], rtol=1e-13, atol=1e-13)


def test_sddmm_one_hot_rows_return_values_on_matches():
    # X[i] = e_{i mod K}, Y[j] = e_{j mod K}: <X_i, Y_j> = [i = j mod K]
    M, Kc, K = 40, 56, 8
    A = wl.random_pattern(M, Kc, 0.3, seed=77)
    X = np.zeros((M, K), dtype=np.float16)
    X[np.arange(M), np.arange(M) % K] = 1
    Y = np.zeros((Kc, K), dtype=np.float16)
    Y[np.arange(Kc), np.arange(Kc) % K] = 1
    out, _ = oracle.sddmm(A.rowptr, A.col, A.val, X, Y)
    rows = np.repeat(np.arange(M), np.diff(A.rowptr))
    want = np.where(rows % K == A.col % K, A.val.astype(np.float64), 0.0)
    assert np.array_equal(out, want)


def test_sddmm_row_sums_tie_to_spmm():
    # sum_p out[p] over row i  ==  X_i . (A Y)_i
    A = wl.random_pattern(60, 45, 0.2, seed=13)
    X = wl.dense_small_int(60, 16, seed=3)
    Y = wl.dense_small_int(45, 16, seed=4)
    A.val = np.random.default_rng(2).integers(-2, 3, size=A.nnz).astype(np.float16)
    A.val[A.val == 0] = 1
    out, _ = oracle.sddmm(A.rowptr, A.col, A.val, X, Y)
    AY, _ = oracle.spmm(A.rowptr, A.col, A.val, Y)
    lhs = np.array([out[A.rowptr[i]:A.rowptr[i + 1]].sum() for i in range(A.M)])
    rhs = (X.astype(np.float64) * AY).sum(axis=1)
    assert np.array_equal(lhs, rhs)


def test_sddmm_subset_equals_full():
    A = wl.random_pattern(90, 70, 0.15, seed=5)
    X = wl.dense_normal(90, 32, seed=1)
    Y = wl.dense_normal(70, 32, seed=2)
    out, S = oracle.sddmm(A.rowptr, A.col, A.val, X, Y)
    idx = np.random.default_rng(0).integers(0, A.nnz, size=50)
    o2, S2 = oracle.sddmm(A.rowptr, A.col, A.val, X, Y, idx=idx)
    assert np.array_equal(o2, out[idx]) and np.array_equal(S2, S[idx])


# ------------------------------------------------------------------- softmax
def test_edge_softmax_against_scipy_rows_and_invariants():
    A = wl.random_pattern(70, 50, 0.2, seed=31, empty_rows=0.2)
    rng = np.random.default_rng(3)
    s = rng.standard_normal(A.nnz) * 4
    a = oracle.edge_softmax(A.rowptr, s, scale=0.7)
    for i in range(A.M):
        lo, hi = A.rowptr[i], A.rowptr[i + 1]
        if hi > lo:
            np.testing.assert_allclose(a[lo:hi], scipy.special.softmax(0.7 * s[lo:hi]), rtol=1e-13)
            assert abs(a[lo:hi].sum() - 1.0) < 1e-14
    # shift invariance per row and the constant-score closed form 1/deg
    shift = np.repeat(rng.standard_normal(A.M), np.diff(A.rowptr))
    np.testing.assert_allclose(oracle.edge_softmax(A.rowptr, s + shift, 1.0), oracle.edge_softmax(A.rowptr, s, 1.0), rtol=1e-12)
    c = oracle.edge_softmax(A.rowptr, np.full(A.nnz, 3.25), 1.0)
    deg = np.repeat(np.diff(A.rowptr), np.diff(A.rowptr))
    np.testing.assert_allclose(c, 1.0 / deg, rtol=1e-15)


def test_attention_head_constant_features_give_neighbourhood_mean():
    # X = 0 -> all scores 0 -> alpha = 1/deg -> C = mean of B over the neighbours
    A = wl.random_pattern(40, 40, 0.2, seed=17)
    A.val = wl.unit_values(A.nnz)
    X = np.zeros((40, 8), dtype=np.float16)
    Y = wl.dense_normal(40, 8, seed=1)
    B = wl.dense_small_int(40, 8, seed=2)
    _s, a16, C, _S = oracle.attention_head(A.rowptr, A.col, A.val, X, Y, B, scale=0.5)
    for i in range(A.M):
        lo, hi = A.rowptr[i], A.rowptr[i + 1]
        if hi > lo:
            w = np.float64(np.float16(1.0 / (hi - lo)))
            np.testing.assert_allclose(C[i], w * B[A.col[lo:hi]].astype(np.float64).sum(axis=0), rtol=1e-12)


def test_attention_head_against_dense_softmax_with_nonzero_features():
    # scores are kept as fp32 (the kernel's output type) before the softmax, the scale multiplies the scores inside
    # the exponential, alpha is rounded once to fp16: every step redone with dense numpy / scipy on a small graph
    from scipy.special import softmax
    M = Kc = 48
    K = 8
    A = wl.random_pattern(M, Kc, 0.25, seed=23)
    rng = np.random.default_rng(5)
    A.val = wl.uniform_values(rng, A.nnz)
    X = wl.dense_normal(M, K, seed=3)
    Y = wl.dense_normal(Kc, K, seed=4)
    B = wl.dense_normal(Kc, 8, seed=6)
    scale = 0.37
    s32, a16, C, _S = oracle.attention_head(A.rowptr, A.col, A.val, X, Y, B, scale=scale)
    assert s32.dtype == np.float32 and a16.dtype == np.float16
    D = np.zeros((M, Kc))
    for i in range(M):
        D[i, A.col[A.rowptr[i]:A.rowptr[i + 1]]] = A.val[A.rowptr[i]:A.rowptr[i + 1]].astype(np.float64)
    full = D * (X.astype(np.float64) @ Y.astype(np.float64).T)          # scores on the pattern, exact products in double
    want_C = np.zeros((M, B.shape[1]))
    changed_by_scale = 0
    for i in range(M):
        lo, hi = A.rowptr[i], A.rowptr[i + 1]
        if hi == lo:
            assert not C[i].any()
            continue
        cols = A.col[lo:hi]
        sc = full[i, cols].astype(np.float32)                            # one rounding to fp32
        np.testing.assert_array_equal(s32[lo:hi], sc)
        alpha = softmax(scale * sc.astype(np.float64))
        np.testing.assert_array_equal(a16[lo:hi], alpha.astype(np.float16))
        changed_by_scale += int(np.any(softmax(sc.astype(np.float64)).astype(np.float16) != a16[lo:hi]))
        want_C[i] = alpha.astype(np.float16).astype(np.float64) @ B[cols].astype(np.float64)
    np.testing.assert_allclose(C, want_C, rtol=1e-13, atol=1e-15)
    assert changed_by_scale > M // 2        # a dropped or misplaced scale would be seen


# ------------------------------------------------------------- error measure
def test_graded_error_is_relative_for_ordinary_outputs_and_scaled_for_cancelled():
    ref = np.array([1.0, 1e-9])
    S = np.array([4.0, 4.0])
    got = ref + np.array([1e-3, 1e-3])
    e = oracle.graded_error(got, ref, S, 16)
    assert abs(e - 1e-3) < 1e-12            # second entry: 1e-3 / (4/4) = 1e-3 as well
    assert oracle.graded_error(ref, ref, S, 16) == 0.0
