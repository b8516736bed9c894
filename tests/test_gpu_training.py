"""Training-side use of the operators (Section 5.5 of the paper trains GNNs with them): the transposed pattern,
SDDMM without A's values, the softmax gradient, and the chain rule on top of them, each against the CPU oracle
applied to the textbook formula of the gradient."""
import numpy as np
import pytest

import oracle
from paper_2506_22714_amd import binding as lb
from paper_2506_22714_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    lb.lib()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def transpose_host(A):
    """Plain definition: nonzeros listed column by column, rows ascending."""
    rows = np.repeat(np.arange(A.M, dtype=np.int64), np.diff(A.rowptr))
    order = np.lexsort((rows, A.col))
    rowptr_t = np.zeros(A.Kc + 1, dtype=np.int32)
    np.cumsum(np.bincount(A.col, minlength=A.Kc), out=rowptr_t[1:])
    return wl.Csr(A.Kc, A.M, rowptr_t, rows[order].astype(np.int32), A.val[order]), order


def assert_close_after_fp16_rounding(got, ref, S, d):
    """The wrapper rounds a gradient once to fp16: half an ulp of the value (2^-11 relative, or 2^-25 absolute in the
    subnormal range) on top of the kernel's fp32 accumulation error, graded as in the parity tests."""
    lim = 2.0 ** -10 * np.maximum(np.abs(ref), S / np.sqrt(np.maximum(d, 1.0))) + 2.0 ** -24
    assert np.all(np.abs(got - ref) <= lim), float(np.max(np.abs(got - ref) - lim))


def graft(A):
    return wl.with_long_rows(wl.random_pattern(300, 260, 0.03, seed=4, empty_rows=0.2), [7, 150], 200, seed=5) if A is None else A


def test_transposed_pattern_matches_the_definition():
    for A in (graft(None), wl.make("powerlaw", small=True), wl.random_pattern(1, 40, 0.5, seed=2), wl.random_pattern(50, 3, 0.4, seed=3)):
        At, order = transpose_host(A)
        rp_t, col_t, perm_t = lb.transpose_csr(A.M, A.Kc, dev(A.rowptr.astype(np.int32)), dev(A.col.astype(np.int32)))
        assert np.array_equal(rp_t.cpu().numpy(), At.rowptr)
        assert np.array_equal(col_t.cpu().numpy(), At.col)
        assert np.array_equal(perm_t.cpu().numpy(), order)
    # no nonzeros: all offsets zero
    rp_t, col_t, perm_t = lb.transpose_csr(4, 6, torch.zeros(5, dtype=torch.int32, device="cuda"), torch.zeros(0, dtype=torch.int32, device="cuda"))
    assert rp_t.cpu().tolist() == [0] * 7 and col_t.numel() == 0


@pytest.mark.parametrize("K", [32, 128])
def test_sddmm_without_values(K):
    A = graft(None)
    X, Y = wl.dense_normal(A.M, K, seed=1), wl.dense_normal(A.Kc, K, seed=2)
    p = lb.Plan.from_csr(A, flags=lb.FLAG_NO_SPMM, sddmm_min_blk_nnz=8).upload()
    assert 0 < p.stats()["sddmm_dense_nnz"] < A.nnz
    out = p.sddmm(dev(X), dev(Y), pattern_only=True).cpu().numpy()
    ref, S = oracle.sddmm(A.rowptr, A.col, np.ones(A.nnz, dtype=np.float16), X, Y)
    assert oracle.graded_error(out, ref, S, K) <= 16 * np.sqrt(K) * 2.0 ** -24


@pytest.mark.parametrize("adt", ["f16", "f32", "bf16"])
def test_edge_softmax_backward(adt):
    A = wl.make("gat", small=True)              # rows of every length class
    deg = np.diff(A.rowptr)
    assert deg.max() > 2048 and ((deg > 64) & (deg <= 2048)).any()
    rng = np.random.default_rng(3)
    scores = rng.standard_normal(A.nnz).astype(np.float32)
    dalpha = rng.standard_normal(A.nnz).astype(np.float32)
    scale = 0.7
    p = lb.Plan.from_csr(A).upload()
    tdt = {"f16": torch.float16, "f32": torch.float32, "bf16": torch.bfloat16}[adt]
    alpha = p.edge_softmax(dev(scores), scale, out=torch.empty(A.nnz, dtype=tdt, device="cuda"))
    ds = p.edge_softmax_backward(alpha, dev(dalpha), scale).cpu().numpy().astype(np.float64)
    a = alpha.float().cpu().numpy().astype(np.float64)       # the kernel's own (rounded) alpha: the formula is checked, not the rounding
    rows = np.repeat(np.arange(A.M), deg)
    dot = np.bincount(rows, weights=a * dalpha, minlength=A.M)
    ref = scale * a * (dalpha - dot[rows])
    sabs = np.bincount(rows, weights=np.abs(a * dalpha), minlength=A.M)
    tol = 32 * np.sqrt(deg.max()) * 2.0 ** -24
    assert np.max(np.abs(ds - ref) / (scale * a * (np.abs(dalpha) + sabs[rows]) + 1e-30)) <= tol


def test_spmm_and_sddmm_gradients_match_the_formulas():
    from paper_2506_22714_amd import autograd as ag
    A = graft(None)
    At, order = transpose_host(A)
    N = 64
    sm = ag.SparseMatrix(A.M, A.Kc, dev(A.rowptr.astype(np.int32)), dev(A.col.astype(np.int32)), cs=50)
    assert np.array_equal(sm.perm_t.cpu().numpy(), order)
    vals = dev(A.val).requires_grad_()
    Bn = wl.dense_normal(A.Kc, N, seed=11)
    B = dev(Bn).requires_grad_()
    C = ag.spmm(sm, vals, B)
    ref, S = oracle.spmm(A.rowptr, A.col, A.val, Bn)
    deg = np.diff(A.rowptr).astype(np.float64)
    assert oracle.graded_error(C.detach().cpu().numpy(), ref, S, deg[:, None]) <= 16 * np.sqrt(deg.max()) * 2.0 ** -24
    dCn = wl.dense_normal(A.M, N, seed=12)              # an upstream gradient that is exact in fp16
    C.backward(dev(dCn).float())
    # dB = A^T dC
    ref, S = oracle.spmm(At.rowptr, At.col, At.val, dCn)
    degt = np.diff(At.rowptr).astype(np.float64)
    got = B.grad.float().cpu().numpy()                 # rounded to fp16 once by the wrapper
    assert_close_after_fp16_rounding(got, ref, S, degt[:, None])
    # dA_p = <dC_i, B_j>
    ref, S = oracle.sddmm(A.rowptr, A.col, np.ones(A.nnz, dtype=np.float16), dCn, Bn)
    got = vals.grad.float().cpu().numpy()
    assert_close_after_fp16_rounding(got, ref, S, N)

    # SDDMM: out_p = A_p <X_i, Y_j>
    K = 32
    Xn, Yn = wl.dense_normal(A.M, K, seed=13), wl.dense_normal(A.Kc, K, seed=14)
    X, Y = dev(Xn).requires_grad_(), dev(Yn).requires_grad_()
    vals2 = dev(A.val).requires_grad_()
    out = ag.sddmm(sm, vals2, X, Y)
    ref, S = oracle.sddmm(A.rowptr, A.col, A.val, Xn, Yn)
    assert oracle.graded_error(out.detach().cpu().numpy(), ref, S, K) <= 16 * np.sqrt(K) * 2.0 ** -24
    dout = (np.random.default_rng(15).integers(-4, 5, size=A.nnz) / 4.0).astype(np.float32)
    out.backward(dev(dout))
    g = (dout.astype(np.float64) * A.val.astype(np.float64)).astype(np.float16)                  # what the wrapper feeds the kernels
    ref, S = oracle.spmm(A.rowptr, A.col, g, Yn)                                                  # dX = (A o dout) Y
    got = X.grad.float().cpu().numpy()
    assert_close_after_fp16_rounding(got, ref, S, deg[:, None])
    ref, S = oracle.spmm(At.rowptr, At.col, g[order], Xn)                                         # dY = (A o dout)^T X
    got = Y.grad.float().cpu().numpy()
    assert_close_after_fp16_rounding(got, ref, S, degt[:, None])
    ref, S = oracle.sddmm(A.rowptr, A.col, np.ones(A.nnz, dtype=np.float16), Xn, Yn)              # dA_p = dout_p <X_i, Y_j>
    got = vals2.grad.float().cpu().numpy()
    assert_close_after_fp16_rounding(got, dout * ref, np.abs(dout) * S, K)
    sm.close()


def test_fp32_gradients_run_on_both_paths():
    """The same chain rule with fp32 storage (dense tiles on the fp32 matrix instruction): nothing is rounded on the way,
    so every gradient meets the derived bound directly."""
    from paper_2506_22714_amd import autograd as ag
    A = graft(None)
    At, order = transpose_host(A)
    N = 64
    sm = ag.SparseMatrix(A.M, A.Kc, dev(A.rowptr.astype(np.int32)), dev(A.col.astype(np.int32)), dtype=torch.float32, cs=50)
    st = sm.plan.stats()
    assert st["spmm_dense_nnz"] > 0 and st["spmm_res_nnz"] > 0
    v32 = A.val.astype(np.float32)
    vals = dev(v32).requires_grad_()
    Bn = wl.dense_normal(A.Kc, N, seed=11, dtype=np.float32)
    B = dev(Bn).requires_grad_()
    C = ag.spmm(sm, vals, B)
    deg = np.diff(A.rowptr).astype(np.float64)
    degt = np.diff(At.rowptr).astype(np.float64)
    tol = lambda d: 16 * np.sqrt(d) * 2.0 ** -24
    ref, S = oracle.spmm(A.rowptr, A.col, v32, Bn)
    assert oracle.graded_error(C.detach().cpu().numpy(), ref, S, deg[:, None]) <= tol(deg.max())
    dCn = wl.dense_normal(A.M, N, seed=12, dtype=np.float32)
    C.backward(dev(dCn))
    ref, S = oracle.spmm(At.rowptr, At.col, v32[order], dCn)                       # dB = A^T dC
    assert oracle.graded_error(B.grad.cpu().numpy(), ref, S, degt[:, None]) <= tol(degt.max())
    ref, S = oracle.sddmm(A.rowptr, A.col, np.ones(A.nnz, dtype=np.float32), dCn, Bn)    # dA_p = <dC_i, B_j>
    assert oracle.graded_error(vals.grad.cpu().numpy(), ref, S, N) <= tol(N)
    sm.close()


def train_layers(kind, n_layers, steps=12):
    """Optimiser steps of an n-layer graph network on a synthetic power-law graph; returns the losses.  `gcn`: every layer
    is SpMM with the fixed symmetric normalisation 1/sqrt(d_i d_j) (Section 5.5's GCN); `agnn`: every layer is SDDMM ->
    edge softmax -> SpMM with learned attention (its AGNN); layers are residual.  The dense layers are torch matmuls (not part of the library)."""
    from paper_2506_22714_amd import autograd as ag
    torch.manual_seed(0)
    A = wl.make("powerlaw", small=True)
    sm = ag.SparseMatrix(A.M, A.Kc, dev(A.rowptr.astype(np.int32)), dev(A.col.astype(np.int32)))
    F = 32
    feats = dev(wl.dense_normal(A.M, F, seed=5)).float()
    labels = feats[:, :4].argmax(dim=1)           # a target the features determine; residual layers keep it reachable
    Ws = [(torch.randn(F, F, device="cuda") * (0.2 if kind == "agnn" else 0.35)).requires_grad_() for _ in range(n_layers)]
    Wc = (torch.randn(F, 4, device="cuda") * 0.2).requires_grad_()
    ones = torch.ones(sm.nnz, dtype=torch.float16, device="cuda")
    deg = np.maximum(np.diff(A.rowptr), 1).astype(np.float64)
    rows = np.repeat(np.arange(A.M), np.diff(A.rowptr))
    norm = dev((1.0 / np.sqrt(deg[rows] * deg[A.col])).astype(np.float16))
    opt = torch.optim.Adam(Ws + [Wc], lr=2e-2)
    losses = []
    for step in range(steps):
        h = feats
        for Wl in Ws:
            z = (h @ Wl).half()
            if kind == "agnn":
                scores = ag.sddmm(sm, ones, z, z)
                alpha = ag.edge_softmax(sm, scores, 1.0 / np.sqrt(F))
                h = h + torch.relu(ag.spmm(sm, alpha, z))
            else:
                h = h + torch.relu(ag.spmm(sm, norm, z))
        loss = torch.nn.functional.cross_entropy(h @ Wc, labels)
        opt.zero_grad()
        loss.backward()
        assert all(torch.isfinite(w.grad).all() for w in Ws + [Wc])
        opt.step()
        losses.append(float(loss.detach()))
    sm.close()
    return losses


@pytest.mark.parametrize("kind,n_layers", [("agnn", 2), ("agnn", 5), ("gcn", 5)])
def test_graph_networks_train(kind, n_layers):
    """The end-to-end use of Section 5.5 (five-layer GCN and AGNN) on a synthetic graph: the loss goes down and every
    gradient is finite."""
    losses = train_layers(kind, n_layers)
    print(kind, n_layers, "losses", [round(x, 4) for x in losses], flush=True)
    assert losses[-1] < losses[0] - 0.02


def test_matrix_cores_and_vector_alus_run_side_by_side():
    """Section 3.1 of the paper on this GPU: MFMA waves and FMA waves sharing the SIMDs overlap almost completely."""
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    a, b, both = lb.libra_probe_coissue(20000, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
    print(f"coissue probe: MFMA only {a:.1f} us, FMA only {b:.1f} us, both {both:.1f} us", flush=True)
    assert a > 50 and b > 50
    assert both < 0.8 * (a + b)            # far from exclusive


def test_gather_probes_run_on_every_row_width_with_and_without_resident_rows():
    """The bare-gather measurement aids: plain fetches, fetches from a table small enough to hit in the L2s, and the variant
    that keeps the most referenced rows in LDS (negative indices are LDS slots; indices outside the table or the slots
    are clamped or read as zeros by construction, so a wrong index cannot fault)."""
    A = wl.make("powerlaw", small=True)
    stream = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    col = torch.from_numpy(A.col.astype(np.int32)).cuda()
    popularity = np.bincount(A.col, minlength=A.Kc)
    for rb in (64, 128, 256):
        table = torch.randn(A.Kc, rb // 2, device="cuda").half()
        n_hub = min(A.Kc, (96 << 10) // rb)
        hub = np.argsort(-popularity, kind="stable")[:n_hub].astype(np.int32)
        slot = np.full(A.Kc, -1, dtype=np.int64)
        slot[hub] = np.arange(n_hub)
        s_of = slot[A.col]
        enc = np.where(s_of >= 0, -1 - s_of, A.col).astype(np.int32)
        enc[:3] = [A.Kc + 5, -1 - n_hub - 7, np.iinfo(np.int32).max]      # outside the table / the slots: harmless
        enc_d, hub_d = torch.from_numpy(enc).cuda(), torch.from_numpy(hub).cuda()
        lb.libra_probe_gather(table.data_ptr(), A.Kc, rb, col.data_ptr(), A.nnz, sink.data_ptr(), stream)
        lb.libra_probe_gather_hub(table.data_ptr(), A.Kc, rb, col.data_ptr(), A.nnz, 0, 0, sink.data_ptr(), stream)
        lb.libra_probe_gather_hub(table.data_ptr(), A.Kc, rb, enc_d.data_ptr(), A.nnz, hub_d.data_ptr(), n_hub, sink.data_ptr(), stream)
        torch.cuda.synchronize()
        assert float(sink.item()) in (0.0, 1.0)
