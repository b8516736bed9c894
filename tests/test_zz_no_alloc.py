"""The allocation-free transposition (libra_csr_transpose_device_static: its workspace is a fixed array in the library's
device image) against the entry point that takes a caller's workspace, through the C ABI: identical outputs (integer
work), on two calls in a row, the second with a smaller matrix, so that whatever the first call left in the shared
array is there when the second one runs."""
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


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _outputs(A):
    return (torch.full((A.Kc + 1,), -7, dtype=torch.int32, device="cuda"), torch.full((max(A.nnz, 1),), -7, dtype=torch.int32, device="cuda"),
            torch.full((max(A.nnz, 1),), -7, dtype=torch.int32, device="cuda"))


def _with_workspace(A, rp, col):
    rpt, ct, pt = _outputs(A)
    nb = lb.libra_csr_transpose_workspace(A.nnz)
    ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
    lb.libra_csr_transpose_device(A.M, A.Kc, A.nnz, rp.data_ptr(), col.data_ptr(), rpt.data_ptr(), ct.data_ptr(), pt.data_ptr(),
                                  ws.data_ptr(), nb, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return rpt, ct, pt


def _static(A, rp, col):
    rpt, ct, pt = _outputs(A)
    lb.libra_csr_transpose_device_static(A.M, A.Kc, A.nnz, rp.data_ptr(), col.data_ptr(), rpt.data_ptr(), ct.data_ptr(), pt.data_ptr(),
                                         torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return rpt, ct, pt


def test_static_transposition_equals_the_workspace_one_on_two_calls_in_a_row():
    big = wl.rmat(scale=15, avg_degree=12, seed=71)                # ~0.7 M nonzeros, near the array's limit
    small = wl.random_pattern(301, 977, 0.02, seed=72, empty_rows=0.2)   # ragged shapes, empty rows and columns
    assert small.nnz < big.nnz <= lb.TRANSPOSE_STATIC_MAX_NNZ
    for A in (big, small):
        rp, col = _dev(A.rowptr), _dev(A.col)
        want = _with_workspace(A, rp, col)
        got = _static(A, rp, col)
        for w, g, name in zip(want, got, ("rowptr_t", "col_t", "perm_t")):
            assert torch.equal(w, g), (name, A.M, A.nnz)
        # and against the definition, on the host: the transposed pattern column by column, rows ascending
        rows = np.repeat(np.arange(A.M), np.diff(A.rowptr))
        order = np.lexsort((rows, A.col))
        assert np.array_equal(got[2].cpu().numpy()[:A.nnz], order.astype(np.int32))
        assert np.array_equal(got[1].cpu().numpy()[:A.nnz], rows[order].astype(np.int32))
        assert np.array_equal(got[0].cpu().numpy(), np.concatenate([[0], np.cumsum(np.bincount(A.col, minlength=A.Kc))]).astype(np.int32))


def test_static_transposition_limits_and_empty_matrix():
    A = wl.random_pattern(64, 64, 0.1, seed=3)
    rp, col = _dev(A.rowptr), _dev(A.col)
    rpt, ct, pt = _outputs(A)
    with pytest.raises(lb.LibraError) as e:        # more nonzeros than the fixed array serves: refused before anything is launched
        lb.libra_csr_transpose_device_static(A.M, A.Kc, lb.TRANSPOSE_STATIC_MAX_NNZ + 1, rp.data_ptr(), col.data_ptr(), rpt.data_ptr(),
                                             ct.data_ptr(), pt.data_ptr(), 0)
    assert e.value.code == lb.ERR["TOO_LARGE"]
    with pytest.raises(lb.LibraError) as e:
        lb.libra_csr_transpose_device_static(A.M, A.Kc, A.nnz, 0, col.data_ptr(), rpt.data_ptr(), ct.data_ptr(), pt.data_ptr(), 0)
    assert e.value.code == lb.ERR["NULL"]
    z = torch.zeros(9, dtype=torch.int32, device="cuda")
    out = torch.full((6,), -7, dtype=torch.int32, device="cuda")
    lb.libra_csr_transpose_device_static(8, 5, 0, z.data_ptr(), 0, out.data_ptr(), 0, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert not out.any()
