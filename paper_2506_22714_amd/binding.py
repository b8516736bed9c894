"""ctypes binding of the C ABI in ``include/libra.h``.

Argument marshalling only: every step of the SpMM / SDDMM path runs inside
``liblibra.so``.  The module-level functions carry the same names as the C
entry points; :class:`Plan` bundles a plan handle with the device buffer that
backs it.  There is no fallback: if the shared library is missing, loading
raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LIBRA_LIBRARY selects another build of the same library (e.g. an experimental one); default: the in-tree build
LIB_PATH = os.environ.get("LIBRA_LIBRARY") or os.path.join(_HERE, "liblibra.so")

F16, BF16, F32 = 0, 1, 2
MODE_HYBRID, MODE_DENSE_ONLY, MODE_SCALAR_ONLY = 0, 1, 2
FLAG_NO_FILL_PADDING, FLAG_NO_SPMM, FLAG_NO_SDDMM, FLAG_NATURAL_ORDER, FLAG_XCD_ORDER, FLAG_NO_XCD_ORDER = 1, 2, 4, 8, 16, 32
FLAG_SEGMENTS_BY_COLUMN, FLAG_TWO_KERNELS, FLAG_SEGMENTS_BY_COST = 64, 128, 256
TASK_WINDOW, TASK_CHUNK = 0, 1
OP_SPMM, OP_SDDMM = 1, 2
OK = 0
ERR = dict(NULL=-1, SHAPE=-2, ROWPTR=-3, COLUMN=-4, UNSORTED=-5, TOO_LARGE=-6, DTYPE=-7, OPTION=-8,
           UNSUPPORTED=-9, NOT_UPLOADED=-10, BUFFER=-11, NOT_BUILT=-12, HIP=-13, NOMEM=-14)


class LibraError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


class PlanOpts(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("mode", C.c_int32), ("window_rows", C.c_int32),
                ("block_cols", C.c_int32), ("spmm_min_vec_nnz", C.c_int32), ("sddmm_min_blk_nnz", C.c_int32),
                ("ts", C.c_int32), ("cs", C.c_int32), ("short_len", C.c_int32), ("sddmm_cs", C.c_int32),
                ("flags", C.c_uint32), ("threads", C.c_int32), ("sddmm_ts", C.c_int32), ("sddmm_min_dense_pct", C.c_int32)]

    def __init__(self, **kw):
        super().__init__(**kw)
        self.struct_size = C.sizeof(PlanOpts)


class Task(C.Structure):
    _fields_ = [("kind", C.c_int32), ("id", C.c_int32), ("blk_begin", C.c_int32), ("blk_end", C.c_int32),
                ("res_begin", C.c_int32), ("res_end", C.c_int32),
                ("scalar_mask", C.c_uint32), ("atomic_mask", C.c_uint32), ("store_mask", C.c_uint32),
                ("cost", C.c_uint32)]


TASK_DTYPE = np.dtype([("kind", "<i4"), ("id", "<i4"), ("blk_begin", "<i4"), ("blk_end", "<i4"),
                       ("res_begin", "<i4"), ("res_end", "<i4"),
                       ("scalar_mask", "<u4"), ("atomic_mask", "<u4"), ("store_mask", "<u4"), ("cost", "<u4")])


class SubplanView(C.Structure):
    _fields_ = [("n_windows", C.c_int64), ("n_blocks", C.c_int64), ("n_dense_nnz", C.c_int64),
                ("n_res_nnz", C.c_int64), ("n_tasks", C.c_int64), ("n_zero_rows", C.c_int64),
                ("window_rows", C.c_int32), ("block_cols", C.c_int32), ("words_per_block", C.c_int32),
                ("value_dtype", C.c_int32),
                ("win_blkptr", C.c_void_p), ("blk_cols", C.c_void_p), ("blk_bitmap", C.c_void_p),
                ("blk_valptr", C.c_void_p), ("dense_val", C.c_void_p), ("dense_perm", C.c_void_p),
                ("win_resptr", C.c_void_p), ("res_row", C.c_void_p), ("res_col", C.c_void_p),
                ("res_val", C.c_void_p), ("res_perm", C.c_void_p), ("tasks", C.c_void_p),
                ("zero_rows", C.c_void_p)]


_STATS_I64 = ["M", "Kc", "nnz", "n_windows", "n_vectors", "n_vectors_nnz1",
              "spmm_dense_vectors", "spmm_blocks", "spmm_pad_slots", "spmm_dense_nnz", "spmm_res_nnz",
              "spmm_tasks", "spmm_chunk_tasks", "spmm_zero_rows",
              "spmm_short_rows", "spmm_long_rows", "spmm_split_rows", "spmm_gather_rows",
              "sddmm_dense_vectors", "sddmm_blocks", "sddmm_pad_slots", "sddmm_dense_nnz", "sddmm_res_nnz",
              "sddmm_tasks", "sddmm_gather_rows"]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in _STATS_I64] + [("plan_seconds", C.c_double), ("neighbour_share", C.c_double),
                                                               ("xcd_order", C.c_int64), ("device_seconds", C.c_double)]


_lib = None


def lib() -> C.CDLL:
    """Load liblibra.so (built by ``paper_2506_22714_amd.build``).  Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2506_22714_amd.build` "
                               "(or __graft_entry__.build()) first")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        L.libra_plan.argtypes = [i64, i64, vp, vp, vp, C.c_int, C.POINTER(PlanOpts), C.POINTER(vp)]
        L.libra_plan_device_workspace.argtypes = [i64, i64, C.POINTER(PlanOpts), C.POINTER(sz)]
        L.libra_plan_device_buffer_bound.argtypes = [i64, i64, C.c_int, C.POINTER(PlanOpts), C.POINTER(sz)]
        L.libra_plan_device.argtypes = [i64, i64, i64, vp, vp, vp, C.c_int, C.POINTER(PlanOpts), vp, sz, vp, sz, C.c_int,
                                        vp, C.POINTER(vp)]
        L.libra_plan_device_bytes.argtypes = [vp, C.POINTER(sz)]
        L.libra_plan_upload.argtypes = [vp, vp, sz, vp]
        L.libra_spmm.argtypes = [vp, vp, i32, i64, vp, i64, vp]
        L.libra_sddmm.argtypes = [vp, vp, vp, i32, vp, vp]
        L.libra_sddmm_pattern.argtypes = [vp, vp, vp, i32, vp, vp]
        L.libra_edge_softmax.argtypes = [vp, vp, C.c_float, vp, C.c_int, vp]
        L.libra_edge_softmax_backward.argtypes = [vp, vp, C.c_int, vp, C.c_float, vp, vp]
        L.libra_probe_coissue.argtypes = [C.c_int, vp, C.POINTER(C.c_float * 3), vp]
        L.libra_probe_gather.argtypes = [vp, i64, i32, vp, i64, vp, vp]
        L.libra_probe_gather_hub.argtypes = [vp, i64, i32, vp, i64, vp, i32, vp, vp]
        L.libra_csr_transpose_workspace.argtypes = [i64, C.POINTER(sz)]
        L.libra_csr_transpose_device.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, vp, sz, vp]
        L.libra_csr_transpose_device_static.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, vp]
        L.libra_plan_set_values.argtypes = [vp, vp, C.c_int, vp]
        L.libra_plan_set_values_for.argtypes = [vp, vp, C.c_int, C.c_int, vp]
        L.libra_plan_export.argtypes = [vp, C.c_int, C.POINTER(SubplanView)]
        L.libra_plan_stats.argtypes = [vp, C.POINTER(Stats)]
        L.libra_plan_destroy.argtypes = [vp]
        L.libra_plan_destroy.restype = None
        L.libra_strerror.argtypes = [C.c_int]
        L.libra_strerror.restype = C.c_char_p
        L.libra_version.restype = C.c_int
        for n in ("libra_plan", "libra_plan_device_bytes", "libra_plan_upload", "libra_spmm", "libra_sddmm",
                  "libra_edge_softmax", "libra_plan_set_values", "libra_plan_export", "libra_plan_stats"):
            getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().libra_strerror(code).decode()


def libra_version() -> int:
    return int(lib().libra_version())


def _np_ptr(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _np_dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float16:
        return F16
    if a.dtype == np.float32:
        return F32
    raise TypeError(f"unsupported value dtype {a.dtype}")


def _check(rc: int, what: str):
    if rc != OK:
        raise LibraError(rc, what)


# ---- entry points, same names as the C ABI (raw pointers / numpy host arrays in, codes checked) ----
def libra_plan(M: int, Kc: int, rowptr: np.ndarray, col: np.ndarray, val: np.ndarray, opts: PlanOpts | None = None,
               val_dtype: int | None = None) -> C.c_void_p:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val)
    handle = C.c_void_p()
    rc = lib().libra_plan(M, Kc, _np_ptr(rowptr), _np_ptr(col), _np_ptr(val),
                          _np_dtype_code(val) if val_dtype is None else val_dtype,
                          C.byref(opts) if opts is not None else None, C.byref(handle))
    _check(rc, "libra_plan")
    return handle


def libra_plan_device_workspace(M: int, nnz: int, opts: PlanOpts | None = None) -> int:
    n = C.c_size_t()
    _check(lib().libra_plan_device_workspace(M, nnz, C.byref(opts) if opts is not None else None, C.byref(n)),
           "libra_plan_device_workspace")
    return int(n.value)


def libra_plan_device_buffer_bound(M: int, nnz: int, val_dtype: int, opts: PlanOpts | None = None) -> int:
    n = C.c_size_t()
    _check(lib().libra_plan_device_buffer_bound(M, nnz, val_dtype, C.byref(opts) if opts is not None else None, C.byref(n)),
           "libra_plan_device_buffer_bound")
    return int(n.value)


def libra_plan_device(M: int, Kc: int, nnz: int, rowptr_ptr: int, col_ptr: int, val_ptr: int, val_dtype: int,
                      opts: PlanOpts | None, ws_ptr: int, ws_bytes: int, plan_ptr: int = 0, plan_bytes: int = 0,
                      keep_host_copy: bool = True, stream: int = 0) -> C.c_void_p:
    handle = C.c_void_p()
    rc = lib().libra_plan_device(M, Kc, nnz, C.c_void_p(rowptr_ptr), C.c_void_p(col_ptr), C.c_void_p(val_ptr), val_dtype,
                                 C.byref(opts) if opts is not None else None, C.c_void_p(ws_ptr), ws_bytes,
                                 C.c_void_p(plan_ptr), plan_bytes, 1 if keep_host_copy else 0,
                                 C.c_void_p(stream), C.byref(handle))
    _check(rc, "libra_plan_device")
    return handle


def libra_plan_device_bytes(plan) -> int:
    n = C.c_size_t()
    _check(lib().libra_plan_device_bytes(plan, C.byref(n)), "libra_plan_device_bytes")
    return int(n.value)


def libra_plan_upload(plan, dev_ptr: int, nbytes: int, stream: int = 0):
    _check(lib().libra_plan_upload(plan, C.c_void_p(dev_ptr), nbytes, C.c_void_p(stream)), "libra_plan_upload")


def libra_spmm(plan, B_ptr: int, N: int, ldb: int, C_ptr: int, ldc: int, stream: int = 0):
    _check(lib().libra_spmm(plan, C.c_void_p(B_ptr), N, ldb, C.c_void_p(C_ptr), ldc, C.c_void_p(stream)), "libra_spmm")


def libra_sddmm(plan, X_ptr: int, Y_ptr: int, K: int, out_ptr: int, stream: int = 0):
    _check(lib().libra_sddmm(plan, C.c_void_p(X_ptr), C.c_void_p(Y_ptr), K, C.c_void_p(out_ptr), C.c_void_p(stream)),
           "libra_sddmm")


def libra_sddmm_pattern(plan, X_ptr: int, Y_ptr: int, K: int, out_ptr: int, stream: int = 0):
    _check(lib().libra_sddmm_pattern(plan, C.c_void_p(X_ptr), C.c_void_p(Y_ptr), K, C.c_void_p(out_ptr), C.c_void_p(stream)),
           "libra_sddmm_pattern")


def libra_edge_softmax_backward(plan, alpha_ptr: int, alpha_dtype: int, dalpha_ptr: int, scale: float, dscores_ptr: int,
                                stream: int = 0):
    _check(lib().libra_edge_softmax_backward(plan, C.c_void_p(alpha_ptr), alpha_dtype, C.c_void_p(dalpha_ptr), C.c_float(scale),
                                             C.c_void_p(dscores_ptr), C.c_void_p(stream)), "libra_edge_softmax_backward")


def libra_probe_coissue(iters: int, sink_ptr: int, stream: int = 0):
    """(MFMA only, FMA only, both) in microseconds."""
    t = (C.c_float * 3)()
    _check(lib().libra_probe_coissue(iters, C.c_void_p(sink_ptr), C.byref(t), C.c_void_p(stream)), "libra_probe_coissue")
    return tuple(float(x) for x in t)


def libra_probe_gather(table_ptr: int, table_rows: int, row_bytes: int, idx_ptr: int, n: int, sink_ptr: int, stream: int = 0):
    _check(lib().libra_probe_gather(C.c_void_p(table_ptr), table_rows, row_bytes, C.c_void_p(idx_ptr), n, C.c_void_p(sink_ptr),
                                    C.c_void_p(stream)), "libra_probe_gather")


def libra_probe_gather_hub(table_ptr: int, table_rows: int, row_bytes: int, idx_ptr: int, n: int, hub_rows_ptr: int, n_hub: int,
                           sink_ptr: int, stream: int = 0):
    _check(lib().libra_probe_gather_hub(C.c_void_p(table_ptr), table_rows, row_bytes, C.c_void_p(idx_ptr), n,
                                        C.c_void_p(hub_rows_ptr), n_hub, C.c_void_p(sink_ptr), C.c_void_p(stream)), "libra_probe_gather_hub")


def libra_csr_transpose_workspace(nnz: int) -> int:
    n = C.c_size_t()
    _check(lib().libra_csr_transpose_workspace(nnz, C.byref(n)), "libra_csr_transpose_workspace")
    return int(n.value)


def libra_csr_transpose_device(M: int, Kc: int, nnz: int, rowptr_ptr: int, col_ptr: int, rowptr_t_ptr: int, col_t_ptr: int,
                               perm_t_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0):
    _check(lib().libra_csr_transpose_device(M, Kc, nnz, C.c_void_p(rowptr_ptr), C.c_void_p(col_ptr), C.c_void_p(rowptr_t_ptr),
                                            C.c_void_p(col_t_ptr), C.c_void_p(perm_t_ptr), C.c_void_p(ws_ptr), ws_bytes,
                                            C.c_void_p(stream)), "libra_csr_transpose_device")


TRANSPOSE_STATIC_MAX_NNZ = 1 << 20


def libra_csr_transpose_device_static(M: int, Kc: int, nnz: int, rowptr_ptr: int, col_ptr: int, rowptr_t_ptr: int, col_t_ptr: int,
                                      perm_t_ptr: int, stream: int = 0):
    _check(lib().libra_csr_transpose_device_static(M, Kc, nnz, C.c_void_p(rowptr_ptr), C.c_void_p(col_ptr), C.c_void_p(rowptr_t_ptr),
                                                   C.c_void_p(col_t_ptr), C.c_void_p(perm_t_ptr), C.c_void_p(stream)),
           "libra_csr_transpose_device_static")


def _csr_operands(M: int, rowptr, col) -> int:
    """Checks the device CSR arrays a planner or the transposition reads (sizes, types, layout, device); returns nnz."""
    import torch
    for name, t in (("rowptr", rowptr), ("col", col)):
        if not isinstance(t, torch.Tensor) or t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError(f"{name}: expected a contiguous int32 torch tensor")
    if rowptr.numel() != M + 1:
        raise ValueError(f"rowptr: {rowptr.numel()} elements, expected M + 1 = {M + 1}")
    if not rowptr.is_cuda or not col.is_cuda or col.device != rowptr.device:
        raise ValueError("rowptr and col must be on one GPU")
    return int(col.numel())


def transpose_csr(M: int, Kc: int, rowptr, col):
    """(rowptr_t, col_t, perm_t) of the transposed pattern, torch int32 tensors on the device of the inputs."""
    import torch
    nnz = int(col.numel())
    _csr_operands(M, rowptr, col)
    rowptr_t = torch.empty(Kc + 1, dtype=torch.int32, device=rowptr.device)
    col_t = torch.empty(nnz, dtype=torch.int32, device=rowptr.device)
    perm_t = torch.empty(nnz, dtype=torch.int32, device=rowptr.device)
    nb = libra_csr_transpose_workspace(nnz)
    ws = torch.empty(nb, dtype=torch.uint8, device=rowptr.device)
    libra_csr_transpose_device(M, Kc, nnz, rowptr.data_ptr(), col.data_ptr() if nnz else 0, rowptr_t.data_ptr(),
                               col_t.data_ptr() if nnz else 0, perm_t.data_ptr() if nnz else 0, ws.data_ptr(), nb,
                               torch.cuda.current_stream().cuda_stream)
    return rowptr_t, col_t, perm_t


def libra_edge_softmax(plan, scores_ptr: int, scale: float, out_ptr: int, out_dtype: int, stream: int = 0):
    _check(lib().libra_edge_softmax(plan, C.c_void_p(scores_ptr), C.c_float(scale), C.c_void_p(out_ptr), out_dtype,
                                    C.c_void_p(stream)), "libra_edge_softmax")


def libra_plan_set_values(plan, vals_ptr: int, dtype: int, stream: int = 0):
    _check(lib().libra_plan_set_values(plan, C.c_void_p(vals_ptr), dtype, C.c_void_p(stream)), "libra_plan_set_values")


def libra_plan_set_values_for(plan, vals_ptr: int, dtype: int, ops: int, stream: int = 0):
    _check(lib().libra_plan_set_values_for(plan, C.c_void_p(vals_ptr), dtype, ops, C.c_void_p(stream)),
           "libra_plan_set_values_for")


def libra_plan_destroy(plan):
    lib().libra_plan_destroy(plan)


def _arr(ptr, n, dtype):
    if not ptr or n == 0:
        return np.zeros(0, dtype=dtype)
    buf = (C.c_char * (n * np.dtype(dtype).itemsize)).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype).copy()


def libra_plan_export(plan, which: int) -> dict:
    """Copies of one sub-plan's host arrays as numpy arrays (0 = SpMM, 1 = SDDMM)."""
    v = SubplanView()
    _check(lib().libra_plan_export(plan, which, C.byref(v)), "libra_plan_export")
    vt = {F16: np.float16, BF16: np.uint16, F32: np.float32}[v.value_dtype]      # bfloat16 comes back as bit patterns
    nb, KB, wpb = v.n_blocks, v.block_cols, v.words_per_block
    out = dict(n_windows=v.n_windows, n_blocks=nb, n_dense_nnz=v.n_dense_nnz, n_res_nnz=v.n_res_nnz,
               n_tasks=v.n_tasks, window_rows=v.window_rows, block_cols=KB, words_per_block=wpb,
               win_blkptr=_arr(v.win_blkptr, v.n_windows + 1, np.int32),
               blk_cols=_arr(v.blk_cols, nb * KB, np.int32).reshape(nb, KB),
               blk_bitmap=_arr(v.blk_bitmap, nb * wpb, np.uint64).reshape(nb, wpb),
               blk_valptr=_arr(v.blk_valptr, nb + 1, np.int32),
               dense_val=_arr(v.dense_val, v.n_dense_nnz, vt),
               dense_perm=_arr(v.dense_perm, v.n_dense_nnz, np.int32),
               res_row=_arr(v.res_row, v.n_res_nnz, np.int32),
               res_col=_arr(v.res_col, v.n_res_nnz, np.int32),
               res_val=_arr(v.res_val, v.n_res_nnz, vt),
               res_perm=_arr(v.res_perm, v.n_res_nnz, np.int32),
               tasks=_arr(v.tasks, v.n_tasks, TASK_DTYPE),
               zero_rows=_arr(v.zero_rows, v.n_zero_rows, np.int32))
    if which == 0:
        out["win_resptr"] = _arr(v.win_resptr, v.n_windows + 1, np.int32)
    return out


def libra_plan_stats(plan) -> dict:
    s = Stats()
    _check(lib().libra_plan_stats(plan, C.byref(s)), "libra_plan_stats")
    return {n: getattr(s, n) for n, _t in Stats._fields_}


def _with_tuned(opts: dict, tuned, val_dtype: int, N, K) -> dict:
    """Plan options with the entries of a tuner table filled in (argument marshalling: the table is data, the choice was
    made by the tuner); options given explicitly (non-zero) are kept."""
    if tuned is None:
        return opts
    from .tune import tuned_options
    t = tuned_options(tuned, {F16: "f16", BF16: "bf16", F32: "f32"}[val_dtype], N=N, K=K)
    return {**t, **{k: v for k, v in opts.items() if v or k not in t}}


# ---- convenience wrapper: a plan handle plus the torch buffer that backs its device copy ----
class Plan:
    def __init__(self, M, Kc, rowptr, col, val, val_dtype: int | None = None, tuned=None, N: int | None = None,
                 K: int | None = None, **opts):
        """`val_dtype=BF16` with `val` as uint16 bit patterns builds a bfloat16 plan (numpy has no such type).
        `tuned`: a table written by `python -m paper_2506_22714_amd.tune --emit` (path or dict); the options of the
        classes of the feature widths `N` (SpMM) and `K` (SDDMM) are taken from it, explicit options win."""
        self.M, self.Kc = int(M), int(Kc)
        self.val_dtype = _np_dtype_code(np.asarray(val)) if val_dtype is None else int(val_dtype)
        opts = _with_tuned(opts, tuned, self.val_dtype, N, K)
        self.handle = libra_plan(self.M, self.Kc, rowptr, col, val, PlanOpts(**opts) if opts else None,
                                 val_dtype=self.val_dtype)
        self.nnz = libra_plan_stats(self.handle)["nnz"]
        self._buf = None

    @classmethod
    def from_device_csr(cls, M, Kc, rowptr, col, val, resident: bool = False, keep_host_copy: bool = True, tuned=None,
                        N: int | None = None, K: int | None = None, **opts):
        """Plan built on the GPU from torch tensors (int32 rowptr/col, float16 / bfloat16 / float32 values).
        ``resident``: the device copy is written during planning into a buffer of the bound size (no upload).
        ``tuned``, ``N``, ``K``: as in the constructor."""
        import torch
        nnz = _csr_operands(M, rowptr, col)
        if val.dtype not in (torch.float16, torch.bfloat16, torch.float32):
            raise ValueError(f"val: dtype {val.dtype} is not float16, bfloat16 or float32")
        if val.numel() != nnz or not val.is_contiguous():
            raise ValueError(f"val: {val.numel()} elements (contiguous: {val.is_contiguous()}), expected {nnz} contiguous")
        if not val.is_cuda or val.device != rowptr.device:
            raise ValueError("val: must be on the same GPU as rowptr")
        self = cls.__new__(cls)
        self.M, self.Kc = int(M), int(Kc)
        self.val_dtype = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}[val.dtype]
        opts = _with_tuned(opts, tuned, self.val_dtype, N, K)
        o = PlanOpts(**opts) if opts else None
        ws_bytes = libra_plan_device_workspace(self.M, nnz, o)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=rowptr.device)
        self.handle = None
        self._buf = None
        if resident:
            nb = libra_plan_device_buffer_bound(self.M, nnz, self.val_dtype, o)
            self._buf = torch.empty(nb, dtype=torch.uint8, device=rowptr.device)
        self.handle = libra_plan_device(self.M, self.Kc, nnz, rowptr.data_ptr(), col.data_ptr() if nnz else 0,
                                        val.data_ptr() if nnz else 0, self.val_dtype, o, ws.data_ptr(), ws_bytes,
                                        self._buf.data_ptr() if resident else 0, self._buf.numel() if resident else 0,
                                        keep_host_copy or not resident, torch.cuda.current_stream().cuda_stream)
        del ws
        self.nnz = libra_plan_stats(self.handle)["nnz"]
        return self

    @classmethod
    def from_csr(cls, csr, val=None, val_dtype: int | None = None, tuned=None, N: int | None = None, K: int | None = None, **opts):
        return cls(csr.M, csr.Kc, csr.rowptr, csr.col, csr.val if val is None else val, val_dtype=val_dtype, tuned=tuned, N=N, K=K, **opts)

    def close(self):
        if self.handle is not None:
            libra_plan_destroy(self.handle)
            self.handle = None
            self._buf = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def stats(self) -> dict:
        return libra_plan_stats(self.handle)

    def export(self, which: int) -> dict:
        return libra_plan_export(self.handle, which)

    def upload(self, device="cuda"):
        import torch
        n = libra_plan_device_bytes(self.handle)
        self._buf = torch.empty(n, dtype=torch.uint8, device=device)
        libra_plan_upload(self.handle, self._buf.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
        return self

    def _torch_dtype(self):
        import torch
        return {F16: torch.float16, BF16: torch.bfloat16, F32: torch.float32}[self.val_dtype]

    # The C ABI sees pointers only: the sizes behind them are checked here, before any launch, and a mismatch raises
    # (an undersized operand would make a kernel read or write past its end).  Shape, type and layout first, the device last.
    @staticmethod
    def _operand(t, name, dtype, shape=None, numel=None, rows_contiguous=False):
        import torch
        if not isinstance(t, torch.Tensor):
            raise ValueError(f"{name}: expected a torch tensor, got {type(t).__name__}")
        if dtype is not None and t.dtype != dtype:
            raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
        if shape is not None:
            if t.dim() != len(shape) or any(want is not None and int(have) != int(want) for have, want in zip(t.shape, shape)):
                raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple('*' if w is None else w for w in shape)}")
        if numel is not None and t.numel() != numel:
            raise ValueError(f"{name}: {t.numel()} elements, expected {numel}")
        if rows_contiguous:
            if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or (t.shape[0] > 1 and t.stride(0) < t.shape[1]):
                raise ValueError(f"{name}: rows must be contiguous (strides {tuple(t.stride())})")
        elif not t.is_contiguous():
            raise ValueError(f"{name}: must be contiguous")
        if not t.is_cuda:
            raise ValueError(f"{name}: must be a GPU tensor")

    def _value_code(self, t, name):
        import torch
        code = {torch.float16: F16, torch.bfloat16: BF16, torch.float32: F32}.get(t.dtype)
        if code is None:
            raise ValueError(f"{name}: dtype {t.dtype} is not float16, bfloat16 or float32")
        return code

    def spmm(self, B, out=None):
        import torch
        self._operand(B, "B", self._torch_dtype(), shape=(self.Kc, None), rows_contiguous=True)
        N = int(B.shape[1])
        if out is None:
            out = torch.empty((self.M, N), dtype=torch.float32, device=B.device)
        self._operand(out, "out", torch.float32, shape=(self.M, N), rows_contiguous=True)
        if out.device != B.device:
            raise ValueError("out: on another device than B")
        libra_spmm(self.handle, B.data_ptr(), N, B.stride(0), out.data_ptr(), out.stride(0),
                   torch.cuda.current_stream().cuda_stream)
        return out

    def sddmm(self, X, Y, out=None, pattern_only: bool = False):
        import torch
        self._operand(X, "X", self._torch_dtype(), shape=(self.M, None))
        self._operand(Y, "Y", self._torch_dtype(), shape=(self.Kc, int(X.shape[1])))
        if out is None:
            out = torch.empty(self.nnz, dtype=torch.float32, device=X.device)
        self._operand(out, "out", torch.float32, numel=self.nnz)
        if Y.device != X.device or out.device != X.device:
            raise ValueError("X, Y and out must be on one device")
        (libra_sddmm_pattern if pattern_only else libra_sddmm)(self.handle, X.data_ptr(), Y.data_ptr(), X.shape[1], out.data_ptr(),
                                                               torch.cuda.current_stream().cuda_stream)
        return out

    def edge_softmax(self, scores, scale: float, out=None):
        import torch
        self._operand(scores, "scores", torch.float32, numel=self.nnz)
        if out is None:
            out = torch.empty(self.nnz, dtype=self._torch_dtype(), device=scores.device)
        code = self._value_code(out, "out")
        self._operand(out, "out", None, numel=self.nnz)
        if out.device != scores.device:
            raise ValueError("out: on another device than scores")
        libra_edge_softmax(self.handle, scores.data_ptr(), scale, out.data_ptr(), code,
                           torch.cuda.current_stream().cuda_stream)
        return out

    def edge_softmax_backward(self, alpha, dalpha, scale: float, out=None):
        import torch
        code = self._value_code(alpha, "alpha")
        self._operand(alpha, "alpha", None, numel=self.nnz)
        self._operand(dalpha, "dalpha", torch.float32, numel=self.nnz)
        if out is None:
            out = torch.empty(self.nnz, dtype=torch.float32, device=alpha.device)
        self._operand(out, "out", torch.float32, numel=self.nnz)
        if dalpha.device != alpha.device or out.device != alpha.device:
            raise ValueError("alpha, dalpha and out must be on one device")
        libra_edge_softmax_backward(self.handle, alpha.data_ptr(), code, dalpha.data_ptr(), scale, out.data_ptr(),
                                    torch.cuda.current_stream().cuda_stream)
        return out

    def set_values(self, vals, ops: int = OP_SPMM | OP_SDDMM, one_call: bool = False):
        """New values of A in CSR order.  ``one_call``: through libra_plan_set_values (both operators) instead of
        libra_plan_set_values_for."""
        import torch
        self._operand(vals, "vals", self._torch_dtype(), numel=self.nnz)
        if one_call:
            if ops != OP_SPMM | OP_SDDMM:
                raise ValueError("one_call refreshes both operators")
            libra_plan_set_values(self.handle, vals.data_ptr(), self.val_dtype, torch.cuda.current_stream().cuda_stream)
        else:
            libra_plan_set_values_for(self.handle, vals.data_ptr(), self.val_dtype, ops, torch.cuda.current_stream().cuda_stream)
