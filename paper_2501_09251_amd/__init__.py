"""Python binding of libaccspmm.so (see include/acc_spmm.h for the contract of each call).

Argument marshalling only: every step of the SpMM path runs in the library's HIP
kernels and host code.  The functions keep the C names.  Device buffers are passed either
as torch tensors (their data pointers are taken) or as integer device addresses; torch is
used by callers for device memory and streams, never for arithmetic.

There is no fallback: if the shared library is missing, ``load()`` raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaccspmm.so")
_lib = None

ACC_SPMM_OFF, ACC_SPMM_ON, ACC_SPMM_AUTO = 0, 1, 2
ACC_SPMM_FP16, ACC_SPMM_BF16 = 0, 1

(ACC_SPMM_ARR_PERM, ACC_SPMM_ARR_IPERM, ACC_SPMM_ARR_ROW_WINDOW_OFFSET, ACC_SPMM_ARR_TC_OFFSET,
 ACC_SPMM_ARR_SPARSE_A_TO_B, ACC_SPMM_ARR_TC_LOCAL_BIT, ACC_SPMM_ARR_VALUES, ACC_SPMM_ARR_WORK_ITEMS,
 ACC_SPMM_ARR_DENDROGRAM_PARENT, ACC_SPMM_ARR_COL_ORDER, ACC_SPMM_ARR_COL_RANK) = range(11)

_ARRAY_DTYPES = {
    ACC_SPMM_ARR_PERM: np.int32, ACC_SPMM_ARR_IPERM: np.int32, ACC_SPMM_ARR_ROW_WINDOW_OFFSET: np.int32,
    ACC_SPMM_ARR_TC_OFFSET: np.int32, ACC_SPMM_ARR_SPARSE_A_TO_B: np.int32, ACC_SPMM_ARR_TC_LOCAL_BIT: np.uint64,
    ACC_SPMM_ARR_VALUES: np.uint16, ACC_SPMM_ARR_WORK_ITEMS: np.int32, ACC_SPMM_ARR_DENDROGRAM_PARENT: np.int32,
    ACC_SPMM_ARR_COL_ORDER: np.int32, ACC_SPMM_ARR_COL_RANK: np.int32,
}

EXPORTED_SYMBOLS = [
    "acc_spmm_plan", "acc_spmm_plan_ex", "acc_spmm_plan_device", "acc_spmm_execute", "acc_spmm_execute_c16", "acc_spmm_execute_static", "acc_spmm_execute_timed", "acc_spmm_execute_csr_naive", "acc_spmm_destroy",
    "acc_spmm_last_error", "acc_spmm_plan_stats", "acc_spmm_plan_traffic", "acc_spmm_plan_export",
    "acc_spmm_dendrogram_host", "acc_spmm_schedule_host", "acc_spmm_calibration_copy", "acc_spmm_calibration_gather", "acc_spmm_permute_rows", "acc_spmm_sddmm", "acc_spmm_update_values", "acc_spmm_plan_save", "acc_spmm_plan_load",
    "acc_spmm_mtx_open", "acc_spmm_mtx_shape", "acc_spmm_mtx_csr", "acc_spmm_mtx_close",
]


class acc_spmm_options(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_int32), ("reorder", ctypes.c_int32), ("load_balance", ctypes.c_int32),
        ("max_tiles_per_item", ctypes.c_int32), ("window_height", ctypes.c_int32), ("tile_width", ctypes.c_int32),
        ("segment_length", ctypes.c_int32), ("ibd_threshold", ctypes.c_float), ("keep_csr", ctypes.c_int32),
        ("no_prefetch", ctypes.c_int32), ("streaming_stores", ctypes.c_int32), ("pipeline_depth", ctypes.c_int32),
        ("value_fetch", ctypes.c_int32),
        ("value_type", ctypes.c_int32),
        ("column_order", ctypes.c_int32),
        ("operand_order", ctypes.c_int32),
        ("keep_entry_map", ctypes.c_int32),
        ("dendrogram_on_host", ctypes.c_int32),
        ("lds_staging", ctypes.c_int32),
        ("slabs_per_wave", ctypes.c_int32),
    ]


class acc_spmm_stats(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int64), ("K", ctypes.c_int64), ("nnz", ctypes.c_int64),
        ("window_height", ctypes.c_int32), ("tile_width", ctypes.c_int32),
        ("num_windows", ctypes.c_int64), ("num_tiles", ctypes.c_int64), ("sum_distinct_cols", ctypes.c_int64),
        ("num_tiles_identity", ctypes.c_int64), ("num_items", ctypes.c_int64),
        ("num_split_windows", ctypes.c_int64), ("num_partial_slots", ctypes.c_int64),
        ("max_tiles_per_item", ctypes.c_int32), ("reorder_applied", ctypes.c_int32),
        ("load_balance_applied", ctypes.c_int32),
        ("ibd", ctypes.c_double), ("mean_nnz_per_tile", ctypes.c_double),
        ("index_bytes", ctypes.c_int64), ("schedule_bytes", ctypes.c_int64),
        ("reorder_work_ratio", ctypes.c_double),
        ("t_validate_s", ctypes.c_double), ("t_reorder_s", ctypes.c_double), ("t_encode_s", ctypes.c_double),
        ("t_schedule_s", ctypes.c_double), ("t_total_s", ctypes.c_double),
        ("t_graph_s", ctypes.c_double), ("t_dendrogram_s", ctypes.c_double), ("t_ordering_s", ctypes.c_double),
        ("column_order_applied", ctypes.c_int32), ("num_hot_columns", ctypes.c_int32),
        ("hub_label_skew", ctypes.c_double), ("t_column_order_s", ctypes.c_double),
        ("dendrogram_on_device", ctypes.c_int32), ("pad_", ctypes.c_int32), ("dendrogram_rounds", ctypes.c_int64),
    ]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class AccSpmmError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"acc_spmm error {code}: {msg}")
        self.code = code


def load():
    """Load the shared library.  Raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2501_09251_amd.build` "
                          "(there is no CPU fallback)")
    # One HIP runtime per process: PyTorch ships its own libamdhip64 under the same soname as the system's.
    # Whichever is loaded first serves both; if this library pulled in the system copy before torch is
    # imported, torch would run its bundled HSA runtime under a foreign HIP and see no device.  So a
    # process that has torch gets torch's runtime first.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    L.acc_spmm_plan.restype = vp
    L.acc_spmm_plan.argtypes = [i64, i64, i64, vp, vp, vp]
    L.acc_spmm_plan_ex.restype = vp
    L.acc_spmm_plan_ex.argtypes = [i64, i64, i64, vp, vp, vp, ctypes.POINTER(acc_spmm_options)]
    L.acc_spmm_plan_device.restype = vp
    L.acc_spmm_plan_device.argtypes = [i64, i64, i64, vp, vp, vp, ctypes.POINTER(acc_spmm_options)]
    L.acc_spmm_execute.restype = ctypes.c_int
    L.acc_spmm_execute.argtypes = [vp, vp, i32, vp, vp]
    L.acc_spmm_execute_c16.restype = ctypes.c_int
    L.acc_spmm_execute_c16.argtypes = [vp, vp, i32, vp, vp]
    L.acc_spmm_execute_static.restype = ctypes.c_int
    L.acc_spmm_execute_static.argtypes = [vp, vp, i32, vp, vp]
    L.acc_spmm_execute_timed.restype = ctypes.c_int
    L.acc_spmm_execute_timed.argtypes = [vp, vp, i32, vp, vp] + [ctypes.POINTER(ctypes.c_float)] * 3
    L.acc_spmm_mtx_open.restype = vp
    L.acc_spmm_mtx_open.argtypes = [ctypes.c_char_p, i32]
    L.acc_spmm_mtx_shape.restype = ctypes.c_int
    L.acc_spmm_mtx_shape.argtypes = [vp] + [ctypes.POINTER(i64)] * 3
    L.acc_spmm_mtx_csr.restype = ctypes.c_int
    L.acc_spmm_mtx_csr.argtypes = [vp, vp, vp, vp]
    L.acc_spmm_mtx_close.restype = None
    L.acc_spmm_mtx_close.argtypes = [vp]
    L.acc_spmm_plan_save.restype = ctypes.c_int
    L.acc_spmm_plan_save.argtypes = [vp, ctypes.c_char_p]
    L.acc_spmm_plan_load.restype = vp
    L.acc_spmm_plan_load.argtypes = [ctypes.c_char_p]
    L.acc_spmm_update_values.restype = ctypes.c_int
    L.acc_spmm_update_values.argtypes = [vp, vp, vp]
    L.acc_spmm_sddmm.restype = ctypes.c_int
    L.acc_spmm_sddmm.argtypes = [vp, vp, vp, i32, vp, i32, vp]
    L.acc_spmm_permute_rows.restype = ctypes.c_int
    L.acc_spmm_permute_rows.argtypes = [vp, vp, vp, i64, i32, vp]
    L.acc_spmm_execute_csr_naive.restype = ctypes.c_int
    L.acc_spmm_execute_csr_naive.argtypes = [vp, vp, i32, vp, vp]
    L.acc_spmm_destroy.restype = None
    L.acc_spmm_destroy.argtypes = [vp]
    L.acc_spmm_last_error.restype = ctypes.c_int
    L.acc_spmm_last_error.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
    L.acc_spmm_plan_stats.restype = ctypes.c_int
    L.acc_spmm_plan_stats.argtypes = [vp, ctypes.POINTER(acc_spmm_stats)]
    L.acc_spmm_plan_traffic.restype = ctypes.c_int
    L.acc_spmm_plan_traffic.argtypes = [vp, i32] + [ctypes.POINTER(ctypes.c_int64)] * 4
    L.acc_spmm_plan_export.restype = ctypes.c_int
    L.acc_spmm_plan_export.argtypes = [vp, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_size_t)]
    L.acc_spmm_calibration_copy.restype = ctypes.c_int
    L.acc_spmm_calibration_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.acc_spmm_calibration_gather.restype = ctypes.c_int
    L.acc_spmm_calibration_gather.argtypes = [vp, i64, i64, vp, i64, vp, ctypes.c_size_t, vp, ctypes.c_size_t, i32, i32, vp]
    L.acc_spmm_dendrogram_host.restype = i64
    L.acc_spmm_dendrogram_host.argtypes = [i64, vp, vp, i32, vp, vp, vp, ctypes.POINTER(ctypes.c_double)]
    L.acc_spmm_schedule_host.restype = i64
    L.acc_spmm_schedule_host.argtypes = [i64, vp, i32, i32, ctypes.c_float, ctypes.POINTER(ctypes.c_double), vp, i64,
                                         ctypes.POINTER(ctypes.c_int64)]
    _lib = L
    return L


def acc_spmm_last_error():
    buf = ctypes.create_string_buffer(1024)
    code = load().acc_spmm_last_error(buf, len(buf))
    return code, buf.value.decode(errors="replace")


def _raise():
    raise AccSpmmError(*acc_spmm_last_error())


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data


def _dev_ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()  # torch tensor


def make_options(**kw) -> acc_spmm_options:
    o = acc_spmm_options()
    o.struct_size = ctypes.sizeof(acc_spmm_options)
    o.reorder = ACC_SPMM_AUTO
    o.load_balance = ACC_SPMM_AUTO
    o.column_order = ACC_SPMM_AUTO
    for k, v in kw.items():
        if not hasattr(o, k):
            raise TypeError(f"unknown option {k}")
        setattr(o, k, v)
    return o


def acc_spmm_plan_device(M, K, nnz, csr_rowptr, csr_colidx, csr_vals, options=None):
    """Plan from CSR arrays in device memory (torch tensors: int32, int32, int16/float16 bit patterns)."""
    h = load().acc_spmm_plan_device(M, K, nnz, _dev_ptr(csr_rowptr), _dev_ptr(csr_colidx), _dev_ptr(csr_vals),
                                    ctypes.byref(options) if options is not None else None)
    if not h:
        _raise()
    return h


def acc_spmm_plan(M, K, nnz, csr_rowptr, csr_colidx, csr_vals):
    """Build a plan with default options; returns the opaque handle (an int)."""
    return acc_spmm_plan_ex(M, K, nnz, csr_rowptr, csr_colidx, csr_vals, None)


def acc_spmm_plan_ex(M, K, nnz, csr_rowptr, csr_colidx, csr_vals, options):
    rp, rp_p = _host(csr_rowptr, np.int32)
    ci, ci_p = _host(csr_colidx, np.int32)
    va, va_p = _host(csr_vals, np.uint16)
    if len(rp) != M + 1 or len(ci) < nnz or len(va) < nnz:
        raise ValueError("CSR array lengths do not match M / nnz")
    h = load().acc_spmm_plan_ex(M, K, nnz, rp_p, ci_p, va_p, ctypes.byref(options) if options is not None else None)
    if not h:
        _raise()
    return h


_plan_shape = {}     # plan handle -> (M, K, nnz), for the size checks below
_last_checked = None


def _shape_of(plan):
    shape = _plan_shape.get(plan)
    if shape is None:
        st = acc_spmm_stats()
        if load().acc_spmm_plan_stats(plan, ctypes.byref(st)) != 0:
            return None
        shape = _plan_shape[plan] = (int(st.M), int(st.K), int(st.nnz))
    return shape


def _check_operands(plan, B, N, C, c_bytes_per_value):
    """The C ABI takes bare addresses and cannot know how large the caller's buffers are.  When they come as
    tensors the binding can: a B or C smaller than the call's N needs is refused here instead of being read or
    written past its end by the kernels."""
    global _last_checked
    key = (plan, id(B), id(C), N, c_bytes_per_value)
    if key == _last_checked:
        return                            # the same objects as in the last call (a timing loop): checked already
    if not (hasattr(B, "numel") or hasattr(C, "numel")) or not isinstance(N, int) or N <= 0 or N > 65536:
        return                            # widths out of range are the library's to refuse
    shape = _shape_of(plan)
    if shape is None:
        return                            # not a plan: the library reports it
    M, K, _ = shape
    if hasattr(B, "numel") and B.numel() * B.element_size() < K * N * 2:
        raise ValueError(f"B holds {B.numel() * B.element_size()} bytes, the call reads K x N x 2 = {K * N * 2}")
    if hasattr(C, "numel") and C.numel() * C.element_size() < M * N * c_bytes_per_value:
        raise ValueError(f"C holds {C.numel() * C.element_size()} bytes, the call writes M x N x {c_bytes_per_value} = "
                         f"{M * N * c_bytes_per_value}")
    _last_checked = key


def acc_spmm_execute(plan, B, N, C, stream=None):
    """Enqueue C = A.B.  B, C: torch CUDA tensors or device addresses; stream: hipStream_t as int."""
    _check_operands(plan, B, N, C, 4)
    if load().acc_spmm_execute(plan, _dev_ptr(B), N, _dev_ptr(C), stream) != 0:
        _raise()


def acc_spmm_execute_c16(plan, B, N, C, stream=None):
    """Enqueue C = A.B with C in the plan's 16-bit value type (fp32 accumulation, one rounding)."""
    _check_operands(plan, B, N, C, 2)
    if load().acc_spmm_execute_c16(plan, _dev_ptr(B), N, _dev_ptr(C), stream) != 0:
        _raise()


def acc_spmm_execute_static(plan, B, N, C, stream=None):
    """acc_spmm_execute that allocates nothing: its temporary buffers live in the library's static device array."""
    _check_operands(plan, B, N, C, 4)
    if load().acc_spmm_execute_static(plan, _dev_ptr(B), N, _dev_ptr(C), stream) != 0:
        _raise()


STATIC_SCRATCH_BYTES = 64 << 20


def acc_spmm_execute_timed(plan, B, N, C, stream=None):
    """Blocking execute; returns (tile kernel ms, combine kernel ms, B gather ms) from HIP events on `stream`."""
    _check_operands(plan, B, N, C, 4)
    t, c, g = ctypes.c_float(), ctypes.c_float(), ctypes.c_float()
    if load().acc_spmm_execute_timed(plan, _dev_ptr(B), N, _dev_ptr(C), stream, ctypes.byref(t), ctypes.byref(c),
                                     ctypes.byref(g)) != 0:
        _raise()
    return t.value, c.value, g.value


def read_matrix_market(path, value_type=ACC_SPMM_FP16):
    """acc_spmm_mtx_open / _shape / _csr / _close in one call: (M, K, rowptr, colidx, vals) as numpy arrays."""
    L = load()
    h = L.acc_spmm_mtx_open(os.fsencode(path), value_type)
    if not h:
        _raise()
    try:
        M, K, nnz = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        if L.acc_spmm_mtx_shape(h, ctypes.byref(M), ctypes.byref(K), ctypes.byref(nnz)) != 0:
            _raise()
        rowptr = np.zeros(M.value + 1, np.int32)
        colidx = np.zeros(nnz.value, np.int32)
        vals = np.zeros(nnz.value, np.uint16)
        if L.acc_spmm_mtx_csr(h, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data) != 0:
            _raise()
    finally:
        L.acc_spmm_mtx_close(h)
    return M.value, K.value, rowptr, colidx, vals


def acc_spmm_plan_save(plan, path):
    if load().acc_spmm_plan_save(plan, os.fsencode(path)) != 0:
        _raise()


def acc_spmm_plan_load(path):
    h = load().acc_spmm_plan_load(os.fsencode(path))
    if not h:
        _raise()
    return h


def acc_spmm_update_values(plan, csr_vals, stream=None):
    if load().acc_spmm_update_values(plan, _dev_ptr(csr_vals), stream) != 0:
        _raise()


def acc_spmm_sddmm(plan, X, Y, N, out, use_values=0, stream=None):
    shape = _shape_of(plan) if isinstance(N, int) and 0 < N <= 65536 else None
    if shape is not None:                 # tensors too small for the call are refused here (see _check_operands)
        for name, t, need in (("X", X, shape[0] * N * 2), ("Y", Y, shape[1] * N * 2), ("out", out, shape[2] * 4)):
            if hasattr(t, "numel") and t.numel() * t.element_size() < need:
                raise ValueError(f"{name} holds {t.numel() * t.element_size()} bytes, the call needs {need}")
    if load().acc_spmm_sddmm(plan, _dev_ptr(X), _dev_ptr(Y), N, _dev_ptr(out), use_values, stream) != 0:
        _raise()


def acc_spmm_permute_rows(plan, src, dst, row_bytes, to_caller=0, stream=None):
    if load().acc_spmm_permute_rows(plan, _dev_ptr(src), _dev_ptr(dst), row_bytes, to_caller, stream) != 0:
        _raise()


def acc_spmm_calibration_copy(dst, src, nbytes, stream=None):
    if load().acc_spmm_calibration_copy(_dev_ptr(dst), _dev_ptr(src), nbytes, stream) != 0:
        _raise()


def acc_spmm_calibration_gather(table, rows, row_bytes, index, n_index, sink, sink_bytes, out=None, out_bytes=0,
                                write_every=0, write_rows=0, stream=None):
    if load().acc_spmm_calibration_gather(_dev_ptr(table), rows, row_bytes, _dev_ptr(index), n_index, _dev_ptr(sink),
                                          sink_bytes, _dev_ptr(out), out_bytes, write_every, write_rows, stream) != 0:
        _raise()


def acc_spmm_execute_csr_naive(plan, B, N, C, stream=None):
    _check_operands(plan, B, N, C, 4)
    if load().acc_spmm_execute_csr_naive(plan, _dev_ptr(B), N, _dev_ptr(C), stream) != 0:
        _raise()


def acc_spmm_destroy(plan):
    if plan:
        global _last_checked
        _plan_shape.pop(plan, None)      # the address may be handed out again
        _last_checked = None
        load().acc_spmm_destroy(plan)


def acc_spmm_plan_stats(plan) -> dict:
    st = acc_spmm_stats()
    if load().acc_spmm_plan_stats(plan, ctypes.byref(st)) != 0:
        _raise()
    return st.as_dict()


def acc_spmm_plan_traffic(plan, N) -> dict:
    a, b, c, f = (ctypes.c_int64() for _ in range(4))
    if load().acc_spmm_plan_traffic(plan, N, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(f)) != 0:
        _raise()
    return dict(a_bytes=a.value, b_bytes=b.value, c_bytes=c.value, mfma_flops=f.value)


def acc_spmm_plan_export(plan, which) -> np.ndarray:
    n = ctypes.c_size_t(0)
    L = load()
    if L.acc_spmm_plan_export(plan, which, None, ctypes.byref(n)) != 0:
        _raise()
    dt = np.dtype(_ARRAY_DTYPES[which])
    out = np.empty(n.value // dt.itemsize, dt)
    if n.value and L.acc_spmm_plan_export(plan, which, out.ctypes.data, ctypes.byref(n)) != 0:
        _raise()
    return out


def acc_spmm_dendrogram_host(M, graph_rowptr, graph_adj, segment_length=0):
    """Host stage of the plan (Step I) on a symmetric adjacency: returns (parent, leaf_sequence,
    segment_start, work_ratio)."""
    rp, rp_p = _host(graph_rowptr, np.int64)
    ci, ci_p = _host(graph_adj, np.int32)
    if len(rp) != M + 1 or len(ci) != rp[-1]:
        raise ValueError("graph array lengths do not match M")
    parent, seq = np.empty(M, np.int32), np.empty(M, np.int32)
    seg = np.empty(M + 1, np.int32)
    work = ctypes.c_double()
    nseg = load().acc_spmm_dendrogram_host(M, rp_p, ci_p, segment_length, parent.ctypes.data, seq.ctypes.data,
                                           seg.ctypes.data, ctypes.byref(work))
    if nseg < 0:
        _raise()
    return parent, seq, seg[: nseg + 1].copy(), work.value


def acc_spmm_schedule_host(row_window_offset, load_balance=ACC_SPMM_AUTO, max_tiles_per_item=0, ibd_threshold=0.0):
    """Host stage of the plan: returns (items[n,4] int32, ibd, num_partial_slots)."""
    rwo, rwo_p = _host(row_window_offset, np.int32)
    W = len(rwo) - 1
    ibd, slots = ctypes.c_double(), ctypes.c_int64()
    L = load()
    n = L.acc_spmm_schedule_host(W, rwo_p, load_balance, max_tiles_per_item, ibd_threshold, ctypes.byref(ibd), None, 0,
                                 ctypes.byref(slots))
    if n < 0:
        _raise()
    items = np.empty((n, 4), np.int32)
    n2 = L.acc_spmm_schedule_host(W, rwo_p, load_balance, max_tiles_per_item, ibd_threshold, None, items.ctypes.data, n,
                                  None)
    if n2 != n:
        _raise()
    return items, ibd.value, slots.value
