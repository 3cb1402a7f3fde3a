"""Thin ctypes binding of libsparsecontract's C ABI (include/sparsecontract.h).

Argument marshalling only: every step of a contraction runs in the library's HIP
kernels.  Function names mirror the C entry points (``sc_plan_create`` ->
``plan_create`` ...).  Device buffers are passed as raw addresses; PyTorch is
used by callers purely as an allocator of device memory and a source of HIP
streams (``tensor.data_ptr()``, ``torch.cuda.current_stream().cuda_stream``).

There is no CPU fallback: if the shared library has not been built the import of
the library fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparsecontract.so")

SC_F32, SC_F64 = 0, 1
SC_SCHED_LINEAR, SC_SCHED_FUSED, SC_SCHED_FISSIONED, SC_SCHED_AUTO = 0, 1, 2, 3

STATUS_NAMES = [
    "SC_OK", "SC_ERR_NULL", "SC_ERR_BAD_ORDER", "SC_ERR_BAD_DTYPE", "SC_ERR_BAD_DIMS", "SC_ERR_BAD_POS",
    "SC_ERR_CRD_RANGE", "SC_ERR_UNSORTED", "SC_ERR_DUPLICATE", "SC_ERR_EXPR_PARSE", "SC_ERR_EXPR_UNSUPPORTED",
    "SC_ERR_SCHED_UNSUPPORTED", "SC_ERR_SHAPE_MISMATCH", "SC_ERR_WORKSPACE_SMALL", "SC_ERR_DEVICE", "SC_ERR_ALLOC",
]

# every symbol include/sparsecontract.h declares
EXPORTS = [
    "sc_version", "sc_status_string", "sc_coo_to_csf_sizes", "sc_coo_to_csf", "sc_plan_create",
    "sc_plan_workspace_bytes", "sc_plan_describe", "sc_plan_model", "sc_plan_intermediate", "sc_execute",
    "sc_plan_set_profiling", "sc_plan_kernel_count", "sc_plan_kernel_time", "sc_plan_tile_count", "sc_plan_tile",
    "sc_tuning_set", "sc_stream_copy", "sc_plan_destroy", "sc_execute_static", "sc_plan_chosen",
]

_c_i32p = ctypes.POINTER(ctypes.c_int32)


class CooView(ctypes.Structure):
    _fields_ = [("order", ctypes.c_int32), ("dims", ctypes.c_int64 * 4), ("nnz", ctypes.c_int64),
                ("dtype", ctypes.c_int), ("crd", ctypes.c_void_p * 4), ("vals", ctypes.c_void_p),
                ("on_device", ctypes.c_int32)]


class CsfView(ctypes.Structure):
    _fields_ = [("order", ctypes.c_int32), ("dims", ctypes.c_int64 * 4), ("nnz", ctypes.c_int64),
                ("dtype", ctypes.c_int), ("nfib", ctypes.c_int64 * 4), ("pos", ctypes.c_void_p * 4),
                ("crd", ctypes.c_void_p * 4), ("vals", ctypes.c_void_p), ("on_device", ctypes.c_int32)]


class DenseView(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int)]


class Schedule(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("n_intermediates", ctypes.c_int32),
                ("intermediate", ctypes.c_char_p * 2), ("fuse_depth", ctypes.c_int32 * 2),
                ("deterministic", ctypes.c_int32)]


class ScError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__(f"{where}: {name}: {status_string(status)}")


_lib = None


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2311_09549_amd.build` "
                "(there is no CPU fallback)")
        # torch ships a HIP runtime of its own and must load it before this library does: the
        # library then binds to that copy.  In the other order the process ends up with two
        # runtimes and torch finds no device.
        import torch  # noqa: F401
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.sc_status_string.restype = ctypes.c_char_p
        _lib.sc_status_string.argtypes = [ctypes.c_int]
        for name in EXPORTS:
            if name != "sc_status_string":
                getattr(_lib, name).restype = ctypes.c_int
    return _lib


def status_string(status: int) -> str:
    return lib().sc_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise ScError(status, where)


def version():
    major, minor = ctypes.c_int(), ctypes.c_int()
    _check(lib().sc_version(ctypes.byref(major), ctypes.byref(minor)), "sc_version")
    return major.value, minor.value


def _dtype_code(dt) -> int:
    dt = np.dtype(dt) if not isinstance(dt, str) or dt not in ("f32", "f64") else np.dtype(
        np.float32 if dt == "f32" else np.float64)
    if dt == np.float32:
        return SC_F32
    if dt == np.float64:
        return SC_F64
    raise TypeError(f"unsupported dtype {dt}")


def _addr(x) -> int:
    """Raw address of a numpy array, a torch tensor, an int or None."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return int(x.data_ptr())


def coo_view(coords, vals, dims, dtype=None, on_device=False) -> CooView:
    v = CooView()
    v.order = len(dims)
    for m, d in enumerate(dims):
        v.dims[m] = int(d)
    v.nnz = int(coords[0].shape[0]) if len(coords) else 0
    v.dtype = _dtype_code(dtype if dtype is not None else vals.dtype)
    for m in range(len(coords)):
        v.crd[m] = _addr(coords[m])
    v.vals = _addr(vals)
    v.on_device = int(on_device)
    return v


class Csf:
    """CSF arrays (numpy on the host, or torch tensors on the device) plus their view."""

    def __init__(self, order, dims, nnz, dtype_code, nfib, pos, crd, vals, on_device):
        self.order, self.dims, self.nnz, self.dtype_code = order, tuple(int(d) for d in dims), int(nnz), dtype_code
        self.nfib = tuple(int(n) for n in nfib)
        self.pos, self.crd, self.vals, self.on_device = pos, crd, vals, bool(on_device)

    def view(self) -> CsfView:
        v = CsfView()
        v.order = self.order
        v.nnz = self.nnz
        v.dtype = self.dtype_code
        for m in range(self.order):
            v.dims[m] = self.dims[m]
            v.nfib[m] = self.nfib[m]
            v.pos[m] = _addr(self.pos[m]) if m else 0
            v.crd[m] = _addr(self.crd[m])
        v.vals = _addr(self.vals)
        v.on_device = int(self.on_device)
        return v

    def to_device(self, device="cuda"):
        import torch
        pos = [None] + [torch.from_numpy(p).to(device) for p in self.pos[1:]]
        crd = [torch.from_numpy(c).to(device) for c in self.crd]
        vals = torch.from_numpy(self.vals).to(device)
        return Csf(self.order, self.dims, self.nnz, self.dtype_code, self.nfib, pos, crd, vals, True)


def coo_to_csf_sizes(coords, vals, dims):
    v = coo_view(coords, vals, dims)
    nfib = (ctypes.c_int64 * 4)()
    _check(lib().sc_coo_to_csf_sizes(ctypes.byref(v), nfib), "sc_coo_to_csf_sizes")
    return [int(nfib[m]) for m in range(len(dims))]


def coo_to_csf(coords, vals, dims) -> Csf:
    """Host conversion of a sorted, duplicate-free coordinate list into CSF level arrays."""
    coords = [np.ascontiguousarray(c, dtype=np.int32) for c in coords]
    vals = np.ascontiguousarray(vals)
    order = len(dims)
    nfib = coo_to_csf_sizes(coords, vals, dims)
    pos = [None] + [np.empty(nfib[m - 1] + 1, dtype=np.int32) for m in range(1, order)]
    crd = [np.empty(nfib[m], dtype=np.int32) for m in range(order)]
    out = CsfView()
    for m in range(order):
        out.pos[m] = _addr(pos[m]) if m else 0
        out.crd[m] = _addr(crd[m])
    out.vals = 0  # the leaf order equals the COO order: reuse the value array
    cv = coo_view(coords, vals, dims)
    _check(lib().sc_coo_to_csf(ctypes.byref(cv), ctypes.byref(out)), "sc_coo_to_csf")
    return Csf(order, dims, out.nnz, out.dtype, [out.nfib[m] for m in range(order)], pos, crd, vals, False)


def dense_view(x, dtype=None, rows=None, cols=None, ld=None) -> DenseView:
    """View of a 2-D row-major numpy array / torch tensor (or of a bare shape when x is None)."""
    v = DenseView()
    if x is None:
        v.data, v.rows, v.cols, v.ld = 0, int(rows), int(cols), int(ld if ld is not None else cols)
        v.dtype = _dtype_code(dtype)
        return v
    r, c = int(x.shape[0]), int(x.shape[1])
    if isinstance(x, np.ndarray):
        assert x.strides[1] == x.itemsize
        stride = x.strides[0] // x.itemsize
        code = _dtype_code(x.dtype)
    else:
        assert x.stride(1) == 1
        stride = int(x.stride(0))
        code = SC_F64 if x.element_size() == 8 else SC_F32
    v.data, v.rows, v.cols, v.ld, v.dtype = _addr(x), r, c, stride, code
    return v


def schedule(kind, intermediates=(), fuse_depth=(), deterministic=False) -> Schedule:
    s = Schedule()
    s.kind = {"linear": SC_SCHED_LINEAR, "fused": SC_SCHED_FUSED, "fissioned": SC_SCHED_FISSIONED, "auto": SC_SCHED_AUTO}.get(kind, kind)
    s.n_intermediates = len(intermediates)
    for t, name in enumerate(list(intermediates)[:2]):
        s.intermediate[t] = name.encode() if name is not None else None
    for t, d in enumerate(list(fuse_depth)[:2]):
        s.fuse_depth[t] = int(d)
    s.deterministic = int(deterministic)
    return s


class Plan:
    def __init__(self, handle):
        self._h = handle

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "_h", None) and _lib is not None:
            try:
                _lib.sc_plan_destroy(self._h)
            except Exception:  # interpreter shutdown
                pass
            self._h = None

    @property
    def handle(self):
        return self._h


def plan_create(expr: str, csf: Csf, factors, sched: Schedule) -> Plan:
    """factors: list of DenseView (only rows / cols / dtype are read) or arrays."""
    fv = (DenseView * len(factors))(*[f if isinstance(f, DenseView) else dense_view(f) for f in factors])
    h = ctypes.c_void_p()
    view = csf.view()
    st = lib().sc_plan_create(ctypes.byref(h), expr.encode(), ctypes.byref(view), fv, ctypes.c_int32(len(factors)),
                              ctypes.byref(sched))
    _check(st, "sc_plan_create")
    return Plan(h)


def plan_workspace_bytes(plan: Plan) -> int:
    n = ctypes.c_size_t()
    _check(lib().sc_plan_workspace_bytes(plan.handle, ctypes.byref(n)), "sc_plan_workspace_bytes")
    return int(n.value)


def plan_describe(plan: Plan) -> str:
    buf = ctypes.create_string_buffer(4096)
    _check(lib().sc_plan_describe(plan.handle, buf, ctypes.c_size_t(len(buf))), "sc_plan_describe")
    return buf.value.decode()


def plan_chosen(plan: Plan):
    """(schedule class name, schedule of Table 2 kernel 5 or 0) the plan runs."""
    kind, variant = ctypes.c_int(), ctypes.c_int32()
    _check(lib().sc_plan_chosen(plan.handle, ctypes.byref(kind), ctypes.byref(variant)), "sc_plan_chosen")
    return ["linear", "fused", "fissioned", "auto"][kind.value], int(variant.value)


def plan_model(plan: Plan):
    fl, by = ctypes.c_double(), ctypes.c_double()
    _check(lib().sc_plan_model(plan.handle, ctypes.byref(fl), ctypes.byref(by)), "sc_plan_model")
    return fl.value, by.value


def plan_intermediate(plan: Plan, index: int):
    off, rows, cols = ctypes.c_size_t(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib().sc_plan_intermediate(plan.handle, ctypes.c_int32(index), ctypes.byref(off), ctypes.byref(rows),
                                      ctypes.byref(cols)), "sc_plan_intermediate")
    return int(off.value), int(rows.value), int(cols.value)


def plan_tile_count(plan: Plan) -> int:
    n = ctypes.c_int64()
    _check(lib().sc_plan_tile_count(plan.handle, ctypes.byref(n)), "sc_plan_tile_count")
    return int(n.value)


def plan_tile(plan: Plan, index: int):
    rec = (ctypes.c_int32 * 9)()
    _check(lib().sc_plan_tile(plan.handle, ctypes.c_int64(index), rec), "sc_plan_tile")
    return [int(x) for x in rec]


def tuning_set(name: str, value: int):
    _check(lib().sc_tuning_set(name.encode(), ctypes.c_int64(value)), "sc_tuning_set")


def stream_copy(dst, src, nbytes: int, stream=0):
    """Queues the library's plain copy kernel (counter calibration) on `stream`."""
    _check(lib().sc_stream_copy(ctypes.c_void_p(_addr(dst)), ctypes.c_void_p(_addr(src)), ctypes.c_size_t(int(nbytes)),
                                ctypes.c_void_p(int(stream))), "sc_stream_copy")


def execute(plan: Plan, csf: Csf, factors, out, workspace=None, workspace_bytes=0, stream=0):
    """Queues the contraction on `stream` (a raw hipStream_t address, 0 = default stream)."""
    fv = (DenseView * len(factors))(*[f if isinstance(f, DenseView) else dense_view(f) for f in factors])
    view = csf.view()
    st = lib().sc_execute(plan.handle, ctypes.byref(view), fv, ctypes.c_int32(len(factors)),
                          ctypes.c_void_p(_addr(out)), ctypes.c_void_p(_addr(workspace)),
                          ctypes.c_size_t(int(workspace_bytes)), ctypes.c_void_p(int(stream)))
    _check(st, "sc_execute")


STATIC_WORKSPACE_BYTES = 32 << 20   # SC_STATIC_WORKSPACE_BYTES of the header


def execute_static(plan: Plan, csf: Csf, factors, out, stream=0):
    """sc_execute with the library's own fixed scratch array as the workspace (allocates nothing)."""
    fv = (DenseView * len(factors))(*[f if isinstance(f, DenseView) else dense_view(f) for f in factors])
    view = csf.view()
    st = lib().sc_execute_static(plan.handle, ctypes.byref(view), fv, ctypes.c_int32(len(factors)),
                                 ctypes.c_void_p(_addr(out)), ctypes.c_void_p(int(stream)))
    _check(st, "sc_execute_static")


def plan_set_profiling(plan: Plan, on: bool):
    _check(lib().sc_plan_set_profiling(plan.handle, ctypes.c_int32(int(on))), "sc_plan_set_profiling")


def plan_kernel_times(plan: Plan):
    """[(kernel name, milliseconds)] of the most recent execute (stream must be synchronised)."""
    n = ctypes.c_int32()
    _check(lib().sc_plan_kernel_count(plan.handle, ctypes.byref(n)), "sc_plan_kernel_count")
    res = []
    for i in range(n.value):
        name = ctypes.create_string_buffer(64)
        ms = ctypes.c_float()
        _check(lib().sc_plan_kernel_time(plan.handle, ctypes.c_int32(i), name, ctypes.c_size_t(64), ctypes.byref(ms)),
               "sc_plan_kernel_time")
        res.append((name.value.decode(), float(ms.value)))
    return res
