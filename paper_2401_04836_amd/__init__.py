"""Python binding of the conststn C-ABI library (argument marshalling only).

Every step of the hot path -- CSF construction, partitioning, the fused contraction kernels
-- runs inside libconststn.so (HIP, gfx950).  PyTorch is used here for device memory and
streams, nothing else.  There is no CPU fallback: if the shared library is missing the
import of this package fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libconststn.so")

MAX_ORDER = 8
OK, EINVAL, ERANGE, EDUP, ESCHED, EUNSUPPORTED, ENOMEM, EHIP = range(8)
_STATUS_NAMES = ["OK", "EINVAL", "ERANGE", "EDUP", "ESCHED", "EUNSUPPORTED", "ENOMEM", "EHIP"]
COALESCE_DUPS = 1
OUT_COMPACT = 1
OPERAND_CSF, OPERAND_DENSE = 0, 1

EXPORTED_SYMBOLS = [
    "conststn_build_csf", "conststn_csf_info", "conststn_csf_export", "conststn_csf_destroy",
    "conststn_plan", "conststn_plan_options", "conststn_schedule_check", "conststn_schedule_search", "conststn_plan_output_size",
    "conststn_plan_output_rows", "conststn_plan_output_csf", "conststn_plan_describe", "conststn_plan_destroy",
    "conststn_execute", "conststn_last_error", "conststn_version",
    "conststn_plan_profile", "conststn_plan_kernel_times", "conststn_measure_peak", "conststn_execute_static",
    "conststn_csf_check", "conststn_plan_check",
]


class ConststnError(RuntimeError):
    def __init__(self, status, message):
        name = _STATUS_NAMES[status] if 0 <= status < len(_STATUS_NAMES) else str(status)
        super().__init__("conststn %s: %s" % (name, message))
        self.status = status
        self.status_name = name


class _OperandDesc(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("kind", ctypes.c_int), ("csf", ctypes.c_void_p),
                ("order", ctypes.c_int), ("dims", ctypes.c_int64 * MAX_ORDER)]


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2401_04836_amd.build` "
            "(hipcc, gfx950); there is no fallback path" % _LIB_PATH)
    L = ctypes.CDLL(_LIB_PATH)
    vp, i64p, ip = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int)
    L.conststn_last_error.restype = ctypes.c_char_p
    L.conststn_version.restype = ctypes.c_char_p
    L.conststn_build_csf.argtypes = [ctypes.c_int, i64p, ctypes.c_int64, ctypes.POINTER(vp), vp, ip,
                                     ctypes.c_uint, vp, ctypes.POINTER(vp)]
    L.conststn_csf_info.argtypes = [vp, ip, i64p, ip, i64p]
    L.conststn_csf_export.argtypes = [vp, ctypes.c_int, ctypes.POINTER(vp), ctypes.POINTER(vp), i64p,
                                      ctypes.POINTER(vp)]
    L.conststn_csf_destroy.argtypes = [vp]
    L.conststn_csf_destroy.restype = None
    L.conststn_plan.argtypes = [ctypes.c_char_p, ip, ctypes.c_int, ctypes.POINTER(_OperandDesc),
                                ctypes.c_uint, ctypes.POINTER(vp)]
    L.conststn_plan_options.argtypes = [ctypes.c_char_p, ip, ctypes.c_int, ctypes.POINTER(_OperandDesc),
                                        ctypes.c_uint, ctypes.c_char_p, ctypes.POINTER(vp)]
    L.conststn_schedule_check.argtypes = [ctypes.c_char_p, ip, ctypes.c_int, ctypes.POINTER(_OperandDesc),
                                          ctypes.c_char_p, ctypes.c_size_t, ip]
    L.conststn_schedule_search.argtypes = [ctypes.c_char_p, ctypes.c_int, ctypes.POINTER(_OperandDesc), ctypes.c_uint,
                                           ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t, ip, ip]
    L.conststn_plan_output_size.argtypes = [vp, i64p, i64p]
    L.conststn_plan_output_rows.argtypes = [vp, ctypes.POINTER(vp), i64p]
    L.conststn_plan_output_csf.argtypes = [vp, ctypes.POINTER(vp)]
    L.conststn_plan_describe.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t]
    L.conststn_plan_destroy.argtypes = [vp]
    L.conststn_plan_destroy.restype = None
    L.conststn_execute.argtypes = [vp, ctypes.POINTER(vp), vp, vp]
    L.conststn_execute_static.argtypes = [vp, ctypes.POINTER(vp), vp, vp]
    L.conststn_plan_profile.argtypes = [vp, ctypes.c_int]
    L.conststn_plan_kernel_times.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.c_int, ip]
    L.conststn_measure_peak.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double)]
    L.conststn_csf_check.argtypes = [vp]
    L.conststn_plan_check.argtypes = [vp]
    for name in EXPORTED_SYMBOLS:
        getattr(L, name)
    return L


_lib = _load()


def library_path():
    return _LIB_PATH


def version():
    return _lib.conststn_version().decode()


PEAK_COPY, PEAK_WRITE, PEAK_MFMA_F64, PEAK_MFMA_CLOCK, PEAK_VALU_CLOCK = 0, 1, 2, 3, 4


def measure_peak(what, size, repeats=5, stream=None):
    """Measured ceiling of the current device (GB/s for the copy and the fill, TFLOP/s for the matrix loop)."""
    r = ctypes.c_double(0.0)
    _check(_lib.conststn_measure_peak(int(what), int(size), int(repeats), _stream_handle(stream), ctypes.byref(r)))
    return r.value


def _check(status):
    if status != OK:
        raise ConststnError(status, _lib.conststn_last_error().decode())


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _borrow(ptr, count, dtype, device, owner):
    """A torch view of library-owned device memory (no copy); `owner` is kept alive by it."""
    if count == 0 or not ptr:
        return torch.empty(0, dtype=dtype, device=device)
    itemsize = torch.empty(0, dtype=dtype).element_size()

    class _Mem:
        pass
    m = _Mem()
    typestr = {torch.int32: "<i4", torch.int64: "<i8", torch.float64: "<f8"}[dtype]
    m.__cuda_array_interface__ = {"shape": (int(count),), "typestr": typestr,
                                  "data": (int(ptr), False), "version": 2, "strides": None}
    m._owner = owner
    t = torch.as_tensor(m, device=device)
    assert t.element_size() == itemsize
    return t


class CSF:
    """Handle of a device-resident CSF tensor (conststn_csf_t)."""

    def __init__(self, handle, device):
        self._h = handle
        self.device = device
        order = ctypes.c_int()
        dims = (ctypes.c_int64 * MAX_ORDER)()
        mo = (ctypes.c_int * MAX_ORDER)()
        nnz = ctypes.c_int64()
        _check(_lib.conststn_csf_info(self._h, ctypes.byref(order), dims, mo, ctypes.byref(nnz)))
        self.order = order.value
        self.dims = tuple(dims[i] for i in range(self.order))
        self.mode_order = tuple(mo[i] for i in range(self.order))
        self.nnz = nnz.value

    def export(self, level):
        """(idx, ptr, vals) device tensors of one level, borrowed from the handle."""
        idx, ptr, vals = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        nodes = ctypes.c_int64()
        _check(_lib.conststn_csf_export(self._h, level, ctypes.byref(idx), ctypes.byref(ptr),
                                        ctypes.byref(nodes), ctypes.byref(vals)))
        n = nodes.value
        ti = _borrow(idx.value, n, torch.int32, self.device, self)
        tp = _borrow(ptr.value, n + 1, torch.int64, self.device, self) if ptr.value else None
        tv = _borrow(vals.value, n, torch.float64, self.device, self) if vals.value else None
        return ti, tp, tv

    def check(self):
        """conststn_csf_check: every invariant of the level arrays, checked on the device (raises on a violation)."""
        _check(_lib.conststn_csf_check(self._h))

    def nodes(self, level):
        nodes = ctypes.c_int64()
        _check(_lib.conststn_csf_export(self._h, level, None, None, ctypes.byref(nodes), None))
        return nodes.value

    def destroy(self):
        if self._h:
            _lib.conststn_csf_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def build_csf(coords, vals, dims, mode_order, flags=0, stream=None):
    """conststn_build_csf: coords = list of int32 device tensors (one per mode), vals fp64."""
    order = len(dims)
    if len(coords) != order or len(mode_order) != order:
        raise ValueError("coords, dims and mode_order must have one entry per mode")
    device = vals.device
    if device.type != "cuda":
        raise ValueError("inputs must live on the GPU")
    keep = []
    cptrs = (ctypes.c_void_p * order)()
    for m in range(order):
        c = coords[m]
        if c.dtype != torch.int32 or c.device != device or c.numel() != vals.numel():
            raise ValueError("coords[%d] must be an int32 tensor on %s with nnz entries" % (m, device))
        c = c.contiguous()
        keep.append(c)
        cptrs[m] = c.data_ptr()
    if vals.dtype != torch.float64:
        raise ValueError("vals must be fp64")
    v = vals.contiguous()
    cdims = (ctypes.c_int64 * order)(*[int(d) for d in dims])
    cmo = (ctypes.c_int * order)(*[int(m) for m in mode_order])
    out = ctypes.c_void_p()
    with torch.cuda.device(device):
        _check(_lib.conststn_build_csf(order, cdims, v.numel(), cptrs, ctypes.c_void_p(v.data_ptr()), cmo,
                                       flags, _stream_handle(stream), ctypes.byref(out)))
    return CSF(out, device)


def _make_descs(operands):
    """operands: list of (name, CSF) | (name, dense_tensor_or_shape) | (name, ("csf", level_dims))."""
    n = len(operands)
    descs = (_OperandDesc * n)()
    keep = []
    for o, (name, obj) in enumerate(operands):
        b = name.encode()
        keep.append(b)
        descs[o].name = b
        if isinstance(obj, CSF):
            descs[o].kind = OPERAND_CSF
            descs[o].csf = obj._h
            descs[o].order = obj.order
        elif isinstance(obj, tuple) and len(obj) == 2 and obj[0] == "csf":
            descs[o].kind = OPERAND_CSF
            descs[o].csf = None
            descs[o].order = len(obj[1])
            for l, d in enumerate(obj[1]):
                descs[o].dims[l] = int(d)
        else:
            shape = tuple(obj.shape) if hasattr(obj, "shape") else tuple(obj)
            descs[o].kind = OPERAND_DENSE
            descs[o].csf = None
            descs[o].order = len(shape)
            for l, d in enumerate(shape):
                descs[o].dims[l] = int(d)
    return descs, keep


def schedule_check(schedule, operands, fusion=None):
    """conststn_schedule_check (host only): returns (lowered_text, reduced_orders)."""
    descs, keep = _make_descs(operands)
    nst = schedule.count(";") + 1
    buf = ctypes.create_string_buffer(1 << 16)
    red = (ctypes.c_int * max(nst, 1))()
    cf = (ctypes.c_int * len(fusion))(*fusion) if fusion is not None else None
    _check(_lib.conststn_schedule_check(schedule.encode(), cf, len(operands), descs, buf, len(buf), red))
    return buf.value.decode(), [red[i] for i in range(nst)]


SEARCH_KEEP_LAYOUT = 1


def schedule_search(tree, operands, flags=0, max_order=0):
    """conststn_schedule_search (host only): returns (schedule_text, l, level_modes) where
    level_modes[o] lists, per level of operand o, the position of its mode in the tree's reference."""
    descs, keep = _make_descs(operands)
    buf = ctypes.create_string_buffer(1 << 16)
    l = ctypes.c_int()
    modes = (ctypes.c_int * (len(operands) * MAX_ORDER))()
    _check(_lib.conststn_schedule_search(tree.encode(), len(operands), descs, flags, max_order, buf, len(buf),
                                         ctypes.byref(l), modes))
    out = []
    for o in range(len(operands)):
        out.append([modes[o * MAX_ORDER + d] for d in range(MAX_ORDER) if modes[o * MAX_ORDER + d] >= 0])
    return buf.value.decode(), l.value, out


class Plan:
    """Handle of a validated schedule bound to its kernels (conststn_plan_t)."""

    def __init__(self, handle, operands, device):
        self._h = handle
        self._operands = operands          # keeps the CSF handles alive
        self.device = device
        # shapes of the dense operands in the order execute() takes them
        self._dense_shapes = [tuple(o.shape) if hasattr(o, "shape") else tuple(o) for o in operands
                              if not isinstance(o, CSF)]
        r, e = ctypes.c_int64(), ctypes.c_int64()
        _check(_lib.conststn_plan_output_size(self._h, ctypes.byref(r), ctypes.byref(e)))
        self.n_rows, self.row_elems = r.value, e.value

    def describe(self):
        buf = ctypes.create_string_buffer(1 << 16)
        _check(_lib.conststn_plan_describe(self._h, buf, len(buf)))
        return buf.value.decode()

    def check(self):
        """conststn_plan_check: the plan's tables stay inside the arrays they index (order-3 MTTKRP / TTMc plans)."""
        _check(_lib.conststn_plan_check(self._h))

    def output_rows(self):
        p, n = ctypes.c_void_p(), ctypes.c_int64()
        _check(_lib.conststn_plan_output_rows(self._h, ctypes.byref(p), ctypes.byref(n)))
        return _borrow(p.value, n.value, torch.int32, self.device, self)

    def output_csf(self):
        """conststn_plan_output_csf: structure of a sparse result (borrowed; lives as long as the plan)."""
        h = ctypes.c_void_p()
        _check(_lib.conststn_plan_output_csf(self._h, ctypes.byref(h)))
        csf = CSF(h, self.device)
        csf.destroy = lambda: None          # owned by the plan
        csf._plan = self
        return csf

    def profile(self, capacity):
        """conststn_plan_profile: keep `capacity` event pairs around the dominant kernel."""
        _check(_lib.conststn_plan_profile(self._h, int(capacity)))

    def kernel_times(self, max_n=4096):
        """conststn_plan_kernel_times: durations (ms) of the dominant kernel, oldest first."""
        buf = (ctypes.c_float * max_n)()
        n = ctypes.c_int()
        _check(_lib.conststn_plan_kernel_times(self._h, buf, max_n, ctypes.byref(n)))
        return [buf[i] for i in range(n.value)]

    def destroy(self):
        if self._h:
            _lib.conststn_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def plan(schedule, operands, fusion=None, flags=0, options=None):
    """conststn_plan / conststn_plan_options: operands = list of (name, CSF) or (name, dense tensor /
    shape); options = None, a "name=value,..." string or a dict of tuning options."""
    if isinstance(options, dict):
        options = ",".join("%s=%d" % (k, int(v)) for k, v in options.items())
    descs, keep = _make_descs(operands)
    cf = (ctypes.c_int * len(fusion))(*fusion) if fusion is not None else None
    out = ctypes.c_void_p()
    device = None
    for _, obj in operands:
        if isinstance(obj, CSF):
            device = obj.device
    if device is None:
        raise ValueError("a plan needs at least one CSF operand")
    with torch.cuda.device(device):
        _check(_lib.conststn_plan_options(schedule.encode(), cf, len(operands), descs, flags,
                                          options.encode() if options else None, ctypes.byref(out)))
    return Plan(out, [obj for _, obj in operands], device)


def _marshal_execute(pl, dense_factors, out):
    n = len(dense_factors)
    if n != len(pl._dense_shapes):
        raise ValueError("the plan has %d dense operands, %d were given" % (len(pl._dense_shapes), n))
    ptrs = (ctypes.c_void_p * max(n, 1))()
    for d, f in enumerate(dense_factors):
        if f.dtype != torch.float64 or f.device != pl.device:
            raise ValueError("dense factor %d must be an fp64 tensor on %s" % (d, pl.device))
        if tuple(f.shape) != pl._dense_shapes[d]:
            raise ValueError("dense factor %d has shape %s, the plan was made for %s"
                             % (d, tuple(f.shape), pl._dense_shapes[d]))
        if not f.is_contiguous():
            # no hidden copy: it would be made on torch's current stream and freed while the kernels,
            # enqueued on the caller's stream, may still read it
            raise ValueError("dense factor %d must be contiguous (row-major)" % d)
        ptrs[d] = f.data_ptr()
    if out is None:
        out = torch.empty(pl.n_rows * pl.row_elems, dtype=torch.float64, device=pl.device)
    elif out.dtype != torch.float64 or out.device != pl.device or out.numel() != pl.n_rows * pl.row_elems \
            or not out.is_contiguous():
        raise ValueError("out must be a contiguous fp64 tensor of n_rows*row_elems elements")
    return ptrs, out


def execute(pl, dense_factors, out=None, stream=None):
    """conststn_execute: dense_factors in the order the dense operands were listed in plan()."""
    ptrs, out = _marshal_execute(pl, dense_factors, out)
    with torch.cuda.device(pl.device):
        _check(_lib.conststn_execute(pl._h, ptrs, ctypes.c_void_p(out.data_ptr()), _stream_handle(stream)))
    return out


def execute_static(pl, dense_factors, out, stream=None):
    """conststn_execute_static: as execute(), with the library's static scratch array; `out` is
    required (the call itself allocates nothing)."""
    if out is None:
        raise ValueError("execute_static needs the output tensor")
    ptrs, out = _marshal_execute(pl, dense_factors, out)
    with torch.cuda.device(pl.device):
        _check(_lib.conststn_execute_static(pl._h, ptrs, ctypes.c_void_p(out.data_ptr()), _stream_handle(stream)))
    return out
