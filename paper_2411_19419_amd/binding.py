"""Thin ctypes binding over libconvspmv.so: argument marshalling only.

Names and meanings are those of ``include/convspmv.h``.  torch supplies device
memory and the stream handle; every step of the path runs in the library's
HIP kernels.  There is no fallback: if the shared library is missing or a call
fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
import threading

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIBNAME = "libconvspmv.so"
_lock = threading.Lock()
_lib = None

EXPORTS = (
    "conv_out_shape", "conv_nnz", "conv_csr_build", "conv_spmv", "conv_plan_shape",
    "conv_spmv_variant", "conv_plan_destroy", "conv_strerror", "conv_last_hip_error",
    "conv_plan_set_march_min_jobs", "conv_test_dispatch_info", "conv_update_kernel", "conv_csr_fill_noalloc",
    "conv_multi_create", "conv_multi_apply", "conv_multi_destroy",
    "conv_csc_build", "conv_plan_is_transposed",
    "conv_compact_build", "conv_plan_is_compact",
    "conv_csr_build_channels", "conv_plan_channels", "conv_spmv_from_csc", "conv_dispatch_info",
    "conv_compact_build_channels",
)


class ConvDispatch(ctypes.Structure):
    """conv_dispatch of include/convspmv.h."""
    _fields_ = [("kernel", ctypes.c_int), ("threads", ctypes.c_int), ("lds_bytes", ctypes.c_int64),
                ("workgroups", ctypes.c_int64), ("strip", ctypes.c_int), ("segment", ctypes.c_int),
                ("ring_lines", ctypes.c_int), ("ring_lines_needed", ctypes.c_int), ("lines_per_step", ctypes.c_int),
                ("lanes_per_row", ctypes.c_int), ("columns_per_lane", ctypes.c_int)]


class ConvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, conv_strerror(status), status))


def library_path() -> str:
    return os.path.join(_HERE, _LIBNAME)


def _load():
    global _lib
    with _lock:
        if _lib is not None:
            return _lib
        path = library_path()
        if not os.path.exists(path):
            raise ImportError(
                "%s is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "from the repository root (hipcc --offload-arch=gfx950)" % path)
        lib = ctypes.CDLL(path)
        i, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
        pi, pi64 = ctypes.POINTER(i), ctypes.POINTER(i64)
        lib.conv_out_shape.argtypes = [i, i, i, i, i, pi, pi]
        lib.conv_out_shape.restype = i
        lib.conv_nnz.argtypes = [i, i, i, i, i]
        lib.conv_nnz.restype = i64
        lib.conv_csr_build.argtypes = [i, i, i, i, i, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
        lib.conv_csr_build.restype = i
        lib.conv_csc_build.argtypes = [i, i, i, i, i, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
        lib.conv_csc_build.restype = i
        lib.conv_plan_is_transposed.argtypes = [vp]
        lib.conv_plan_is_transposed.restype = i
        lib.conv_compact_build.argtypes = [i, i, i, i, i, vp, vp, vp, vp, ctypes.POINTER(vp)]
        lib.conv_compact_build.restype = i
        lib.conv_compact_build_channels.argtypes = [i, i, i, i, i, i, vp, vp, vp, vp, ctypes.POINTER(vp)]
        lib.conv_compact_build_channels.restype = i
        lib.conv_plan_is_compact.argtypes = [vp]
        lib.conv_plan_is_compact.restype = i
        lib.conv_csr_build_channels.argtypes = [i, i, i, i, i, i, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
        lib.conv_csr_build_channels.restype = i
        lib.conv_plan_channels.argtypes = [vp]
        lib.conv_plan_channels.restype = i
        lib.conv_spmv_from_csc.argtypes = [vp, vp, vp, i, vp]
        lib.conv_spmv_from_csc.restype = i
        lib.conv_dispatch_info.argtypes = [i] * 8 + [ctypes.POINTER(ConvDispatch)]
        lib.conv_dispatch_info.restype = i
        lib.conv_spmv.argtypes = [vp, vp, vp, i, vp]
        lib.conv_spmv.restype = i
        lib.conv_plan_shape.argtypes = [vp, pi, pi, pi, pi, pi, pi, pi, pi64]
        lib.conv_plan_shape.restype = i
        lib.conv_spmv_variant.argtypes = [vp, i]
        lib.conv_spmv_variant.restype = ctypes.c_char_p
        lib.conv_plan_destroy.argtypes = [vp]
        lib.conv_plan_destroy.restype = i
        lib.conv_strerror.argtypes = [i]
        lib.conv_strerror.restype = ctypes.c_char_p
        lib.conv_last_hip_error.argtypes = []
        lib.conv_last_hip_error.restype = i
        lib.conv_multi_create.argtypes = [i, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), i,
                                          ctypes.POINTER(vp)]
        lib.conv_multi_create.restype = i
        lib.conv_multi_apply.argtypes = [vp, vp]
        lib.conv_multi_apply.restype = i
        lib.conv_multi_destroy.argtypes = [vp]
        lib.conv_multi_destroy.restype = i
        lib.conv_update_kernel.argtypes = [vp, vp, vp]
        lib.conv_update_kernel.restype = i
        lib.conv_plan_set_march_min_jobs.argtypes = [vp, i]
        lib.conv_plan_set_march_min_jobs.restype = i
        lib.conv_test_dispatch_info.argtypes = [i] * 9 + [ctypes.POINTER(ConvDispatch)]
        lib.conv_test_dispatch_info.restype = i
        lib.conv_csr_fill_noalloc.argtypes = [i, i, i, i, i, vp, vp, vp, vp, vp]
        lib.conv_csr_fill_noalloc.restype = i
        _lib = lib
        return lib


def conv_strerror(status: int) -> str:
    return _load().conv_strerror(int(status)).decode()


def conv_plan_set_march_min_jobs(plan, jobs: int) -> int:
    """Test hook: the plan's threshold for the marching kernels; returns the previous value."""
    prev = _load().conv_plan_set_march_min_jobs(plan._handle, int(jobs))
    if prev < 0:
        raise ConvError(prev, "conv_plan_set_march_min_jobs(%r)" % (jobs,))
    return prev


def conv_dispatch_info(m, n, k, s, p, batch=1, storage=0, channels=1, march_min_jobs=None) -> ConvDispatch:
    """What conv_spmv would launch for this shape (host only, no GPU needed).  march_min_jobs:
    the test hook's threshold (conv_test_dispatch_info) instead of the default."""
    d = ConvDispatch()
    if march_min_jobs is None:
        st = _load().conv_dispatch_info(m, n, k, s, p, int(batch), int(storage), int(channels), ctypes.byref(d))
    else:
        st = _load().conv_test_dispatch_info(m, n, k, s, p, int(batch), int(storage), int(channels),
                                             int(march_min_jobs), ctypes.byref(d))
    if st != 0:
        raise ConvError(st, "conv_dispatch_info%r" % ((m, n, k, s, p, batch, storage, channels),))
    return d


def conv_out_shape(m, n, k, s, p):
    mo, no = ctypes.c_int(), ctypes.c_int()
    st = _load().conv_out_shape(m, n, k, s, p, ctypes.byref(mo), ctypes.byref(no))
    if st != 0:
        raise ConvError(st, "conv_out_shape%r" % ((m, n, k, s, p),))
    return mo.value, no.value


def conv_nnz(m, n, k, s, p) -> int:
    v = int(_load().conv_nnz(m, n, k, s, p))
    if v < 0:
        raise ConvError(v, "conv_nnz%r" % ((m, n, k, s, p),))
    return v


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream), stream


def _on_stream(stream, *tensors):
    """Tensors that this binding allocated (on torch's current stream) and that the library's
    kernels use on `stream`: tell the caching allocator, so that a block is not handed to other
    work while those kernels may still touch it."""
    import torch
    if stream is None or stream == torch.cuda.current_stream():
        return
    for t in tensors:
        if t is not None and t.numel():
            t.record_stream(stream)


class ConvPlan:
    """A built T: the three CSR tensors (torch, device) plus the library's
    plan handle that borrows them."""

    def __init__(self, handle, shape, out_shape, nnz, row_ptr, col_idx, vals, kernel, transposed=False):
        self._handle = handle
        self.transposed = transposed    # the arrays hold T^T (CSC of T): row_ptr is col_ptr, col_idx is row_idx
        self.m, self.n, self.k, self.s, self.p = shape
        self.m_out, self.n_out = out_shape
        self.nnz = nnz
        self.row_ptr, self.col_idx, self.vals = row_ptr, col_idx, vals
        self._kernel = kernel           # keep K alive until the build has run
        self.compact = False
        self.row_desc = self.ktab = None   # structure-aware storage (conv_compact_build)
        self.channels = 1                  # input channels sharing the indices (conv_csr_build_channels)

    @property
    def rows(self):
        return self.m * self.n if self.transposed else self.m_out * self.n_out

    @property
    def cols(self):
        return self.m_out * self.n_out if self.transposed else self.m * self.n * self.channels

    def variant(self, batch: int) -> str:
        v = _load().conv_spmv_variant(self._handle, int(batch))
        return v.decode() if v else ""

    def model_bytes(self, batch: int) -> int:
        """Bytes a CSR SpMM has to move: entries (index + value), row_ptr,
        x once, y once."""
        if self.compact:    # descriptors and the value table instead of the entries
            return (self.rows * 8 + self.k * self.k * 4) * self.channels + self.cols * batch * 4 + self.rows * batch * 4
        return (self.nnz * 4 * (1 + self.channels) + (self.rows + 1) * 4 + self.cols * batch * 4
                + self.rows * batch * 4)

    def close(self):
        if self._handle is not None:
            import torch
            torch.cuda.synchronize()
            _load().conv_plan_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def conv_csc_build(m, n, k, s, p, kernel, stream=None) -> ConvPlan:
    """Build T column-compressed; the plan applies T^T (plan.row_ptr is col_ptr, plan.col_idx is row_idx)."""
    return conv_csr_build(m, n, k, s, p, kernel, stream=stream, _transposed=True)


def conv_csr_build(m, n, k, s, p, kernel, stream=None, _transposed=False) -> ConvPlan:
    """Build T on the device of `kernel` (a k*k float32 CUDA/HIP tensor)."""
    import torch
    lib = _load()
    mo, no = conv_out_shape(m, n, k, s, p)
    nnz = conv_nnz(m, n, k, s, p)
    if not (kernel.is_cuda and kernel.dtype == torch.float32 and kernel.is_contiguous()
            and kernel.numel() == k * k):
        raise ValueError("kernel must be a contiguous float32 device tensor with k*k elements")
    dev = kernel.device
    if nnz >= 2 ** 31 or mo * no >= 2 ** 31 - 1 or m * n >= 2 ** 31 - 1:
        raise ConvError(-3, "conv_csr_build%r" % ((m, n, k, s, p),))
    row_ptr = torch.empty((m * n if _transposed else mo * no) + 1, dtype=torch.int32, device=dev)
    col_idx = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)[:nnz]
    vals = torch.empty(max(nnz, 1), dtype=torch.float32, device=dev)[:nnz]
    handle = ctypes.c_void_p()
    with torch.cuda.device(dev):
        sh, _ = _stream_handle(stream)
        fn = lib.conv_csc_build if _transposed else lib.conv_csr_build
        st = fn(m, n, k, s, p, kernel.data_ptr(), row_ptr.data_ptr(),
                col_idx.data_ptr(), vals.data_ptr(), sh, ctypes.byref(handle))
    if st != 0:
        raise ConvError(st, "%s%r" % ("conv_csc_build" if _transposed else "conv_csr_build", (m, n, k, s, p)))
    _on_stream(stream, row_ptr, col_idx, vals)
    return ConvPlan(handle, (m, n, k, s, p), (mo, no), nnz, row_ptr, col_idx, vals, kernel, transposed=_transposed)


def conv_csr_fill_noalloc(m, n, k, s, p, kernel, row_ptr, col_idx, vals, stream=None) -> None:
    """The three CSR arrays of conv_csr_build written into caller-provided tensors, with no
    allocation by the library and no plan (see include/convspmv.h)."""
    import torch
    for t, dt in ((kernel, torch.float32), (row_ptr, torch.int32), (col_idx, torch.int32), (vals, torch.float32)):
        if not (t.is_cuda and t.dtype == dt and t.is_contiguous()):
            raise ValueError("operands must be contiguous device tensors of the documented types")
    mo, no = conv_out_shape(m, n, k, s, p)
    nnz = conv_nnz(m, n, k, s, p)
    if kernel.numel() != k * k or row_ptr.numel() != mo * no + 1 or col_idx.numel() < nnz or vals.numel() < nnz:
        raise ValueError("operand sizes do not match the shape")
    with torch.cuda.device(kernel.device):
        sh, _ = _stream_handle(stream)
        st = _load().conv_csr_fill_noalloc(m, n, k, s, p, kernel.data_ptr(), row_ptr.data_ptr(),
                                           col_idx.data_ptr() if nnz else None, vals.data_ptr() if nnz else None, sh)
    if st != 0:
        raise ConvError(st, "conv_csr_fill_noalloc%r" % ((m, n, k, s, p),))


def conv_csr_build_channels(m, n, k, s, p, kernels, channels, stream=None) -> ConvPlan:
    """Build [T_1 | ... | T_C]: shared row_ptr / col_idx, plan.vals holds `channels` arrays of nnz
    values one after the other.  `kernels`: channels*k*k float32 device tensor."""
    import torch
    lib = _load()
    mo, no = conv_out_shape(m, n, k, s, p)
    nnz = conv_nnz(m, n, k, s, p)
    if not (kernels.is_cuda and kernels.dtype == torch.float32 and kernels.is_contiguous()
            and channels >= 1 and kernels.numel() == channels * k * k):
        raise ValueError("kernels must be a contiguous float32 device tensor with channels*k*k elements")
    dev = kernels.device
    if nnz >= 2 ** 31 or mo * no >= 2 ** 31 - 1 or m * n * channels >= 2 ** 31 - 1:
        raise ConvError(-3, "conv_csr_build_channels%r" % ((m, n, k, s, p, channels),))
    row_ptr = torch.empty(mo * no + 1, dtype=torch.int32, device=dev)
    col_idx = torch.empty(max(nnz, 1), dtype=torch.int32, device=dev)[:nnz]
    vals = torch.empty(max(nnz * channels, 1), dtype=torch.float32, device=dev)[:nnz * channels]
    handle = ctypes.c_void_p()
    with torch.cuda.device(dev):
        sh, _ = _stream_handle(stream)
        st = lib.conv_csr_build_channels(m, n, k, s, p, int(channels), kernels.data_ptr(), row_ptr.data_ptr(),
                                         col_idx.data_ptr(), vals.data_ptr(), sh, ctypes.byref(handle))
    if st != 0:
        raise ConvError(st, "conv_csr_build_channels%r" % ((m, n, k, s, p, channels),))
    _on_stream(stream, row_ptr, col_idx, vals)
    plan = ConvPlan(handle, (m, n, k, s, p), (mo, no), nnz, row_ptr, col_idx, vals, kernels)
    plan.channels = int(channels)
    return plan


def conv_compact_build(m, n, k, s, p, kernel, stream=None, channels: int = 1) -> ConvPlan:
    """Build T in the structure-aware storage: plan.row_desc is int32 (rows, 2) = per row the
    column of its first entry and the packed tap ranges, plan.ktab the value table (k*k numbers
    per channel; with channels > 1 the plan computes the sum over the stacked input planes)."""
    import torch
    lib = _load()
    mo, no = conv_out_shape(m, n, k, s, p)
    nnz = conv_nnz(m, n, k, s, p)
    if not (kernel.is_cuda and kernel.dtype == torch.float32 and kernel.is_contiguous()
            and channels >= 1 and kernel.numel() == channels * k * k):
        raise ValueError("kernel must be a contiguous float32 device tensor with channels*k*k elements")
    dev = kernel.device
    if mo * no >= 2 ** 31 - 1 or m * n * channels >= 2 ** 31 - 1:
        raise ConvError(-3, "conv_compact_build%r" % ((m, n, k, s, p),))
    row_desc = torch.empty((mo * no, 2), dtype=torch.int32, device=dev)
    ktab = torch.empty(channels * k * k, dtype=torch.float32, device=dev)
    handle = ctypes.c_void_p()
    with torch.cuda.device(dev):
        sh, _ = _stream_handle(stream)
        st = lib.conv_compact_build_channels(m, n, k, s, p, int(channels), kernel.data_ptr(), row_desc.data_ptr(),
                                             ktab.data_ptr(), sh, ctypes.byref(handle))
    if st != 0:
        raise ConvError(st, "conv_compact_build%r" % ((m, n, k, s, p),))
    _on_stream(stream, row_desc, ktab)
    plan = ConvPlan(handle, (m, n, k, s, p), (mo, no), nnz, None, None, None, kernel)
    plan.compact = True
    plan.channels = int(channels)
    plan.row_desc, plan.ktab = row_desc, ktab
    return plan


def conv_update_kernel(plan: ConvPlan, kernel, stream=None) -> None:
    """Rewrite plan.vals for a new k*k kernel (device tensor); indices are untouched."""
    import torch
    if plan._handle is None:
        raise ValueError("plan is closed")
    if not (kernel.is_cuda and kernel.dtype == torch.float32 and kernel.is_contiguous()
            and kernel.numel() == plan.k * plan.k * plan.channels):
        raise ValueError("kernel must be a contiguous float32 device tensor with channels*k*k elements")
    with torch.cuda.device(kernel.device):
        sh, _ = _stream_handle(stream)
        st = _load().conv_update_kernel(plan._handle, kernel.data_ptr(), sh)
    if st != 0:
        raise ConvError(st, "conv_update_kernel")
    plan._kernel = kernel


def conv_spmv(plan: ConvPlan, x, y=None, batch: int = 1, stream=None):
    """y = T x for `batch` batch-minor vectors.  Allocates y when not given."""
    import torch
    if plan._handle is None:
        raise ValueError("plan is closed")
    if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()):
        raise ValueError("x must be a contiguous float32 device tensor")
    if batch >= 1 and x.numel() != plan.cols * batch:
        raise ValueError("x has %d elements, expected m*n*batch = %d" % (x.numel(), plan.cols * batch))
    if y is None:
        y = torch.empty(plan.rows * max(batch, 1), dtype=torch.float32, device=x.device)
        _on_stream(stream, y)
    elif not (y.is_cuda and y.dtype == torch.float32 and y.is_contiguous()
              and y.numel() == plan.rows * batch):
        raise ValueError("y must be a contiguous float32 device tensor with m_out*n_out*batch elements")
    if x.device.index == torch.cuda.current_device():        # the usual case: no device switch
        sh, _ = _stream_handle(stream)
        st = _load().conv_spmv(plan._handle, x.data_ptr(), y.data_ptr(), int(batch), sh)
    else:
        with torch.cuda.device(x.device):
            sh, _ = _stream_handle(stream)
            st = _load().conv_spmv(plan._handle, x.data_ptr(), y.data_ptr(), int(batch), sh)
    if st != 0:
        raise ConvError(st, "conv_spmv(batch=%d)" % batch)
    return y


def conv_spmv_from_csc(plan: ConvPlan, x, y=None, batch: int = 1, stream=None):
    """y = T x from the column-compressed arrays of a conv_csc_build plan (a scatter)."""
    import torch
    if plan._handle is None:
        raise ValueError("plan is closed")
    if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.numel() == plan.m * plan.n * batch):
        raise ValueError("x must be a contiguous float32 device tensor with m*n*batch elements")
    out = plan.m_out * plan.n_out * batch
    if y is None:
        y = torch.empty(out, dtype=torch.float32, device=x.device)
        _on_stream(stream, y)
    elif not (y.is_cuda and y.dtype == torch.float32 and y.is_contiguous() and y.numel() == out):
        raise ValueError("y must be a contiguous float32 device tensor with m_out*n_out*batch elements")
    with torch.cuda.device(x.device):
        sh, _ = _stream_handle(stream)
        st = _load().conv_spmv_from_csc(plan._handle, x.data_ptr(), y.data_ptr(), int(batch), sh)
    if st != 0:
        raise ConvError(st, "conv_spmv_from_csc(batch=%d)" % batch)
    return y


class ConvMulti:
    """n plans bound to their operands; apply() is one kernel launch for all of them."""

    def __init__(self, plans, xs, ys, batch: int = 1):
        import torch
        n = len(plans)
        if not (n == len(xs) == len(ys)) or n == 0:
            raise ValueError("plans, xs and ys must be non-empty and of equal length")
        for pl, x, y in zip(plans, xs, ys):
            if pl._handle is None:
                raise ValueError("a plan is closed")
            for t, size in ((x, pl.cols * batch), (y, pl.rows * batch)):
                if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == size):
                    raise ValueError("operands must be contiguous float32 device tensors of the plan's size")
        arr = ctypes.c_void_p * n
        handle = ctypes.c_void_p()
        with torch.cuda.device(xs[0].device):
            st = _load().conv_multi_create(n, arr(*[pl._handle for pl in plans]), arr(*[x.data_ptr() for x in xs]),
                                           arr(*[y.data_ptr() for y in ys]), int(batch), ctypes.byref(handle))
        if st != 0:
            raise ConvError(st, "conv_multi_create")
        self._handle = handle
        self._keep = (list(plans), list(xs), list(ys))     # borrowed by the library
        self.ys = list(ys)
        self.batch = batch

    def apply(self, stream=None):
        sh, _ = _stream_handle(stream)
        st = _load().conv_multi_apply(self._handle, sh)
        if st != 0:
            raise ConvError(st, "conv_multi_apply")
        return self.ys

    def close(self):
        if self._handle is not None:
            import torch
            torch.cuda.synchronize()
            _load().conv_multi_destroy(self._handle)
            self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
