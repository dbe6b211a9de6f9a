"""Thin ctypes binding of the C ABI in include/fq.h (same names, argument marshalling only).

Every step of the computation runs in the HIP kernels of libfq.so; nothing here does
arithmetic on tensor data and there is no CPU fallback: importing this module raises if the
compiled library is missing (build it with `python -m paper_2511_12653_amd.build` or
`__graft_entry__.build()`).

PyTorch is used by callers only to own device memory and streams; `FqTensor.from_torch`
reads data pointers and shapes from torch tensors, and `stream=None` means torch's current
stream.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfq.so")

FQ_F16, FQ_F32 = 0, 1
FQ_FLAG_NO_DX, FQ_FLAG_TWO_PASS = 1, 2
FQ_MODE_FORWARD, FQ_MODE_BACKWARD = 1, 2
FLT_MIN = 1.1754943508222875e-38


def library_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libfq.so is not built (%s missing); run `python -m paper_2511_12653_amd.build`. "
            "There is no CPU fallback." % _LIB_PATH)
    return ctypes.CDLL(_LIB_PATH)


class FqAdam(ctypes.Structure):
    """Mirror of `struct fq_adam` (host struct; m, v, theta_out are device pointers)."""
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("step", ctypes.c_int64),
                ("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("theta_out", ctypes.c_void_p)]

    @classmethod
    def from_torch(cls, m, v, theta_out, lr, beta1=0.9, beta2=0.999, eps=1e-8, step=1):
        import torch
        for t in (m, v, theta_out):
            if t.dtype != torch.float32 or not t.is_contiguous():
                raise TypeError("Adam state must be contiguous float32")
        return cls(lr, beta1, beta2, eps, step, m.data_ptr(), v.data_ptr(), theta_out.data_ptr())


class FqTensor(ctypes.Structure):
    """Mirror of `struct fq_tensor` (host struct holding device pointers)."""
    _fields_ = [
        ("outer", ctypes.c_int64), ("channels", ctypes.c_int64), ("inner", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("qmin", ctypes.c_int32), ("qmax", ctypes.c_int32),
        ("eps", ctypes.c_float), ("s_min", ctypes.c_float), ("s_max", ctypes.c_float),
        ("flags", ctypes.c_uint32),
        ("x", ctypes.c_void_p), ("y", ctypes.c_void_p), ("q", ctypes.c_void_p),
        ("theta", ctypes.c_void_p), ("s", ctypes.c_void_p),
        ("gy", ctypes.c_void_p), ("gx", ctypes.c_void_p),
        ("gs", ctypes.c_void_p), ("gtheta", ctypes.c_void_p),
        ("adam", ctypes.POINTER(FqAdam)),
    ]

    def set_adam(self, adam):
        """Attach (or with None detach) a fused Adam step; keeps the FqAdam object alive."""
        self._adam_ref = adam
        self.adam = ctypes.pointer(adam) if adam is not None else ctypes.POINTER(FqAdam)()
        return self

    @classmethod
    def from_torch(cls, outer, channels, inner, qmin, qmax, x=None, y=None, q=None, theta=None,
                   s=None, gy=None, gx=None, gs=None, gtheta=None, eps=0.0, s_min=FLT_MIN,
                   s_max=float("inf"), flags=0, dtype=None, adam=None):
        """Marshal torch tensors (device memory owned by the caller) into a descriptor."""
        import torch

        def ptr(t, want_dtype=None):
            if t is None:
                return None
            if not t.is_contiguous():
                raise ValueError("tensors must be contiguous")
            if want_dtype is not None and t.dtype != want_dtype:
                raise TypeError("expected %s, got %s" % (want_dtype, t.dtype))
            return t.data_ptr()

        ref = x if x is not None else gy
        if dtype is None:
            if ref is None:
                raise ValueError("dtype needed when no data tensor is given")
            dtype = {torch.float16: FQ_F16, torch.float32: FQ_F32}[ref.dtype]
        tdt = torch.float16 if dtype == FQ_F16 else torch.float32
        n = outer * channels * inner
        for t in (x, y, gy, gx, q):
            if t is not None and t.numel() != n:
                raise ValueError("tensor has %d elements, view says %d" % (t.numel(), n))
        for t in (theta, s, gs, gtheta):
            if t is not None and t.numel() != channels:
                raise ValueError("per-channel tensor has %d elements, want %d" % (t.numel(), channels))
        t = cls(outer, channels, inner, dtype, qmin, qmax, eps, s_min, s_max, flags,
                ptr(x, tdt), ptr(y, tdt), ptr(q, torch.int8), ptr(theta, torch.float32),
                ptr(s, torch.float32), ptr(gy, tdt), ptr(gx, tdt), ptr(gs, torch.float32),
                ptr(gtheta, torch.float32))
        if adam is not None:
            t.set_adam(adam)
        return t


class FqDistill(ctypes.Structure):
    """Mirror of `struct fq_distill` (host struct; the pointers inside are device pointers)."""
    _fields_ = [("n", ctypes.c_int64), ("channels", ctypes.c_int64), ("inner", ctypes.c_int64),
                ("dtype", ctypes.c_int32), ("lam", ctypes.c_float), ("eps", ctypes.c_float),
                ("upstream", ctypes.c_float),
                ("student", ctypes.c_void_p), ("teacher", ctypes.c_void_p),
                ("gstudent", ctypes.c_void_p), ("out", ctypes.c_void_p)]

    @classmethod
    def from_torch(cls, n, channels, inner, student, teacher, out, gstudent=None, lam=1.0, eps=1e-8,
                   upstream=1.0):
        import torch
        if student.dtype not in (torch.float16, torch.float32):
            raise TypeError("student must be float16 or float32")
        for t in (teacher, gstudent):
            if t is not None and (t.dtype != student.dtype or not t.is_contiguous()):
                raise TypeError("teacher / gstudent must be contiguous and of the student's dtype")
        if out.dtype != torch.float64 or out.numel() < 3 or not out.is_contiguous() or not student.is_contiguous():
            raise TypeError("out must be 3 contiguous float64 values; student must be contiguous")
        self = cls(n, channels, inner, FQ_F16 if student.dtype == torch.float16 else FQ_F32, lam, eps,
                   upstream, student.data_ptr(), teacher.data_ptr(),
                   None if gstudent is None else gstudent.data_ptr(), out.data_ptr())
        self._keep = (student, teacher, gstudent, out)
        return self


class FqLayoutInfo(ctypes.Structure):
    """Mirror of `struct fq_layout_info`."""
    _fields_ = [("blocks", ctypes.c_int64), ("units_per_channel", ctypes.c_int64),
                ("unit_elems", ctypes.c_int64), ("wave_units", ctypes.c_int32), ("extra_slots", ctypes.c_int32)]


class FqError(RuntimeError):
    def __init__(self, status):
        self.status = int(status)
        super().__init__("libfq: %s (status %d)" % (fq_status_string(status), status))


_lib = _load()
_lib.fq_workspace_bytes.argtypes = [ctypes.POINTER(FqTensor), ctypes.c_int, ctypes.c_int]
_lib.fq_workspace_bytes.restype = ctypes.c_size_t
_lib.fq_validate.argtypes = [ctypes.POINTER(FqTensor), ctypes.c_int, ctypes.c_int]
_lib.fq_validate.restype = ctypes.c_int
_lib.fq_workspace_init.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fq_workspace_init.restype = ctypes.c_int
_lib.fq_forward.argtypes = [ctypes.POINTER(FqTensor), ctypes.c_void_p]
_lib.fq_forward.restype = ctypes.c_int
_lib.fq_backward.argtypes = [ctypes.POINTER(FqTensor), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fq_backward.restype = ctypes.c_int
_lib.fq_backward_static.argtypes = [ctypes.POINTER(FqTensor), ctypes.c_void_p]
_lib.fq_backward_static.restype = ctypes.c_int
_lib.fq_probe_stream.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                 ctypes.c_void_p]
_lib.fq_probe_stream.restype = ctypes.c_int
_lib.fq_multi_tensor.argtypes = [ctypes.POINTER(FqTensor), ctypes.c_int, ctypes.c_int,
                                 ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fq_multi_tensor.restype = ctypes.c_int
_lib.fq_plan_create.argtypes = [ctypes.POINTER(FqTensor), ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                ctypes.c_size_t, ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
_lib.fq_plan_create.restype = ctypes.c_int
_lib.fq_plan_run.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
_lib.fq_plan_run.restype = ctypes.c_int
_lib.fq_plan_run_adam.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
_lib.fq_plan_run_adam.restype = ctypes.c_int
_lib.fq_plan_destroy.argtypes = [ctypes.c_void_p]
_lib.fq_plan_destroy.restype = None
_lib.fq_distill_workspace_bytes.argtypes = [ctypes.POINTER(FqDistill)]
_lib.fq_distill_workspace_bytes.restype = ctypes.c_size_t
_lib.fq_distill_loss.argtypes = [ctypes.POINTER(FqDistill), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.fq_distill_loss.restype = ctypes.c_int
_lib.fq_distill_reads_of_pair.argtypes = [ctypes.POINTER(FqDistill)]
_lib.fq_distill_reads_of_pair.restype = ctypes.c_int
_lib.fq_layout.argtypes = [ctypes.POINTER(FqTensor), ctypes.POINTER(FqLayoutInfo)]
_lib.fq_layout.restype = ctypes.c_int
_lib.fq_status_string.argtypes = [ctypes.c_int]
_lib.fq_status_string.restype = ctypes.c_char_p


class FqTensorArray:
    """A host array of descriptors marshalled once (`fq_tensor_array`) and reused across calls."""

    def __init__(self, tensors):
        tensors = list(tensors)
        self.n = len(tensors)
        self.array = (FqTensor * max(1, self.n))(*tensors)


def fq_tensor_array(tensors) -> FqTensorArray:
    return FqTensorArray(tensors)


def _array(tensors):
    if isinstance(tensors, FqTensorArray):
        return tensors.array, tensors.n
    if isinstance(tensors, FqTensor):
        tensors = [tensors]
    a = FqTensorArray(tensors)
    return a.array, a.n


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ws(workspace):
    if workspace is None:
        return None, 0
    if isinstance(workspace, tuple):
        return workspace
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def _check(status):
    if status != 0:
        raise FqError(status)


def fq_status_string(status) -> str:
    return _lib.fq_status_string(int(status)).decode()


def fq_workspace_bytes(tensors, mode) -> int:
    arr, n = _array(tensors)
    return int(_lib.fq_workspace_bytes(arr, n, mode))


def fq_validate(tensors, mode) -> int:
    """Returns the fq_status (0 = ok) without raising."""
    arr, n = _array(tensors)
    return int(_lib.fq_validate(arr, n, mode))


def fq_workspace_init(workspace, stream=None):
    p, nbytes = _ws(workspace)
    _check(_lib.fq_workspace_init(p, nbytes, _stream(stream)))


def fq_forward(t: FqTensor, stream=None):
    _check(_lib.fq_forward(ctypes.byref(t), _stream(stream)))


def fq_backward(t: FqTensor, workspace, stream=None):
    p, nbytes = _ws(workspace)
    _check(_lib.fq_backward(ctypes.byref(t), p, nbytes, _stream(stream)))


def fq_backward_static(t: FqTensor, stream=None):
    _check(_lib.fq_backward_static(ctypes.byref(t), _stream(stream)))


def fq_multi_tensor(tensors, mode, workspace, stream=None):
    arr, n = _array(tensors)
    p, nbytes = _ws(workspace)
    _check(_lib.fq_multi_tensor(arr, n, mode, p, nbytes, _stream(stream)))


def fq_plan_create(tensors, mode, workspace, stream=None):
    """Returns an opaque plan handle (ctypes.c_void_p); release it with fq_plan_destroy."""
    arr, n = _array(tensors)
    p, nbytes = _ws(workspace)
    plan = ctypes.c_void_p()
    _check(_lib.fq_plan_create(arr, n, mode, p, nbytes, _stream(stream), ctypes.byref(plan)))
    return plan


def fq_plan_run(plan, stream=None):
    _check(_lib.fq_plan_run(plan, _stream(stream)))


def fq_plan_run_adam(plan, step, stream=None):
    _check(_lib.fq_plan_run_adam(plan, int(step), _stream(stream)))


def fq_plan_destroy(plan):
    _lib.fq_plan_destroy(plan)


def fq_distill_workspace_bytes(d: FqDistill) -> int:
    return int(_lib.fq_distill_workspace_bytes(ctypes.byref(d)))


def fq_distill_reads_of_pair(d: FqDistill) -> int:
    return int(_lib.fq_distill_reads_of_pair(ctypes.byref(d)))


def fq_distill_loss(d: FqDistill, workspace, stream=None):
    p, nbytes = _ws(workspace)
    _check(_lib.fq_distill_loss(ctypes.byref(d), p, nbytes, _stream(stream)))


def fq_probe_stream(inputs, a, b, out, nbytes, stream=None):
    """a, b, out: torch tensors (or None where unused); see include/fq.h."""
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(_lib.fq_probe_stream(int(inputs), ptr(a), ptr(b), ptr(out), int(nbytes), _stream(stream)))


def fq_probe_stream_raw(inputs, a_ptr, b_ptr, out_ptr, nbytes, stream_ptr):
    """The same with raw device addresses and a raw stream handle (0 = none / default stream)."""
    _check(_lib.fq_probe_stream(inputs, a_ptr or None, b_ptr or None, out_ptr or None, nbytes, stream_ptr or None))


def fq_layout(t: FqTensor) -> FqLayoutInfo:
    info = FqLayoutInfo()
    _check(_lib.fq_layout(ctypes.byref(t), ctypes.byref(info)))
    return info
