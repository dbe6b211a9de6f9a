"""ctypes front end of the CPU oracle (oracle/fq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
CPU-baseline leg of the benchmark.  It takes and returns numpy arrays; FP16
tensors are numpy float16 arrays (passed to C as their 16-bit patterns).

Operations follow DPVO-QAT++ Sec. 3.2: scale Eq. (3)-(4), fake quantization
Eq. (5)-(6), straight-through-estimator backward.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

_DT = {np.dtype(np.float16): 0, np.dtype(np.float32): 1}


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = ctypes.CDLL(path)
        i64, i32, f32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p
        L.fqo_half_to_float.argtypes = [ctypes.c_uint16]
        L.fqo_half_to_float.restype = f32
        L.fqo_float_to_half.argtypes = [f32]
        L.fqo_float_to_half.restype = ctypes.c_uint16
        L.fqo_scale.argtypes = [vp, i64, f32, f32, f32, vp, vp]
        L.fqo_scale.restype = None
        L.fqo_forward.argtypes = [vp, ctypes.c_int, i64, i64, i64, vp, i32, i32, vp, vp]
        L.fqo_forward.restype = None
        L.fqo_backward.argtypes = [vp, vp, ctypes.c_int, i64, i64, i64, vp, vp, vp, i32, i32,
                                   vp, vp, vp, vp, vp]
        L.fqo_backward.restype = None
        L.fqo_distill.argtypes = [vp, vp, ctypes.c_int, i64, i64, i64, ctypes.c_double, ctypes.c_double,
                                  ctypes.c_double, vp, vp]
        L.fqo_distill.restype = None
        L.fqo_adam.argtypes = [vp, i64, f32, f32, f32, f32, f32, f32, f32, f32, vp, vp, vp, vp]
        L.fqo_adam.restype = None
        L.fqo_set_threads.argtypes = [ctypes.c_int]
        L.fqo_set_threads.restype = None
        L.fqo_get_threads.argtypes = []
        L.fqo_get_threads.restype = ctypes.c_int
        _LIB = L
    return _LIB


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def half_to_float(bits: int) -> float:
    return float(lib().fqo_half_to_float(int(bits)))


def float_to_half(value) -> int:
    return int(lib().fqo_float_to_half(float(np.float32(value))))


FLT_MIN = float(np.finfo(np.float32).tiny)


def set_threads(n: int) -> int:
    """Threads for forward / backward (channels are split over them; results do not change).
    Returns the count now in force."""
    lib().fqo_set_threads(int(n))
    return int(lib().fqo_get_threads())


def scale(theta, eps=0.0, s_min=FLT_MIN, s_max=float("inf")):
    """Eq. (3)-(4).  theta float32 [C] -> (s float32 [C], clip_active uint8 [C])."""
    theta = np.ascontiguousarray(theta, dtype=np.float32).reshape(-1)
    s = np.empty_like(theta)
    active = np.empty(theta.shape, dtype=np.uint8)
    lib().fqo_scale(_p(theta), theta.size, eps, s_min, s_max, _p(s), _p(active))
    return s, active


def _view3(x, outer, channels, inner):
    x = np.ascontiguousarray(x)
    if x.dtype not in _DT:
        raise TypeError("oracle tensors are float16 or float32")
    if x.size != outer * channels * inner:
        raise ValueError("shape mismatch")
    return x


def forward(x, s, qmin, qmax, outer, channels, inner, want_q=True):
    """Eq. (5).  x: float16/float32, viewed as [outer, channels, inner]; s float32 [channels].
    Returns (y same dtype/shape as x, q int32 or None)."""
    x = _view3(x, outer, channels, inner)
    s = np.ascontiguousarray(s, dtype=np.float32).reshape(-1)
    assert s.size == channels
    y = np.empty_like(x)
    q = np.empty(x.shape, dtype=np.int32) if want_q else None
    lib().fqo_forward(_p(x), _DT[x.dtype], outer, channels, inner, _p(s), qmin, qmax, _p(y), _p(q))
    return y, q


def backward(x, gy, s, theta, clip_active, qmin, qmax, outer, channels, inner, want_gx=True):
    """STE backward.  Returns dict(gx, gs, gtheta, acc (float64), aabs (float64))."""
    x = _view3(x, outer, channels, inner)
    gy = _view3(gy, outer, channels, inner)
    assert gy.dtype == x.dtype
    s = np.ascontiguousarray(s, dtype=np.float32).reshape(-1)
    theta = np.ascontiguousarray(theta, dtype=np.float32).reshape(-1)
    clip_active = np.ascontiguousarray(clip_active, dtype=np.uint8).reshape(-1)
    assert s.size == channels and theta.size == channels and clip_active.size == channels
    gx = np.empty_like(x) if want_gx else None
    acc = np.empty(channels, dtype=np.float64)
    aabs = np.empty(channels, dtype=np.float64)
    gs = np.empty(channels, dtype=np.float32)
    gtheta = np.empty(channels, dtype=np.float32)
    lib().fqo_backward(_p(x), _p(gy), _DT[x.dtype], outer, channels, inner, _p(s), _p(theta),
                       _p(clip_active), qmin, qmax, _p(gx), _p(acc), _p(aabs), _p(gs), _p(gtheta))
    return dict(gx=gx, gs=gs, gtheta=gtheta, acc=acc, aabs=aabs)


def adam_constants(lr, beta1, beta2, eps, step):
    """The eight float32 constants of one Adam step, each evaluated in float64 and rounded once:
    lr, beta1, 1-beta1, beta2, 1-beta2, eps, 1-beta1^t, 1-beta2^t."""
    f = lambda x: float(np.float32(x))
    return (f(lr), f(beta1), f(1.0 - beta1), f(beta2), f(1.0 - beta2), f(eps),
            f(1.0 - beta1 ** step), f(1.0 - beta2 ** step))


def adam(g, m, v, theta, lr, beta1, beta2, eps, step):
    """One Adam step (Kingma & Ba Alg. 1, float32).  Returns (theta_new, m_new, v_new)."""
    g = np.ascontiguousarray(g, dtype=np.float32).reshape(-1)
    m = np.array(m, dtype=np.float32).reshape(-1).copy()
    v = np.array(v, dtype=np.float32).reshape(-1).copy()
    theta = np.ascontiguousarray(theta, dtype=np.float32).reshape(-1)
    out = np.empty_like(theta)
    lr_, b1, omb1, b2, omb2, eps_, bc1, bc2 = adam_constants(lr, beta1, beta2, eps, step)
    lib().fqo_adam(_p(g), g.size, lr_, b1, omb1, b2, omb2, eps_, bc1, bc2, _p(m), _p(v), _p(theta), _p(out))
    return out, m, v


def distill(a, b, lam, eps=1e-8, upstream=1.0, want_grad=True):
    """Eq. (7) for one (student, teacher) pair [N, C, M].  Returns (mse, cosim, loss, ga or None)."""
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    assert a.shape == b.shape and a.ndim == 3 and a.dtype == b.dtype and a.dtype in _DT
    n, c, m = a.shape
    ga = np.empty_like(a) if want_grad else None
    out = np.empty(3, dtype=np.float64)
    lib().fqo_distill(_p(a), _p(b), _DT[a.dtype], n, c, m, lam, eps, upstream, _p(ga), _p(out))
    return float(out[0]), float(out[1]), float(out[2]), ga
