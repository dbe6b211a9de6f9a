"""torch.autograd front door to the library: `fake_quantize(x, theta, ...)`.

Marshalling only: the forward is one fq_forward call, the backward one fq_backward call (STE for
x, per-channel reduction for theta; Sec. 3.2, Eq. (3)-(6)).  Nothing is saved by the forward but
references to x and theta; the backward re-reads x and recomputes the quotient.  PyTorch owns the
memory (outputs and the small backward workspace come from its caching allocator) and the stream
(kernels are enqueued on the current one).  There is no CPU path: CPU tensors raise.
"""
import torch

from . import binding as fq


def _view(x, channel_dim):
    """(outer, channels, inner) of the contiguous tensor x for scales along channel_dim."""
    if channel_dim is None:
        return 1, 1, x.numel()
    d = channel_dim % x.dim()
    outer = 1
    for n in x.shape[:d]:
        outer *= n
    inner = 1
    for n in x.shape[d + 1:]:
        inner *= n
    return outer, x.shape[d], inner


class _FakeQuantize(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, theta, qmin, qmax, channel_dim, eps, s_min, s_max):
        if not x.is_cuda or not theta.is_cuda:
            raise RuntimeError("fake_quantize runs on the GPU only (no CPU fallback)")
        x = x.contiguous()
        th = theta.detach().contiguous().view(-1)
        outer, channels, inner = _view(x, channel_dim)
        if th.numel() != channels or th.dtype != torch.float32:
            raise ValueError("theta must hold %d float32 values" % channels)
        y = torch.empty_like(x)
        t = fq.FqTensor.from_torch(outer, channels, inner, qmin, qmax, x=x.detach(), y=y, theta=th, eps=eps,
                                   s_min=s_min, s_max=s_max)
        fq.fq_forward(t)
        ctx.save_for_backward(x, theta)
        ctx.meta = (outer, channels, inner, qmin, qmax, eps, s_min, s_max)
        return y

    @staticmethod
    def backward(ctx, gy):
        x, theta = ctx.saved_tensors
        outer, channels, inner, qmin, qmax, eps, s_min, s_max = ctx.meta
        want_gx, want_gtheta = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        if not (want_gx or want_gtheta):
            return (None,) * 8
        gy = gy.contiguous()
        th = theta.detach().contiguous().view(-1)
        gx = torch.empty_like(x) if want_gx else None
        gtheta = torch.empty_like(th)
        t = fq.FqTensor.from_torch(outer, channels, inner, qmin, qmax, x=x.detach(), theta=th, gy=gy, gx=gx,
                                   gtheta=gtheta, eps=eps, s_min=s_min, s_max=s_max,
                                   flags=0 if want_gx else fq.FQ_FLAG_NO_DX)
        # the workspace must start zeroed; a fresh one per call keeps concurrent streams apart
        ws = torch.zeros(fq.fq_workspace_bytes(t, fq.FQ_MODE_BACKWARD) // 4, dtype=torch.int32, device=x.device)
        fq.fq_backward(t, ws)
        return gx, (gtheta.view_as(theta) if want_gtheta else None), None, None, None, None, None, None


def fake_quantize(x, theta, qmin=-127, qmax=127, channel_dim=None, eps=0.0, s_min=fq.FLT_MIN,
                  s_max=float("inf")):
    """y = s * round(clip(x / s, qmin, qmax)), s = clip(softplus(theta) + eps, s_min, s_max).

    x: float16 or float32 CUDA tensor.  theta: float32 CUDA tensor with one value per channel of
    `channel_dim` (None: one value for the whole tensor).  Differentiable with respect to x
    (straight-through) and theta; a frozen x (requires_grad False) skips its gradient entirely.
    """
    return _FakeQuantize.apply(x, theta, int(qmin), int(qmax), channel_dim, float(eps), float(s_min),
                               float(s_max))
