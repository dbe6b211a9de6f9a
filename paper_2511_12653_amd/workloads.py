"""Seeded synthetic inputs shaped like the tensors of a DPVO front end.

This module only *generates inputs* (tensor values, upstream gradients and the
learnable scale parameters theta).  It contains none of the quantizer's
arithmetic and imports neither the GPU binding nor the CPU oracle, so both can
be fed the very same bytes.

The tensors stand in for the feature maps and 3x3 convolution weights of the
DPVO patchifier evaluated on EuRoC / TartanAir frames (Sec. 4.1.1, 4.1.5 of the
DPVO-QAT++ paper: features at 1/4 image scale, 22 quantized Conv2d layers);
neither the datasets nor trained weights are used.

Every tensor is described as a contiguous [outer, channels, inner] view:
  per-channel NCHW activation -> outer=N, channels=C, inner=H*W
  per-output-channel weight   -> outer=1, channels=C_out, inner=C_in*kh*kw
  per-tensor                  -> outer=1, channels=1, inner=numel
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 251112653 * 10
FLT_MIN = float(np.finfo(np.float32).tiny)

WORKLOAD_NAMES = (
    "act_fp32_per_tensor",        # FP32 1x128x30x40, one learnable scale, fwd+bwd
    "feature_fp16_per_channel",   # FP16 1x384x120x160, 384 scales (headline tensor)
    "conv_weights_fp32",          # FP32 384x384x3x3 and 128x128x3x3, per output channel
    "train_batch_fp16",           # FP16 15x128x120x160, 128 scales, fwd+bwd
    "multi_tensor_mixed",         # 64 mixed tensors, about 1 GiB of inputs, one launch
)


@dataclass
class TensorCase:
    name: str
    shape: Tuple[int, ...]
    outer: int
    channels: int
    inner: int
    qmin: int
    qmax: int
    x: np.ndarray                      # float16 or float32, C-contiguous, `shape`
    theta: np.ndarray                  # float32 [channels]
    gy: Optional[np.ndarray] = None    # same dtype/shape as x (None: forward only)
    eps: float = 0.0
    s_min: float = FLT_MIN
    s_max: float = float("inf")
    flags: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def numel(self) -> int:
        return self.outer * self.channels * self.inner

    @property
    def itemsize(self) -> int:
        return self.x.dtype.itemsize


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def theta_for_scale(s) -> np.ndarray:
    """The parameter value whose softplus is `s` (evaluated in float64, stored as float32)."""
    s = np.asarray(s, dtype=np.float64)
    return np.log(np.expm1(s)).astype(np.float32)


def _normal(rng, shape, dtype, chunk=1 << 24):
    """Standard normal of `shape`, generated in float32 blocks to bound host memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=dtype)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        out[a:b] = rng.standard_normal(b - a, dtype=np.float32)
    return out.reshape(shape)


def _per_channel_activation(rng, n, c, h, w, dtype):
    """Channel c ~ N(mu_c, sigma_c), mu_c ~ U(-1,1), sigma_c ~ U(0.2,3)."""
    mu = rng.uniform(-1.0, 1.0, size=c).astype(np.float32)
    sigma = rng.uniform(0.2, 3.0, size=c).astype(np.float32)
    x = np.empty((n, c, h * w), dtype=dtype)
    for i in range(n):
        z = rng.standard_normal((c, h * w), dtype=np.float32)
        x[i] = z * sigma[:, None] + mu[:, None]
    return x.reshape(n, c, h, w), mu, sigma


def _absmax_scale(x3, qmax):
    """max|x| over each channel of an [outer, C, inner] view, divided by qmax (float64)."""
    m = np.abs(x3.astype(np.float32)).max(axis=(0, 2)).astype(np.float64)
    m = np.maximum(m, 1e-6)
    return m / float(qmax)


def act_fp32_per_tensor(seed=BASE_SEED + 1, shape=(1, 128, 30, 40)) -> List[TensorCase]:
    rng = _rng(seed)
    x = _normal(rng, shape, np.float32)
    flat = x.reshape(-1)
    n_out = max(1, flat.size // 100)
    idx = rng.choice(flat.size, size=n_out, replace=False)
    flat[idx] *= 10.0
    gy = _normal(rng, shape, np.float32)
    theta = np.array([0.5], dtype=np.float32)
    return [TensorCase("act", tuple(shape), 1, 1, flat.size, -128, 127, x, theta, gy)]


def feature_fp16_per_channel(seed=BASE_SEED + 2, shape=(1, 384, 120, 160),
                             with_grad=True) -> List[TensorCase]:
    rng = _rng(seed)
    n, c, h, w = shape
    x, _, _ = _per_channel_activation(rng, n, c, h, w, np.float16)
    theta = theta_for_scale(_absmax_scale(x.reshape(n, c, h * w), 127))
    gy = _normal(rng, shape, np.float16) if with_grad else None
    return [TensorCase("feature", tuple(shape), n, c, h * w, -128, 127, x, theta, gy)]


def conv_weights_fp32(seed=BASE_SEED + 3, shapes=((384, 384, 3, 3), (128, 128, 3, 3))
                      ) -> List[TensorCase]:
    cases = []
    for k, shp in enumerate(shapes):
        rng = _rng(seed + 100 * k)
        co, ci, kh, kw = shp
        fan_in = ci * kh * kw
        wgt = _normal(rng, shp, np.float32) * np.float32(np.sqrt(2.0 / fan_in))
        theta = theta_for_scale(_absmax_scale(wgt.reshape(1, co, fan_in), 127))
        gy = _normal(rng, shp, np.float32) * np.float32(0.1)   # variance 1e-2
        cases.append(TensorCase("w%dx%d" % (co, ci), tuple(shp), 1, co, fan_in, -127, 127,
                                wgt, theta, gy))
    return cases


def train_batch_fp16(seed=BASE_SEED + 4, shape=(15, 128, 120, 160)) -> List[TensorCase]:
    rng = _rng(seed)
    n, c, h, w = shape
    x, mu, sigma = _per_channel_activation(rng, n, c, h, w, np.float16)
    # about 0.3 % of each channel falls outside the code range, so all three
    # branches of the scale gradient occur
    s = (np.abs(mu).astype(np.float64) + 3.0 * sigma.astype(np.float64)) / 127.0
    theta = theta_for_scale(s)
    gy = _normal(rng, shape, np.float16)
    return [TensorCase("batch", tuple(shape), n, c, h * w, -128, 127, x, theta, gy)]


def multi_tensor_mixed(seed=BASE_SEED + 5, n_act=48, n_wgt=16, target_bytes=1 << 30,
                       max_batch=8) -> List[TensorCase]:
    """64 tensors for one multi-tensor launch: mixed FP16/FP32, 4/8 bit, per-tensor/per-channel.

    The batch sizes of the activations are adjusted (in a seeded order) until the sum of
    the x bytes is within 5 % of `target_bytes`.
    """
    rng = _rng(seed)
    chans = (64, 128, 384)
    specs = []
    for t in range(n_act):
        specs.append(dict(kind="act", c=int(rng.choice(chans)), h=int(rng.integers(30, 121)),
                          w=int(rng.integers(40, 161)), n=int(rng.integers(1, max_batch + 1)),
                          f16=bool(rng.integers(0, 2)), bits=int(rng.choice((4, 8))),
                          per_channel=bool(rng.integers(0, 2))))
    for t in range(n_wgt):
        specs.append(dict(kind="wgt", co=int(rng.choice(chans)), ci=int(rng.choice(chans)),
                          f16=bool(rng.integers(0, 2)), bits=int(rng.choice((4, 8))),
                          per_channel=bool(rng.integers(0, 2))))

    def nbytes(sp):
        b = 2 if sp["f16"] else 4
        if sp["kind"] == "act":
            return sp["n"] * sp["c"] * sp["h"] * sp["w"] * b
        return sp["co"] * sp["ci"] * 9 * b

    order = rng.permutation(n_act)
    for _ in range(64):
        total = sum(nbytes(sp) for sp in specs)
        if abs(total - target_bytes) <= 0.05 * target_bytes:
            break
        changed = False
        for j in order:
            sp = specs[int(j)]
            total = sum(nbytes(s_) for s_ in specs)
            if total < 0.95 * target_bytes and sp["n"] < max_batch:
                sp["n"] += 1
                changed = True
            elif total > 1.05 * target_bytes and sp["n"] > 1:
                sp["n"] -= 1
                changed = True
        if not changed:
            break

    cases = []
    for t, sp in enumerate(specs):
        trng = _rng(seed + 1000 + t)
        dtype = np.float16 if sp["f16"] else np.float32
        qmin, qmax = (-8, 7) if sp["bits"] == 4 else (-128, 127)
        if sp["kind"] == "act":
            shp = (sp["n"], sp["c"], sp["h"], sp["w"])
            x, _, _ = _per_channel_activation(trng, *shp, dtype)
            gy = _normal(trng, shp, dtype)
            if sp["per_channel"]:
                outer, c, inner = sp["n"], sp["c"], sp["h"] * sp["w"]
            else:
                outer, c, inner = 1, 1, x.size
        else:
            shp = (sp["co"], sp["ci"], 3, 3)
            fan_in = sp["ci"] * 9
            x = (_normal(trng, shp, np.float32) * np.float32(np.sqrt(2.0 / fan_in))).astype(dtype)
            gy = (_normal(trng, shp, np.float32) * np.float32(0.1)).astype(dtype)
            if sp["per_channel"]:
                outer, c, inner = 1, sp["co"], fan_in
            else:
                outer, c, inner = 1, 1, x.size
        theta = theta_for_scale(_absmax_scale(x.reshape(outer, c, inner), qmax))
        cases.append(TensorCase("%s%02d" % (sp["kind"], t), shp, outer, c, inner, qmin, qmax,
                                x, theta, gy, meta=dict(sp)))
    return cases


def make(name: str, **kw) -> List[TensorCase]:
    """Build the named workload (one of WORKLOAD_NAMES); keyword arguments override shapes/seeds."""
    if name not in WORKLOAD_NAMES:
        raise KeyError(name)
    return globals()[name](**kw)
