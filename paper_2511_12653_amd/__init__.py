"""Fused learnable-scale fake quantization for MI355X (gfx950).

`workloads` generates seeded synthetic inputs (numpy only).  The GPU entry points live in
`binding` (thin ctypes marshalling onto the C-ABI library built from csrc/); it is imported
on first use and raises if the compiled library is missing -- there is no CPU fallback.
`fake_quantize` (module `autograd`) wraps the forward and backward calls in a torch.autograd Function.
"""
from . import workloads  # noqa: F401

_API = ("fq_forward", "fq_backward", "fq_multi_tensor", "fq_workspace_bytes", "fq_workspace_init",
        "fq_validate", "fq_status_string", "fq_plan_create", "fq_plan_run", "fq_plan_run_adam", "fq_plan_destroy",
        "fq_layout", "FqLayoutInfo", "fq_distill_loss", "fq_distill_workspace_bytes", "FqDistill", "FqTensor", "FqAdam", "FqTensorArray", "fq_tensor_array", "FqError", "library_path",
        "FQ_F16", "FQ_F32", "FQ_FLAG_NO_DX", "FQ_FLAG_TWO_PASS", "FQ_MODE_FORWARD", "FQ_MODE_BACKWARD")


def __getattr__(name):
    if name == "fake_quantize":
        from .autograd import fake_quantize
        return fake_quantize
    if name == "binding" or name in _API:
        import importlib
        mod = importlib.import_module(__name__ + ".binding")
        return mod if name == "binding" else getattr(mod, name)
    raise AttributeError(name)
