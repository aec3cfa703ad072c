"""Shared test plumbing: device tensors from the seeded generator, plans, and oracle comparison.

The HIP path is reached only through the binding (C ABI); the oracle only through oracle.oracle.
Layout conversion (logical NCHW/KCRS <-> physical NHWC/KRSC) is done here with plain permutes.
"""
from __future__ import annotations

import numpy as np

from oracle import oracle
from paper_1901_00041_amd import st_conv as sc
from paper_1901_00041_amd import synth

_TORCH_DT = None


def torch_dtype(name):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[name]


def to_device_nhwc(a_nchw: np.ndarray, dtype: str):
    """float32 NCHW (or KCRS) values, exactly representable in `dtype` -> device tensor, channel-last."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a_nchw.transpose(0, 2, 3, 1)))
    return t.to(torch_dtype(dtype)).cuda().contiguous()


def from_device_nhwc(t) -> np.ndarray:
    """device NHWC tensor of any dtype -> float64 NCHW numpy."""
    import torch
    return t.detach().to(torch.float64).cpu().numpy().transpose(0, 3, 1, 2)


class Tenant:
    """One tenant's tensors on the host (logical layout) and on the device (physical layout)."""

    def __init__(self, shape: synth.ConvShape, x: np.ndarray, w: np.ndarray, residual: np.ndarray | None = None,
                 relu: bool = False):
        import torch
        self.shape, self.x, self.w, self.residual, self.relu = shape, x, w, residual, relu
        self.dx = to_device_nhwc(x, shape.dtype)
        self.dw = to_device_nhwc(w, shape.dtype)
        self.dres = to_device_nhwc(residual, shape.out_dtype) if residual is not None else None
        self.dy = torch.full((shape.N, shape.P, shape.Q, shape.K), float("nan"), dtype=torch_dtype(shape.out_dtype),
                             device="cuda")

    def desc(self):
        s = self.shape
        epi = (sc.ST_EPI_RELU if self.relu else 0) | (sc.ST_EPI_RESIDUAL if self.dres is not None else 0)
        return sc.make_desc(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.dtype, s.out_dtype,
                            self.dx, self.dw, self.dy, self.dres, epi)

    def reference(self) -> np.ndarray:
        s = self.shape
        return oracle.conv_layer(self.x, self.w, s.stride, s.pad, self.residual, self.relu)

    def result(self) -> np.ndarray:
        return from_device_nhwc(self.dy)

    def clear(self):
        self.dy.fill_(float("nan"))


def make_tenants(cfg: int, shapes=None, gain: float = 1.0):
    shapes = shapes if shapes is not None else synth.config_shapes(cfg)
    return [Tenant(s, synth.gen_input(cfg, t, 0, s), synth.gen_weight(cfg, t, 0, s, gain)) for t, s in enumerate(shapes)]


def plan_for(tenants, **opts):
    return sc.st_conv_plan([t.desc() for t in tenants], sc.plan_opts(**opts) if opts else None, keep=list(tenants))


def tolerance(shape: synth.ConvShape, ref: np.ndarray) -> np.ndarray:
    """Element-wise bound.  fp32 path: 1e-4 absolute.  16-bit inputs with fp32 outputs: products are exact
    in fp32, so only the fp32 accumulation order differs: 1e-4*(|ref|+1), far inside the required
    1e-2*(|ref|+1).  16-bit outputs add one rounding of the result (2^-9 relative): 1e-2*(|ref|+1)."""
    if shape.dtype == "f32":
        return np.full_like(ref, 1e-4)
    if shape.out_dtype == "f32":
        return 1e-4 * (np.abs(ref) + 1.0)
    return 1e-2 * (np.abs(ref) + 1.0)


def check_tenant(t: Tenant, what: str = ""):
    ref, got = t.reference(), t.result()
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: output holds NaN/Inf (unwritten or wrong)"
    err = np.abs(got - ref)
    tol = tolerance(t.shape, ref)
    bad = err > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} outside tolerance, max err {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"
    return float(err.max())
