"""Seeded synthetic workloads: shapes and tensor values for the five benchmark configurations.

This module is the one piece shared by the CPU oracle's tests and the HIP path's tests/bench. It
holds no convolution arithmetic: only a counter-based random generator (splitmix64), the shape
recipes, and the cast of generated values to their storage type.  It imports numpy only.

The paper's own workload is synthetic as well (random matrices with the shape of a ResNet-18 layer,
Section 4.1; tenants share an architecture and differ in weights and inputs, Section 2), so the
recipes below stand in for nothing external.

Logical tensor layouts produced here: activations NCHW, weights KCRS, float32 values that are exactly
representable in the requested storage type.  Callers permute to whatever physical layout they need.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np

BASE_SEED = 190100041
_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK = (1 << 64) - 1

WHAT_SHAPE, WHAT_INPUT, WHAT_WEIGHT = 0, 1, 2


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def splitmix64(state: int, count: int, offset: int = 0) -> np.ndarray:
    """Outputs offset .. offset+count-1 (0-based) of splitmix64 started from `state`.

    Output i is mix(state + (i+1)*GAMMA) mod 2^64, so any slice can be produced directly.
    """
    with np.errstate(over="ignore"):
        idx = np.arange(offset + 1, offset + count + 1, dtype=np.uint64)
        return _mix(np.uint64(state & _MASK) + idx * _GAMMA)


def stream_state(cfg: int, tenant: int, layer: int, what: int) -> int:
    """Start state of the stream for (cfg, tenant, layer, what): the first splitmix64 output of the
    key BASE ^ cfg<<48 ^ tenant<<32 ^ layer<<8 ^ what."""
    key = BASE_SEED ^ (cfg << 48) ^ (tenant << 32) ^ (layer << 8) ^ what
    return int(splitmix64(key, 1)[0])


def uniform01(state: int, count: int, offset: int = 0) -> np.ndarray:
    """float64 in [0,1): top 53 bits of each output."""
    return (splitmix64(state, count, offset) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def uniform_pm1(state: int, count: int) -> np.ndarray:
    return 2.0 * uniform01(state, count) - 1.0


def normal(state: int, count: int, sigma: float) -> np.ndarray:
    """Box-Muller on consecutive pairs (u1,u2): sigma*sqrt(-2 ln(1-u1))*cos(2 pi u2), float64."""
    u = uniform01(state, 2 * count)
    u1, u2 = u[0::2], u[1::2]
    return sigma * np.sqrt(-2.0 * np.log1p(-u1)) * np.cos(2.0 * np.pi * u2)


# ---------------------------------------------------------------------------------------------
# storage types
# ---------------------------------------------------------------------------------------------
F32, BF16, F16 = "f32", "bf16", "f16"


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest, ties to even. Finite inputs."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a64: np.ndarray, dtype: str) -> np.ndarray:
    """float64 draws -> float32 -> storage type, returned as float32 holding the stored values."""
    a = a64.astype(np.float32)
    if dtype == F32:
        return a
    if dtype == BF16:
        return bf16_bits_to_f32(f32_to_bf16_bits(a)).reshape(a.shape)
    if dtype == F16:
        return a.astype(np.float16).astype(np.float32)
    raise ValueError(dtype)


# ---------------------------------------------------------------------------------------------
# shapes
# ---------------------------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class ConvShape:
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    dtype: str = BF16       # storage type of x and w
    out_dtype: str = F32    # storage type of y

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def gemm(self):
        """(M, Ngemm, Kgemm) of the im2col product (Section 4.1's worked example fixes the reading)."""
        return (self.N * self.P * self.Q, self.K, self.C * self.R * self.S)

    @property
    def flops(self) -> int:
        m, n, k = self.gemm
        return 2 * m * n * k

    @property
    def bytes(self) -> int:
        """x + w + y, each element once, in storage types."""
        es = {F32: 4, BF16: 2, F16: 2}
        m, n, k = self.gemm
        return (self.N * self.C * self.H * self.W + self.K * self.C * self.R * self.S) * es[self.dtype] \
            + m * n * es[self.out_dtype]


def config_shapes(cfg: int) -> List[ConvShape]:
    """Per-tenant conv problems of configurations 1-4 (configuration 5 is `resnet50_steps`)."""
    if cfg == 1:
        return [ConvShape(1, 32, 28, 28, 32, 3, 3, 1, 1, F32, F32) for _ in range(2)]
    if cfg == 2:
        return [ConvShape(1, c, h, h, c, 3, 3, 1, 1) for c, h in ((64, 56), (128, 28), (256, 14), (512, 7))]
    if cfg == 3:
        out = []
        for t in range(8):
            u = splitmix64(stream_state(3, t, 0, WHAT_SHAPE), 1)
            out.append(ConvShape((1, 2, 4)[int(u[0] % np.uint64(3))], 256, 14, 14, 256, 3, 3, 1, 1))
        return out
    if cfg == 4:
        out = []
        for t in range(16):
            u = [int(v) for v in splitmix64(stream_state(4, t, 0, WHAT_SHAPE), 4)]
            b = 1 + u[0] % 8
            if t % 8 == 7:
                out.append(ConvShape(b, 3, 224, 224, 64, 7, 7, 2, 3))
            elif t % 2 == 0:
                ch = (64, 128, 256, 512, 1024)
                c, k, h = ch[u[1] % 5], ch[u[2] % 5], (7, 14, 28, 56)[u[3] % 4]
                out.append(ConvShape(b, c, h, h, k, 1, 1, 1, 0))
            else:
                c, h = (64, 128, 256, 512)[u[1] % 4], (7, 14, 28, 56)[u[2] % 4]
                out.append(ConvShape(b, c, h, h, c, 3, 3, 1, 1))
        return out
    raise ValueError(f"config_shapes: cfg must be 1..4, got {cfg}")


N_TENANTS = {1: 2, 2: 4, 3: 8, 4: 16, 5: 8}


@dataclasses.dataclass(frozen=True)
class Step:
    """One conv step of the ResNet-50-shaped stack (same for every tenant).

    Buffers are named by small integers; `src` feeds the conv, `dst` receives it, `res` (or None) is
    added to the fp32 accumulator before ReLU.  `pool_after`: a 3x3/stride-2/pad-1 max-pool of `dst`
    into buffer `pool_dst` follows the step.
    """
    index: int
    name: str
    shape: ConvShape
    src: int
    dst: int
    res: Optional[int]
    relu: bool
    pool_after: bool = False
    pool_dst: Optional[int] = None


def resnet50_steps(batch: int = 1, image: int = 224) -> List[Step]:
    """53 conv steps: stem, then per bottleneck [projection], 1x1, 3x3 (carries the stride), 1x1.

    No batch-norm.  Data flow: a=ReLU(conv1(x)); b=ReLU(conv2(a)); c=conv3(b); shortcut = x or
    proj(x) (no ReLU); out = ReLU(c + shortcut).  Buffer ids: 0 network input, 1 stem output,
    7 pooled stem output (input of the first block), 2/3 alternate as block output/input afterwards,
    4 = a, 5 = b, 6 = projection output.
    """
    steps: List[Step] = []
    h = image
    stem = ConvShape(batch, 3, h, h, 64, 7, 7, 2, 3, BF16, BF16)
    steps.append(Step(0, "stem", stem, 0, 1, None, True, True, 7))
    h = stem.P
    h = (h + 2 - 3) // 2 + 1
    cur, nxt = 7, 2
    c_in = 64
    for stage, (width, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3))):
        for b in range(blocks):
            stride = 2 if (b == 0 and stage > 0) else 1
            c_out = 4 * width
            tag = f"s{stage + 2}b{b}"
            res = cur
            if b == 0:
                proj = ConvShape(batch, c_in, h, h, c_out, 1, 1, stride, 0, BF16, BF16)
                steps.append(Step(len(steps), tag + ".proj", proj, cur, 6, None, False))
                res = 6
            s1 = ConvShape(batch, c_in, h, h, width, 1, 1, 1, 0, BF16, BF16)
            steps.append(Step(len(steps), tag + ".conv1", s1, cur, 4, None, True))
            s2 = ConvShape(batch, width, h, h, width, 3, 3, stride, 1, BF16, BF16)
            steps.append(Step(len(steps), tag + ".conv2", s2, 4, 5, None, True))
            h2 = s2.P
            s3 = ConvShape(batch, width, h2, h2, c_out, 1, 1, 1, 0, BF16, BF16)
            steps.append(Step(len(steps), tag + ".conv3", s3, 5, nxt, res, True))
            cur, nxt = nxt, (3 if nxt == 2 else 2)
            c_in, h = c_out, h2
    return steps


# ---------------------------------------------------------------------------------------------
# tensor values
# ---------------------------------------------------------------------------------------------
def gen_input(cfg: int, tenant: int, layer: int, shape: ConvShape) -> np.ndarray:
    """x ~ U(-1,1), logical NCHW float32, already rounded to shape.dtype."""
    n = shape.N * shape.C * shape.H * shape.W
    v = uniform_pm1(stream_state(cfg, tenant, layer, WHAT_INPUT), n)
    return to_storage(v, shape.dtype).reshape(shape.N, shape.C, shape.H, shape.W)


def gen_weight(cfg: int, tenant: int, layer: int, shape: ConvShape, gain: float = 1.0) -> np.ndarray:
    """w ~ N(0, gain/fan_in), logical KCRS float32, already rounded to shape.dtype."""
    fan_in = shape.C * shape.R * shape.S
    n = shape.K * fan_in
    v = normal(stream_state(cfg, tenant, layer, WHAT_WEIGHT), n, float(np.sqrt(gain / fan_in)))
    return to_storage(v, shape.dtype).reshape(shape.K, shape.C, shape.R, shape.S)
