"""Seeded synthetic conv-layer workloads shared by the tests, the smoke check and the bench.

This module only *names* layer shapes and *draws* input tensors.  It holds none of the
convolution's arithmetic, imports neither the CPU oracle nor the HIP path, and is the one
piece both sides are allowed to share.

Shapes follow the paper's notation (section 2.1) renamed as
N, C=C_I, HxW=H_I x W_I, RxS=H_F x W_F, K=C_O, PxQ=H_O x W_O; tensors are dense
NHWC (input), KRSC (filters), NPQK (output).

Input recipe (stands in for ImageNet-inference activations and trained filters of the paper's
seven CNNs, which dense-convolution timing does not depend on):
    x ~ U[-1,1],  w ~ U[-1,1] / sqrt(C_real * R * S)
drawn in fp64 from numpy's PCG64 at fixed per-layer seeds, cast to fp32, and then rounded
(round-to-nearest-even) onto the grid of the layer's 16-bit input type, so that the values
handed to either side are exactly representable in that type.  The result is returned as fp32
arrays holding those representable values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

DT_F32, DT_BF16, DT_F16 = "f32", "bf16", "f16"


@dataclass(frozen=True)
class ConvLayer:
    name: str
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    dilation: int
    dtype: str = DT_BF16
    seed_id: int = 0
    c_real: int | None = None  # channels that carry data (the rest are zero padding)

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.dilation * (self.R - 1) - 1) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.dilation * (self.S - 1) - 1) // self.stride + 1

    @property
    def M(self) -> int:
        return self.N * self.P * self.Q

    @property
    def k_gemm(self) -> int:
        return self.C * self.R * self.S

    @property
    def flops(self) -> int:
        """2*M*K*C*R*S with the channels as stored (zero padding channels included)."""
        return 2 * self.M * self.K * self.k_gemm

    @property
    def flops_real(self) -> int:
        c = self.c_real if self.c_real is not None else self.C
        return 2 * self.M * self.K * c * self.R * self.S

    def elt_bytes(self) -> int:
        return 4 if self.dtype == DT_F32 else 2

    def algorithmic_bytes(self, out_bytes: int = 4) -> int:
        """Compulsory traffic: every touched input pixel once, the filters once, the output once.

        For a 1x1 filter with stride > 1 only the sampled pixels count as touched."""
        e = self.elt_bytes()
        if self.R == 1 and self.S == 1 and self.stride > 1:
            x_elems = self.N * self.P * self.Q * self.C
        else:
            x_elems = self.N * self.H * self.W * self.C
        return x_elems * e + self.K * self.k_gemm * e + self.M * self.K * out_bytes

    def shape_args(self):
        return (self.N, self.H, self.W, self.C, self.K, self.R, self.S,
                self.stride, self.pad, self.dilation)


# The five benchmark configurations (seven layers).  Seeds: x -> 1000+seed_id, w -> 2000+seed_id.
LAYERS = {
    "cfg1": ConvLayer("cfg1", 1, 8, 8, 16, 16, 3, 3, 1, 1, 1, DT_F32, 1),
    "cfg2": ConvLayer("cfg2", 32, 56, 56, 64, 64, 3, 3, 1, 1, 1, DT_BF16, 2),
    "cfg3a": ConvLayer("cfg3a", 32, 56, 56, 128, 128, 3, 3, 2, 1, 1, DT_BF16, 30),
    "cfg3b": ConvLayer("cfg3b", 32, 56, 56, 256, 512, 1, 1, 2, 0, 1, DT_BF16, 31),
    "cfg4": ConvLayer("cfg4", 8, 64, 64, 256, 256, 3, 3, 1, 2, 2, DT_BF16, 4),
    "cfg5a": ConvLayer("cfg5a", 64, 224, 224, 4, 64, 7, 7, 2, 3, 1, DT_BF16, 50, c_real=3),
    "cfg5b": ConvLayer("cfg5b", 64, 7, 7, 512, 512, 3, 3, 1, 1, 1, DT_BF16, 51),
}
BENCH_LAYER = "cfg2"


def round_to_grid(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values to the nearest value representable in `dtype` (ties to even).

    Returns fp32.  bf16 is done on the bit pattern (keep the top 16 bits of the fp32 word);
    fp16 through numpy's own float16 cast."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == DT_F32:
        return a.copy()
    if dtype == DT_F16:
        return a.astype(np.float16).astype(np.float32)
    if dtype == DT_BF16:
        u = a.view(np.uint32).astype(np.uint64)
        lsb = (u >> 16) & 1
        u = (u + 0x7FFF + lsb) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(a.shape)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_inputs(layer: ConvLayer, seed_offset: int = 0):
    """Return (x[N,H,W,C], w[K,R,S,C]) as fp32 arrays of values representable in layer.dtype."""
    c_real = layer.c_real if layer.c_real is not None else layer.C
    gx = np.random.Generator(np.random.PCG64(1000 + layer.seed_id + seed_offset))
    gw = np.random.Generator(np.random.PCG64(2000 + layer.seed_id + seed_offset))
    x = gx.uniform(-1.0, 1.0, size=(layer.N, layer.H, layer.W, layer.C)).astype(np.float32)
    w = gw.uniform(-1.0, 1.0, size=(layer.K, layer.R, layer.S, layer.C))
    w = (w / np.sqrt(c_real * layer.R * layer.S)).astype(np.float32)
    if c_real < layer.C:
        x[..., c_real:] = 0.0
        w[..., c_real:] = 0.0
    return round_to_grid(x, layer.dtype), round_to_grid(w, layer.dtype)


def small_layer(name, N, H, W, C, K, R, S, stride=1, pad=0, dilation=1, dtype=DT_BF16, seed_id=900):
    return ConvLayer(name, N, H, W, C, K, R, S, stride, pad, dilation, dtype, seed_id)


def study_layers():
    """Shapes of the stride / dilation sensitivity study (the paper's central characterisation,
    section 3.2 and its stride figure): the headline 3x3 layer at strides 1, 2, 4 and dilations
    1, 2, 4 ("same" padding = dilation, so the stride alone sets the output size), batch 32.
    Returns [(label, ConvLayer)]."""
    base = LAYERS["cfg2"]
    out = []
    for stride in (1, 2, 4):
        for dil in (1, 2, 4):
            out.append((f"s{stride}_d{dil}", ConvLayer(f"study_s{stride}_d{dil}", base.N, base.H, base.W, base.C, base.K, 3, 3,
                                                       stride, dil, dil, base.dtype, 600 + 10 * stride + dil)))
    return out


def with_batch(layer, n):
    """The same layer at another batch size (the paper evaluates at batch 8 and 64, section 6)."""
    return ConvLayer(f"{layer.name}_n{n}", n, layer.H, layer.W, layer.C, layer.K, layer.R, layer.S, layer.stride, layer.pad,
                     layer.dilation, layer.dtype, layer.seed_id + 7000 + n, layer.c_real)
