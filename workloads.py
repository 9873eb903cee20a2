"""Seeded synthetic inputs for the forward-convolution workloads.

This module serves both the CPU oracle's tests and the GPU library's tests / benchmark, and for
that reason holds none of the method's arithmetic: only the layer shapes, the random draws, and
the exact conversions between storage dtypes (fp32 / fp16 / bf16) and fp64.

The layer shapes are ResNet-style stages (a 224x224 RGB stem, 56x56 / 28x28 / 7x7 stages).  They
stand in for the GoogLeNet / Inception layers the MIOpen paper benchmarks (Sec. VI, Fig. 5), whose
exact list survives only in the figures' axis labels.

Draws: numpy Generator(PCG64) seeded from SeedSequence([191000078, workload index]), one spawned
child per tensor (x, w, bias), drawn in float64, rounded to float32, then to the storage dtype
with round-to-nearest-even.  The same host arrays feed the oracle (widened exactly to fp64) and
the GPU (copied bit for bit), so no random generator has to agree across languages.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

F32, F16, BF16 = "f32", "f16", "bf16"
BASE_SEED = 191000078


@dataclass(frozen=True)
class ConvWorkload:
    name: str
    dtype: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    pad: Tuple[int, int] = (0, 0)
    stride: Tuple[int, int] = (1, 1)
    dil: Tuple[int, int] = (1, 1)
    groups: int = 1
    x_dist: Tuple[str, float, float] = ("uniform", 0.0, 1.0)
    w_dist: Optional[Tuple[str, float, float]] = None     # None -> He normal, var 2/(C/groups*R*S)
    b_dist: Tuple[str, float, float] = ("uniform", -0.1, 0.1)
    seed_index: int = 0

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad[0] - self.dil[0] * (self.R - 1) - 1) // self.stride[0] + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad[1] - self.dil[1] * (self.S - 1) - 1) // self.stride[1] + 1

    @property
    def flops(self) -> int:
        """2 * N*K*Ho*Wo * (C/groups)*R*S  (bias and activation not counted)."""
        return 2 * self.N * self.K * self.Ho * self.Wo * (self.C // self.groups) * self.R * self.S

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    @property
    def algorithmic_bytes(self) -> int:
        """Every input, weight and bias element read once, every output element written once."""
        e = self.elem_bytes
        return e * (self.N * self.C * self.H * self.W
                    + self.K * (self.C // self.groups) * self.R * self.S
                    + self.K
                    + self.N * self.K * self.Ho * self.Wo)


# The five benchmark configurations (the third and fifth hold two layers each).
WORKLOADS = {
    "c1": ConvWorkload("c1", F32, 1, 8, 8, 8, 8, 3, 3, pad=(1, 1),
                       x_dist=("uniform", -1.0, 1.0), w_dist=("uniform", -1.0, 1.0),
                       b_dist=("uniform", -1.0, 1.0), seed_index=1),
    "c2": ConvWorkload("c2", BF16, 32, 64, 56, 56, 64, 3, 3, pad=(1, 1), seed_index=2),
    "c3a": ConvWorkload("c3a", BF16, 64, 256, 56, 56, 64, 1, 1, seed_index=3),
    "c3b": ConvWorkload("c3b", BF16, 64, 64, 56, 56, 256, 1, 1, seed_index=4),
    "c4": ConvWorkload("c4", F16, 64, 3, 224, 224, 64, 7, 7, pad=(3, 3), stride=(2, 2),
                       x_dist=("uniform", -1.0, 1.0), seed_index=5),
    "c5a": ConvWorkload("c5a", BF16, 128, 512, 7, 7, 512, 3, 3, pad=(1, 1), seed_index=6),
    "c5b": ConvWorkload("c5b", BF16, 128, 256, 28, 28, 256, 3, 3, pad=(1, 1), stride=(2, 2),
                        seed_index=7),
    # not one of the five configurations: the 56x56 stage layer in fp32, the benchmark row of the fp32 path
    "c2f32": ConvWorkload("c2f32", F32, 32, 64, 56, 56, 64, 3, 3, pad=(1, 1), seed_index=8),
}


# ---------------------------------------------------------------------------------------------
# exact dtype conversions (storage <-> float)
# ---------------------------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even; finite inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a32: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array -> storage representation: float32, float16, or uint16 bf16 bit patterns."""
    a32 = np.ascontiguousarray(a32, dtype=np.float32)
    if dtype == F32:
        return a32
    if dtype == F16:
        return a32.astype(np.float16)
    if dtype == BF16:
        return f32_to_bf16_bits(a32)
    raise ValueError(dtype)


def to_f64(stored: np.ndarray, dtype: str) -> np.ndarray:
    """Storage representation -> float64, exactly (every fp32/fp16/bf16 value is an fp64 value)."""
    if dtype == BF16:
        return bf16_bits_to_f32(stored).astype(np.float64)
    return np.asarray(stored).astype(np.float64)


def storage_numpy_dtype(dtype: str):
    return {F32: np.float32, F16: np.float16, BF16: np.uint16}[dtype]


# ---------------------------------------------------------------------------------------------
# seeded draws
# ---------------------------------------------------------------------------------------------
def _draw(rng: np.random.Generator, dist, shape) -> np.ndarray:
    kind, a, b = dist
    if kind == "uniform":
        return rng.uniform(a, b, size=shape)
    if kind == "normal":
        return rng.normal(a, b, size=shape)
    raise ValueError(kind)


def make_inputs(wl: ConvWorkload, seed: int = BASE_SEED, n_override: Optional[int] = None):
    """Return (x, w, bias) in storage representation for the workload.

    n_override draws only the first n images' worth of x (the stream is laid out image-major, so
    the leading images agree with the full draw).
    """
    ss = np.random.SeedSequence([seed, wl.seed_index]).spawn(3)
    N = wl.N if n_override is None else n_override
    cg = wl.C // wl.groups
    w_dist = wl.w_dist or ("normal", 0.0, float(np.sqrt(2.0 / (cg * wl.R * wl.S))))
    x = _draw(np.random.Generator(np.random.PCG64(ss[0])), wl.x_dist, (N, wl.C, wl.H, wl.W))
    w = _draw(np.random.Generator(np.random.PCG64(ss[1])), w_dist, (wl.K, cg, wl.R, wl.S))
    b = _draw(np.random.Generator(np.random.PCG64(ss[2])), wl.b_dist, (wl.K,))
    return (to_storage(x.astype(np.float32), wl.dtype),
            to_storage(w.astype(np.float32), wl.dtype),
            to_storage(b.astype(np.float32), wl.dtype))


def small_variant(wl: ConvWorkload, **changes) -> ConvWorkload:
    """A copy of the workload with some fields replaced (used for reduced-size parity cases)."""
    d = {f: getattr(wl, f) for f in wl.__dataclass_fields__}
    d.update(changes)
    return ConvWorkload(**d)
