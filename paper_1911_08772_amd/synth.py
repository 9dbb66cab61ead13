"""Seeded synthetic workloads: the paper's model sizes (Table 1; d of ResNet-50 from Sec. 3.3)
with bell-shaped, zero-centred values standing in for real gradients (Sec. 3.1).

Input generation only -- nothing of the compression method lives here.  The arrays are host
numpy arrays; the same bytes feed the CPU checker and (after a copy) the GPU path.
"""
import ctypes as C
import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

from . import build as _build

BASE_SEED = 191108772

_lib = None


def _L():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.ensure_synth())
        fp = C.POINTER(C.c_float)
        L.synth_normal.argtypes = [fp, C.c_int64, C.c_uint64, C.c_uint64, C.c_int64, C.c_double]
        L.synth_mixture.argtypes = [fp, C.c_int64, C.c_uint64, C.c_uint64, C.c_int64, C.c_double,
                                    C.c_double, C.c_double]
        L.synth_student_t3.argtypes = [fp, C.c_int64, C.c_uint64, C.c_uint64, C.c_int64,
                                       C.c_double]
        L.synth_uniform.argtypes = [C.POINTER(C.c_double), C.c_int64, C.c_uint64, C.c_uint64,
                                    C.c_int64]
        for f in (L.synth_normal, L.synth_mixture, L.synth_student_t3, L.synth_uniform):
            f.restype = None
        _lib = L
    return _lib


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def normal(n: int, seed: int, stream: int, sigma: float, out: Optional[np.ndarray] = None,
           index0: int = 0) -> np.ndarray:
    out = np.empty(n, np.float32) if out is None else out
    _L().synth_normal(_fp(out), n, seed, stream, index0, sigma)
    return out


def mixture(n: int, seed: int, stream: int, sigma_a: float, sigma_b: float, p_b: float,
            out: Optional[np.ndarray] = None) -> np.ndarray:
    out = np.empty(n, np.float32) if out is None else out
    _L().synth_mixture(_fp(out), n, seed, stream, 0, sigma_a, sigma_b, p_b)
    return out


def student_t3(n: int, seed: int, stream: int, scale: float,
               out: Optional[np.ndarray] = None) -> np.ndarray:
    out = np.empty(n, np.float32) if out is None else out
    _L().synth_student_t3(_fp(out), n, seed, stream, 0, scale)
    return out


def uniform(n: int, seed: int, stream: int) -> np.ndarray:
    out = np.empty(n, np.float64)
    _L().synth_uniform(out.ctypes.data_as(C.POINTER(C.c_double)), n, seed, stream, 0)
    return out


def k_of(d: int, rho_den: int) -> int:
    """k = ceil(d / rho_den) in integer arithmetic (rho = 1/rho_den)."""
    return (d + rho_den - 1) // rho_den


@dataclass
class Workload:
    """One benchmark/parity configuration: sizes, density, steps and the gradient recipe."""
    name: str
    d: int
    rho_den: int          # rho = 1 / rho_den
    steps: int
    dist: str             # "normal" | "mixture" | "student_t3" | "segmented_normal"
    params: Tuple
    seed: int
    seg_off: Optional[np.ndarray] = None     # int64[L+1] for the layer-wise workload
    seg_sigma: Optional[np.ndarray] = None   # float64[L]
    seg_k: Optional[np.ndarray] = field(default=None)

    @property
    def k(self) -> int:
        return k_of(self.d, self.rho_den)

    def describe(self) -> str:
        """One line naming the sizes and the gradient recipe (for benchmark records)."""
        recipe = {"normal": lambda: f"g~N(0, sigma={self.params[0]:g})",
                  "mixture": lambda: (f"g~N(0, {self.params[0]:g}) w.p. {1 - self.params[2]:g}, "
                                      f"N(0, {self.params[1]:g}) w.p. {self.params[2]:g} per element"),
                  "student_t3": lambda: f"g={self.params[0]:g}*Student-t(3)",
                  "segmented_normal": lambda: "per-segment N(0, sigma_l), sigma_l log-uniform"}
        return f"{self.name}: d={self.d}, k={self.k}, {recipe[self.dist]()} seeded"

    def grad(self, step: int, out: Optional[np.ndarray] = None) -> np.ndarray:
        """Fresh gradient of iteration `step` (stream = step)."""
        if self.dist == "normal":
            return normal(self.d, self.seed, step, self.params[0], out)
        if self.dist == "mixture":
            return mixture(self.d, self.seed, step, *self.params, out=out)
        if self.dist == "student_t3":
            return student_t3(self.d, self.seed, step, self.params[0], out)
        if self.dist == "segmented_normal":
            out = np.empty(self.d, np.float32) if out is None else out
            for l in range(self.seg_sigma.size):
                a, b = int(self.seg_off[l]), int(self.seg_off[l + 1])
                normal(b - a, self.seed, step, float(self.seg_sigma[l]), out[a:b], index0=a)
            return out
        raise ValueError(self.dist)


def segment_layout(d_total: int, num_segments: int, lo: float, hi: float, seed: int,
                   rho_den: int = 1000):
    """Segment sizes log-uniform in [lo, hi], rescaled (floor, remainder to the largest) to sum
    to d_total; per-segment k = max(1, ceil(d_l / rho_den))."""
    u = uniform(num_segments, seed, 1 << 40)
    raw = np.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))
    sizes = np.maximum(1, np.floor(raw * (d_total / raw.sum()))).astype(np.int64)
    sizes[int(np.argmax(sizes))] += d_total - int(sizes.sum())
    assert sizes.min() >= 1 and int(sizes.sum()) == d_total
    seg_off = np.zeros(num_segments + 1, np.int64)
    np.cumsum(sizes, out=seg_off[1:])
    seg_k = np.maximum(1, (sizes + rho_den - 1) // rho_den).astype(np.int64)
    return seg_off, seg_k


def workload(name: str) -> Workload:
    """The five configurations (sizes from the paper's Table 1 and Sec. 3.3)."""
    if name == "cfg1_resnet20":
        return Workload(name, 269_722, 1000, 10, "normal", (0.01,), BASE_SEED + 1)
    if name == "cfg2_vgg16":
        return Workload(name, 14_728_266, 1000, 50, "mixture", (1e-3, 1e-2, 0.1), BASE_SEED + 2)
    if name == "cfg3_resnet50":
        return Workload(name, 25_557_032, 1000, 20, "normal", (1e-3,), BASE_SEED + 3)
    if name == "cfg3_resnet50_rho01":
        return Workload(name, 25_557_032, 100, 20, "normal", (1e-3,), BASE_SEED + 3)
    if name == "cfg4_segmented":
        seed = BASE_SEED + 4
        seg_off, seg_k = segment_layout(25_557_032, 54, 64.0, 2.4e6, seed)
        u = uniform(54, seed, (1 << 40) + 1)
        sig = np.exp(math.log(1e-4) + u * (math.log(1e-1) - math.log(1e-4)))
        return Workload(name, 25_557_032, 1000, 20, "segmented_normal", (), seed, seg_off, sig,
                        seg_k)
    if name == "cfg5_lstm":
        return Workload(name, 66_034_000, 1000, 100, "student_t3", (1e-3,), BASE_SEED + 5)
    if name.startswith("normal_d"):  # e.g. normal_d41943040: the d-sweep's vectors as a chain
        return Workload(name, int(name[len("normal_d"):]), 1000, 20, "normal", (1e-3,), BASE_SEED + 9)
    raise KeyError(name)


ALL_WORKLOADS: List[str] = ["cfg1_resnet20", "cfg2_vgg16", "cfg3_resnet50", "cfg3_resnet50_rho01",
                            "cfg4_segmented", "cfg5_lstm"]
