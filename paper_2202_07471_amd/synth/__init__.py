"""Seeded synthetic weight tensors with the shapes of the evaluated networks.

Input plumbing only: no quantization arithmetic lives here.  The tensors stand
in for the trained ImageNet CNN weights the paper quantizes (Section 4): real
layer shapes, He-normal values (optionally heavy tailed).  Values come from the
counter-based generator in ``synth_gen.c`` and are produced once on the host;
the same buffer is handed to the GPU library and to the CPU reference checker.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "synth_gen.c")
_LIB = os.path.join(_HERE, "libsquant_synth.so")

DEFAULT_SEED = 20220215

Shape = Tuple[int, int, int, int]  # (cout, cin_per_group, kh, kw)


def build(force: bool = True) -> str:
    """Compile the generator (host C, OpenMP)."""
    if force or not os.path.exists(_LIB):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        lib = ctypes.CDLL(_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        lib.synth_fill_normal.argtypes = [f32p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32,
                                          ctypes.c_double]
        lib.synth_fill_student_t3.argtypes = lib.synth_fill_normal.argtypes
        lib.synth_fill_normal_laplace.argtypes = lib.synth_fill_normal.argtypes + [
            ctypes.c_double, ctypes.c_double]
        lib.synth_coin.argtypes = [ctypes.c_uint64, ctypes.c_uint32]
        lib.synth_coin.restype = ctypes.c_int32
        for fn in (lib.synth_fill_normal, lib.synth_fill_student_t3, lib.synth_fill_normal_laplace):
            fn.restype = None
        _lib = lib
    return _lib


def he_sigma(shape: Shape) -> float:
    """Fan-in He-normal standard deviation sqrt(2 / (cin_per_group * kh * kw))."""
    _, cin, kh, kw = shape
    return math.sqrt(2.0 / (cin * kh * kw))


def _out(shape: Shape, out):
    n = int(np.prod(shape))
    if out is None:
        out = np.empty(shape, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == n and out.flags["C_CONTIGUOUS"]
    return out, n, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def stream_id(config: int, tensor: int) -> int:
    return (config << 20) | tensor


def normal(shape: Shape, seed: int, stream: int, sigma: float, out=None) -> np.ndarray:
    out, n, p = _out(shape, out)
    _load().synth_fill_normal(p, n, seed, stream, sigma)
    return out


def student_t3(shape: Shape, seed: int, stream: int, sigma: float, out=None) -> np.ndarray:
    out, n, p = _out(shape, out)
    _load().synth_fill_student_t3(p, n, seed, stream, sigma)
    return out


def normal_laplace(shape: Shape, seed: int, stream: int, sigma: float, prob: float, b: float,
                   out=None) -> np.ndarray:
    out, n, p = _out(shape, out)
    _load().synth_fill_normal_laplace(p, n, seed, stream, sigma, prob, b)
    return out


def coin(seed: int, stream: int) -> int:
    return int(_load().synth_coin(seed, stream))


# --------------------------------------------------------------------------
# Layer-shape lists (standard architectures; conv and FC weights only)
# --------------------------------------------------------------------------

def resnet18_shapes() -> List[Shape]:
    s: List[Shape] = [(64, 3, 7, 7)]
    s += [(64, 64, 3, 3)] * 4
    for w_in, w in ((64, 128), (128, 256), (256, 512)):
        s += [(w, w_in, 3, 3), (w, w, 3, 3), (w, w_in, 1, 1), (w, w, 3, 3), (w, w, 3, 3)]
    s.append((1000, 512, 1, 1))
    return s


def resnet50_shapes() -> List[Shape]:
    s: List[Shape] = [(64, 3, 7, 7)]
    cin = 64
    for w, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            s += [(w, cin, 1, 1), (w, w, 3, 3), (4 * w, w, 1, 1)]
            if b == 0:
                s.append((4 * w, cin, 1, 1))
            cin = 4 * w
    s.append((1000, 2048, 1, 1))
    return s


def mobilenetv2_shapes() -> List[Shape]:
    s: List[Shape] = [(32, 3, 3, 3)]
    cin = 32
    for t, c, n in ((1, 16, 1), (6, 24, 2), (6, 32, 3), (6, 64, 4), (6, 96, 3), (6, 160, 3),
                    (6, 320, 1)):
        for _ in range(n):
            hidden = t * cin
            if t != 1:
                s.append((hidden, cin, 1, 1))
            s.append((hidden, 1, 3, 3))      # depthwise: one input channel per group
            s.append((c, hidden, 1, 1))
            cin = c
    s.append((1280, 320, 1, 1))
    s.append((1000, 1280, 1, 1))
    return s


def inceptionv3_shapes() -> List[Shape]:
    """Factorised-convolution network in the style of InceptionV3 (main branch, no auxiliary
    head): 1x7 / 7x1, 1x3 / 3x1 and 5x5 kernels beside 3x3 and 1x1 ones."""
    s: List[Shape] = [(32, 3, 3, 3), (32, 32, 3, 3), (64, 32, 3, 3), (80, 64, 1, 1), (192, 80, 3, 3)]
    for cin, pool in ((192, 32), (256, 64), (288, 64)):                 # 35 x 35 blocks
        s += [(64, cin, 1, 1), (48, cin, 1, 1), (64, 48, 5, 5), (64, cin, 1, 1), (96, 64, 3, 3),
              (96, 96, 3, 3), (pool, cin, 1, 1)]
    s += [(384, 288, 3, 3), (64, 288, 1, 1), (96, 64, 3, 3), (96, 96, 3, 3)]   # reduction to 17 x 17
    for c7 in (128, 160, 160, 192):                                     # 17 x 17 blocks
        s += [(192, 768, 1, 1), (c7, 768, 1, 1), (c7, c7, 1, 7), (192, c7, 7, 1),
              (c7, 768, 1, 1), (c7, c7, 7, 1), (c7, c7, 1, 7), (c7, c7, 7, 1), (192, c7, 1, 7),
              (192, 768, 1, 1)]
    s += [(192, 768, 1, 1), (320, 192, 3, 3), (192, 768, 1, 1), (192, 192, 1, 7), (192, 192, 7, 1),
          (192, 192, 3, 3)]                                             # reduction to 8 x 8
    for cin in (1280, 2048):                                            # 8 x 8 blocks
        s += [(320, cin, 1, 1), (384, cin, 1, 1), (384, 384, 1, 3), (384, 384, 3, 1),
              (448, cin, 1, 1), (384, 448, 3, 3), (384, 384, 1, 3), (384, 384, 3, 1), (192, cin, 1, 1)]
    s.append((1000, 2048, 1, 1))
    return s


@dataclass(frozen=True)
class TensorSpec:
    config: int
    index: int
    shape: Shape
    dist: str            # "normal" | "normal_laplace" | "student_t3"
    sigma: float

    @property
    def numel(self) -> int:
        return int(np.prod(self.shape))


def config_specs(config: int, seed: int = DEFAULT_SEED, n_tensors: int | None = None
                 ) -> List[TensorSpec]:
    """Tensor list of workload `config` (1..6).

    1: one [64,64,3,3] He-normal tensor.            2: ResNet-18 layer set, He-normal.
    3: ResNet-50 layer set, He-normal with 1 % Laplace(0, 3 sigma) outliers.
    4: MobileNetV2 layer set, He-normal.
    5: 256 x [512,512,3,3]; a seeded fair coin per tensor picks N(0, sigma) or
       sigma * Student-t(3).  `n_tensors` truncates the list (same leading tensors).
    6: InceptionV3-style layer set (factorised 1x7 / 7x1 / 1x3 / 3x1 and 5x5 kernels), He-normal.
    """
    if config == 1:
        shapes, dist = [(64, 64, 3, 3)], "normal"
    elif config == 2:
        shapes, dist = resnet18_shapes(), "normal"
    elif config == 3:
        shapes, dist = resnet50_shapes(), "normal_laplace"
    elif config == 4:
        shapes, dist = mobilenetv2_shapes(), "normal"
    elif config == 5:
        shapes, dist = [(512, 512, 3, 3)] * 256, "coin"
    elif config == 6:
        shapes, dist = inceptionv3_shapes(), "normal"
    else:
        raise ValueError(f"unknown config {config}")
    if n_tensors is not None:
        shapes = shapes[:n_tensors]
    specs = []
    for i, shp in enumerate(shapes):
        d = dist
        if d == "coin":
            d = "student_t3" if coin(seed, stream_id(config, i)) else "normal"
        specs.append(TensorSpec(config, i, shp, d, he_sigma(shp)))
    return specs


def generate(spec: TensorSpec, seed: int = DEFAULT_SEED, out=None) -> np.ndarray:
    st = stream_id(spec.config, spec.index)
    if spec.dist == "normal":
        return normal(spec.shape, seed, st, spec.sigma, out)
    if spec.dist == "student_t3":
        return student_t3(spec.shape, seed, st, spec.sigma, out)
    if spec.dist == "normal_laplace":
        return normal_laplace(spec.shape, seed, st, spec.sigma, 0.01, 3.0 * spec.sigma, out)
    raise ValueError(spec.dist)
