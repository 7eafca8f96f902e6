"""CPU oracle (test infrastructure): what the pattern-sparse 3x3 convolution path must compute, written from the
paper's definitions.  Only tests, the smoke check and the bench's cpu_baseline leg import this package; the product
package never does.

conv_oracle.c   direct convolution over masked dense weights, double accumulation (built by `build()` with gcc)
pattern_oracle  masking, pattern assignment, connectivity selection, canonical packing (numpy, float64)
admm_oracle     the selection-variable steps of the pruning framework: simplex projection, multiplier update, argmax
backward_oracle input and masked weight gradients of the pruned layer; the 1x1 layer grouped into 3x3 patterns
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .admm_oracle import binarize, proximal_step, simplex_project  # noqa: F401
from .backward_oracle import (  # noqa: F401
    conv1x1, conv3x3_grad_input, conv3x3_grad_weight, conv3x3_grad_weight_at, group_mask_1x1, masked_grad_weight,
)
from .pattern_oracle import (  # noqa: F401
    assign_patterns, filter_similarity_order, library_bits, mask_weights, pack_canonical, retained_energy,
    select_connectivity, unpack_canonical,
)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile conv_oracle.c with gcc.  -ffp-contract=off keeps every product and sum separately rounded."""
    src = os.path.join(_HERE, "conv_oracle.c")
    if force or not os.path.exists(_SO):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _SO, src]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build(force=True)
        lib = ctypes.CDLL(_SO)
        fp, dp, ip = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
        i = ctypes.c_int
        lib.oracle_conv3x3.argtypes = [fp, fp, fp, i, i, i, i, i, i, i, i, dp]
        lib.oracle_conv3x3.restype = i
        lib.oracle_conv3x3_at.argtypes = [fp, fp, fp, i, i, i, i, i, i, i, i, ip, ctypes.c_long, dp]
        lib.oracle_conv3x3_at.restype = i
        lib.oracle_maxpool2x2.argtypes = [fp, ctypes.c_long, i, i, fp]
        lib.oracle_maxpool2x2.restype = i
        lib.oracle_threads.restype = i
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float32)   # fp16 -> fp32 is lossless


def _ptr(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def threads() -> int:
    return int(_load().oracle_threads())


def out_hw(H: int, W: int, stride: int, pad: int):
    return (H + 2 * pad - 3) // stride + 1, (W + 2 * pad - 3) // stride + 1


def conv3x3(x, wm, bias=None, stride: int = 1, pad: int = 1, relu: bool = False) -> np.ndarray:
    """Direct 3x3 convolution of x [N][C][H][W] with (masked) dense weights wm [F][C][3][3]; returns float64."""
    x, wm = _f32(x), _f32(wm)
    N, C, H, W = x.shape
    F = wm.shape[0]
    assert wm.shape == (F, C, 3, 3)
    b = _f32(bias) if bias is not None else None
    Ho, Wo = out_hw(H, W, stride, pad)
    y = np.empty((N, F, max(Ho, 0), max(Wo, 0)), dtype=np.float64)
    rc = _load().oracle_conv3x3(_ptr(x, ctypes.c_float), _ptr(wm, ctypes.c_float), _ptr(b, ctypes.c_float),
                                N, C, F, H, W, stride, pad, int(relu), _ptr(y, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_conv3x3 rejected its arguments (rc={rc})")
    return y


def pattern_conv3x3(x, w, pid, mask, lib, bias=None, stride: int = 1, pad: int = 1, relu: bool = False) -> np.ndarray:
    """The pruned layer: mask the dense weights with each kernel's pattern and connectivity bit, then convolve."""
    return conv3x3(x, mask_weights(w, pid, mask, lib), bias, stride, pad, relu)


def conv3x3_at(x, wm, coords, bias=None, stride: int = 1, pad: int = 1, relu: bool = False) -> np.ndarray:
    """The same sum at the listed output coordinates [npts][4] = (n, f, oy, ox); returns float64 [npts]."""
    x, wm = _f32(x), _f32(wm)
    N, C, H, W = x.shape
    F = wm.shape[0]
    b = _f32(bias) if bias is not None else None
    coords = np.ascontiguousarray(coords, dtype=np.int32).reshape(-1, 4)
    out = np.empty(coords.shape[0], dtype=np.float64)
    rc = _load().oracle_conv3x3_at(_ptr(x, ctypes.c_float), _ptr(wm, ctypes.c_float), _ptr(b, ctypes.c_float),
                                   N, C, F, H, W, stride, pad, int(relu), _ptr(coords, ctypes.c_int32),
                                   coords.shape[0], _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"oracle_conv3x3_at rejected its arguments (rc={rc})")
    return out


def maxpool2x2(x) -> np.ndarray:
    """2x2 max-pool with stride 2 over the last two axes; float32 in, float32 out."""
    x = _f32(x)
    H, W = x.shape[-2:]
    planes = int(np.prod(x.shape[:-2]))
    y = np.empty(x.shape[:-2] + (H // 2, W // 2), dtype=np.float32)
    rc = _load().oracle_maxpool2x2(_ptr(x, ctypes.c_float), planes, H, W, _ptr(y, ctypes.c_float))
    if rc != 0:
        raise ValueError("oracle_maxpool2x2 rejected its arguments")
    return y
