"""Synthetic layer tables and tensors for the five benchmark configurations.

Everything here is a seeded draw or a table of shapes.  The method's own steps
(pattern assignment by retained norm, connectivity top-k, masking, packing,
convolution) are NOT here: the oracle and the HIP library each do them on the
raw tensors this module returns.

Shapes follow VGG-16 (13 conv layers, 3x3, 224x224 input) and the 3x3
convolutions of ResNet-50 bottlenecks; values follow He initialisation for the
weights and a rectified standard normal (half of the entries exactly zero) for
the activations, which is what a layer behind a ReLU sees.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional

import numpy as np

from . import rng

KIND_W, KIND_X, KIND_B, KIND_LIB, KIND_PID, KIND_MASK = 0, 1, 2, 3, 4, 5

# Tap index t = 3*ky + kx; ky = 0 is the tap that reads the row above the output pixel (at pad 1),
# kx = 0 the column to its left.  A pattern is a 9-bit mask with bit t set where the weight is kept.
CENTRE = 4
FIXED4 = (0x01B, 0x036, 0x0D8, 0x1B0)  # {c,up,left,up-left} {c,up,right,up-right} {c,down,left,down-left} {c,down,right,down-right}


def all_masks_4of9() -> List[int]:
    """All 126 = C(9,4) masks with four kept taps, ascending."""
    return [m for m in range(512) if bin(m).count("1") == 4]


def centre_masks() -> List[int]:
    """The 56 = C(8,3) masks that keep the centre tap and three of its eight neighbours, ascending."""
    return [m for m in all_masks_4of9() if (m >> CENTRE) & 1]


def drawn_library(cfg: int, K: int) -> np.ndarray:
    """First K masks of one seeded shuffle of the 56 centre-containing masks: K=4 is inside K=8 inside K=12."""
    order = rng.shuffle(rng.stream_seed(cfg, 0, KIND_LIB), centre_masks())
    return np.asarray(order[:K], dtype=np.uint16)


@dataclass(frozen=True)
class LayerSpec:
    cfg: int
    idx: int
    name: str
    N: int
    C: int
    F: int
    H: int
    W: int
    stride: int = 1
    pad: int = 1
    dtype: str = "f32"          # storage type of x, y, w: "f32" or "f16"; accumulation is always fp32 on the GPU
    K: int = 8
    keep: float = 1.0
    lib_kind: str = "draw"      # "fixed4" (config 0), "draw" (seeded nested draw) or "all126" (every mask; tests)
    assign: str = "argmax"      # "uniform" (config 0: seeded uniform ids) or "argmax" (retained-norm projection)
    conn: str = "topk"          # "bernoulli" (config 0) or "topk"
    relu: bool = False
    pool_after: bool = False

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - 3) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - 3) // self.stride + 1

    @property
    def np_dtype(self):
        return np.float16 if self.dtype == "f16" else np.float32

    def library(self) -> np.ndarray:
        if self.lib_kind == "fixed4":
            return np.asarray(FIXED4[: self.K], dtype=np.uint16)
        if self.lib_kind == "all126":
            return np.asarray(all_masks_4of9()[: self.K], dtype=np.uint16)
        return drawn_library(self.cfg, self.K)

    def n_keep_target(self) -> int:
        """Kernels kept by the top-k rule: floor(keep*F*C + 0.5)."""
        return int(np.floor(self.keep * float(self.F * self.C) + 0.5))


# ----------------------------------------------------------------------------------------------
# raw tensors
# ----------------------------------------------------------------------------------------------

def gen_weights(s: LayerSpec) -> np.ndarray:
    """[F][C][3][3], N(0, 2/(9*Cin)) (the second argument is a variance), rounded to the storage type."""
    z = rng.normal(rng.stream_seed(s.cfg, s.idx, KIND_W), s.F * s.C * 9)
    w = (z * np.sqrt(2.0 / (9.0 * s.C))).astype(np.float32)
    return w.astype(s.np_dtype).reshape(s.F, s.C, 3, 3)


KIND_CLUSTER = 6


def gen_clustered_weights(s: LayerSpec, clusters: int, share: float, damp: float = 0.05) -> np.ndarray:
    """Weights with the connectivity structure of a trained, pruned model rather than of a random draw: every filter
    belongs to one of `clusters` groups (seeded, scattered over the filter indices, equal sizes), every group has its
    own seeded subset of share*C input channels, and a filter's kernels on channels outside its group's subset are
    scaled by `damp` -- so that selection by kernel norm keeps, for similar filters, the same channels.  Same
    distribution otherwise as gen_weights.  Returns (weights, group of every filter)."""
    w = gen_weights(s).astype(np.float32)
    seed = rng.stream_seed(s.cfg, s.idx, KIND_CLUSTER)
    filters = rng.shuffle(seed, list(range(s.F)))
    group = np.empty(s.F, dtype=np.int64)
    for pos, f in enumerate(filters):
        group[f] = pos * clusters // s.F
    n_in = max(1, int(round(share * s.C)))
    for g in range(clusters):
        inside = np.zeros(s.C, dtype=bool)
        inside[rng.shuffle(rng.stream_seed(s.cfg, s.idx, KIND_CLUSTER, g + 1), list(range(s.C)))[:n_in]] = True
        rows = np.nonzero(group == g)[0]
        w[np.ix_(rows, np.nonzero(~inside)[0])] *= damp
    return w.astype(s.np_dtype), group


def gen_bias(s: LayerSpec) -> np.ndarray:
    """[F] fp32, N(0, 0.01) (variance, so sigma = 0.1)."""
    z = rng.normal(rng.stream_seed(s.cfg, s.idx, KIND_B), s.F)
    return (z * 0.1).astype(np.float32)


def gen_image(s: LayerSpec, n: int) -> np.ndarray:
    """[C][H][W] activations of image n: max(z, 0) with z ~ N(0,1), rounded to the storage type."""
    z = rng.normal(rng.stream_seed(s.cfg, s.idx, KIND_X, n), s.C * s.H * s.W)
    return np.maximum(z, 0.0).astype(np.float32).astype(s.np_dtype).reshape(s.C, s.H, s.W)


def gen_activations(s: LayerSpec, images: Optional[List[int]] = None) -> np.ndarray:
    """[N][C][H][W] (or the listed images only)."""
    ids = list(range(s.N)) if images is None else list(images)
    out = np.empty((len(ids), s.C, s.H, s.W), dtype=s.np_dtype)
    for k, n in enumerate(ids):
        out[k] = gen_image(s, n)
    return out


def gen_uniform_pattern_ids(s: LayerSpec) -> np.ndarray:
    """[F][C] uint8, uniform over the library (config 0 only; the other configs assign by retained norm)."""
    return rng.randint(rng.stream_seed(s.cfg, s.idx, KIND_PID), s.F * s.C, s.K).astype(np.uint8).reshape(s.F, s.C)


def gen_bernoulli_mask(s: LayerSpec) -> np.ndarray:
    """[F][C] uint8, 1 = kernel kept, each kernel kept with probability `keep` (config 0 only)."""
    u = rng.uniform01(rng.stream_seed(s.cfg, s.idx, KIND_MASK), s.F * s.C)
    return (u <= s.keep).astype(np.uint8).reshape(s.F, s.C)


# ----------------------------------------------------------------------------------------------
# layer tables
# ----------------------------------------------------------------------------------------------

# (C, F, H) of the 13 VGG-16 conv layers; True = a 2x2 max-pool follows
VGG16 = [
    (3, 64, 224, False), (64, 64, 224, True),
    (64, 128, 112, False), (128, 128, 112, True),
    (128, 256, 56, False), (256, 256, 56, False), (256, 256, 56, True),
    (256, 512, 28, False), (512, 512, 28, False), (512, 512, 28, True),
    (512, 512, 14, False), (512, 512, 14, False), (512, 512, 14, True),
]
VGG16_NAMES = ["conv1_1", "conv1_2", "conv2_1", "conv2_2", "conv3_1", "conv3_2", "conv3_3",
               "conv4_1", "conv4_2", "conv4_3", "conv5_1", "conv5_2", "conv5_3"]
# keep fraction per layer of the config-2 chain: first layer patterns only, then one value per width group
VGG16_KEEP_CHAIN = [1.0, 0.35, 0.35, 0.35, 0.28, 0.28, 0.28, 0.20, 0.20, 0.20, 0.20, 0.20, 0.20]

# (C, H, stride) of the ResNet-50 bottleneck 3x3 convolutions; Cin = Cout
RESNET50_3X3 = [(64, 56, 1), (128, 56, 2), (128, 28, 1), (256, 28, 2), (256, 14, 1), (512, 14, 2), (512, 7, 1)]


def config0() -> LayerSpec:
    return LayerSpec(cfg=0, idx=0, name="tiny16", N=1, C=16, F=16, H=32, W=32, K=4, keep=0.5,
                     lib_kind="fixed4", assign="uniform", conn="bernoulli")


def config1() -> LayerSpec:
    return LayerSpec(cfg=1, idx=0, name="vgg_conv3_x", N=1, C=256, F=256, H=56, W=56, K=8, keep=0.28)


def config2() -> List[LayerSpec]:
    return [LayerSpec(cfg=2, idx=i, name=VGG16_NAMES[i], N=1, C=c, F=f, H=h, W=h, K=8, keep=VGG16_KEEP_CHAIN[i],
                      relu=True, pool_after=p) for i, (c, f, h, p) in enumerate(VGG16)]


def config3(N: int) -> List[LayerSpec]:
    return [LayerSpec(cfg=3, idx=i, name=f"res{c}_{h}_s{st}", N=N, C=c, F=c, H=h, W=h, stride=st, dtype="f16", K=8,
                      keep=0.3) for i, (c, h, st) in enumerate(RESNET50_3X3)]


def vgg_distinct_shapes() -> List[int]:
    """Indices into VGG16 of the 9 distinct (C, F, H) shapes."""
    seen, out = set(), []
    for i, (c, f, h, _) in enumerate(VGG16):
        if (c, f, h) not in seen:
            seen.add((c, f, h))
            out.append(i)
    return out


def config4(K: int = 8, keep: float = 0.28, N: int = 64) -> List[LayerSpec]:
    """One sweep point: the 9 distinct VGG shapes at batch N, fp16 storage; conv1_1 (Cin = 3) stays at keep 1.0."""
    out = []
    for i in vgg_distinct_shapes():
        c, f, h, _ = VGG16[i]
        out.append(LayerSpec(cfg=4, idx=i, name=VGG16_NAMES[i], N=N, C=c, F=f, H=h, W=h, dtype="f16", K=K,
                             keep=1.0 if c == 3 else keep))
    return out


def shrink(s: LayerSpec, **kw) -> LayerSpec:
    """Same recipe at another size (used by tests to get seconds-sized cases)."""
    return replace(s, **kw)
