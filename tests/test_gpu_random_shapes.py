"""GPU parity on seeded random shapes: every kernel form the library has, on layer sizes drawn at random (batch, channel
and filter counts around the chunk and workgroup sizes, heights and widths around the tile sizes, both strides, pads
and storage types, random tunings), element by element against the CPU oracle.  A tuning the library has no kernel
for must say so (PCONV_EUNSUPPORTED) and nothing else.  Every case is printed, flushed, before it touches the GPU."""
import random

import pytest

import paper_2001_07710_amd as pc
from workloads import layers as L

from gpu_util import TOL, GpuLayer, rel_err

pytestmark = pytest.mark.gpu

Q, T, G = pc.KERNEL_QUAD, pc.KERNEL_TILED, pc.KERNEL_GENERIC


@pytest.fixture(scope="module", autouse=True)
def _built():
    pc.ensure_built()


def _run_cases(layer, x, tunings, rnd):
    ok = 0
    for t in tunings:
        relu = rnd.choice([False, True])
        print("[case]", layer.spec, "relu", relu, "tuning", t, flush=True)
        try:
            got = layer.run(x, relu, **t)
        except pc.PconvError as e:
            assert e.code == pc.EUNSUPPORTED, (layer.spec, t, e)
            continue
        err = rel_err(got, layer.oracle(x, relu))
        assert err <= TOL[layer.spec.dtype], (layer.spec, t, relu, err)
        ok += 1
    return ok


@pytest.mark.parametrize("seed", [3, 4])
def test_four_column_kernel_forms_on_random_shapes(seed):
    """One workgroup per tile (with and without channel splits) and the walking forms, widths that are multiples of 4."""
    rnd = random.Random(seed)
    ok = 0
    for it in range(30):
        N = rnd.choice([1, 2, 3, 5, 9, 17, 40, 77])
        C = rnd.choice([1, 3, 8, 16, 17, 33, 48, 70])
        F = rnd.choice([1, 5, 16, 17, 32, 40, 70])
        H, W = rnd.randint(3, 30), 4 * rnd.randint(1, 16)
        keep = rnd.choice([0.1, 0.3, 0.6, 1.0])
        if N * C * F * H * W * 4 * keep > 3e8:
            continue
        spec = L.LayerSpec(cfg=30, idx=100 * seed + it, name="random4", N=N, C=C, F=F, H=H, W=W, pad=rnd.choice([0, 1, 1]),
                           dtype=rnd.choice(["f32", "f16"]), K=8, keep=keep)
        layer = GpuLayer(spec)
        x = L.gen_activations(spec)
        ok += _run_cases(layer, x, [
            dict(kernel=Q, filters_per_wave=rnd.choice([1, 2]), slot_walk=2, channel_order=rnd.choice([0, 1, 2])),
            dict(kernel=Q, filters_per_wave=rnd.choice([1, 2]), channel_splits=rnd.choice([0, 1, 2, 3])),
            dict()], rnd)
        layer.free()
    assert ok >= 40          # (the draw must not degenerate into unsupported cases only)


@pytest.mark.parametrize("seed", [5, 6])
def test_one_column_kernel_forms_on_random_shapes(seed):
    """Every tiling, chunk-buffer count, channel order and split count, both strides and pads, any width."""
    rnd = random.Random(seed)
    ok = 0
    for it in range(30):
        N = rnd.choice([1, 2, 3, 5, 9, 33])
        C = rnd.choice([1, 3, 8, 16, 17, 33, 48, 70, 130])
        F = rnd.choice([1, 5, 16, 17, 32, 40, 70])
        H, W = rnd.randint(1, 34), rnd.randint(1, 70)
        stride, pad = rnd.choice([1, 1, 2]), rnd.choice([0, 1, 1])
        keep = rnd.choice([0.05, 0.3, 0.6, 1.0])
        if H + 2 * pad < 3 or W + 2 * pad < 3 or N * C * F * H * W * 4 * keep > 3e8:
            continue
        spec = L.LayerSpec(cfg=31, idx=100 * seed + it, name="random1", N=N, C=C, F=F, H=H, W=W, stride=stride, pad=pad,
                           dtype=rnd.choice(["f32", "f16"]), K=8, keep=keep)
        layer = GpuLayer(spec)
        x = L.gen_activations(spec)
        tunings = [dict(), dict(kernel=G)]
        for _ in range(3):
            tunings.append(dict(kernel=T, rows=7, waves=rnd.choice([4, 8, 16]), channels_per_wave=rnd.choice([1, 2, 4]),
                                filters_per_wave=rnd.choice([1, 2]), channel_splits=rnd.choice([0, 1, 2, 3]),
                                buffers=rnd.choice([0, 1, 2]), channel_order=rnd.choice([0, 1, 2])))
        ok += _run_cases(layer, x, tunings, rnd)
        layer.free()
    assert ok >= 50


@pytest.mark.parametrize("seed", [7, 8])
def test_matrix_core_kernel_forms_on_random_shapes(seed):
    """Every tile shape, with and without channel splits, row caps and one workgroup per tile; both strides and pads,
    any width (all four piece widths of the loads and of the stores), filter and channel counts around the tile and
    block sizes, batches that make tiles run from one image into the next.  fp16 storage only."""
    M = pc.KERNEL_MFMA
    rnd = random.Random(seed)
    ok = 0
    for it in range(36):
        N = rnd.choice([1, 2, 3, 5, 9, 33, 70])
        C = rnd.choice([1, 3, 8, 16, 17, 33, 48, 70, 130])
        F = rnd.choice([1, 5, 16, 33, 64, 65, 130])
        H, W = rnd.randint(1, 34), rnd.choice([rnd.randint(1, 70), 8 * rnd.randint(1, 8), 4 * rnd.randint(1, 16)])
        stride, pad = rnd.choice([1, 1, 2]), rnd.choice([0, 1, 1])
        keep = rnd.choice([0.05, 0.3, 0.6, 1.0])
        if H + 2 * pad < 3 or W + 2 * pad < 3 or N * C * F * H * W > 6e7:
            continue
        spec = L.LayerSpec(cfg=32, idx=100 * seed + it, name="randomM", N=N, C=C, F=F, H=H, W=W, stride=stride, pad=pad,
                           dtype="f16", K=rnd.choice([4, 8, 12]), keep=keep)
        layer = GpuLayer(spec)
        x = L.gen_activations(spec)
        tunings = [dict(), dict(kernel=M)]
        for _ in range(4):
            tunings.append(dict(kernel=M, mfma_shape=rnd.choice([1, 2, 3, 4]), channel_splits=rnd.choice([0, 0, 1, 2, 4]),
                                rows=rnd.choice([0, 0, 1, 3]), slot_walk=rnd.choice([0, 0, 1])))
        ok += _run_cases(layer, x, tunings, rnd)
        layer.free()
    assert ok >= 80
