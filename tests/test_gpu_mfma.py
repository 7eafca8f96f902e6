"""The matrix-core kernel (fp16 storage) against the oracle: every tile shape, forced, on shapes chosen to hit what its
indexing distinguishes -- tiles that run from one image into the next, a ragged last tile, rows capped per tile,
both strides and paddings, widths that allow 4-, 2- and 1-pixel loads and 8-, 4-, 2- and 1-pixel stores, channel and
filter counts that are not multiples of the 16-channel block and the 32-filter operand, a library that leaves taps
unused, unaligned pointers.  The automatic choice for fp16 storage is this kernel, so every other fp16 parity test
runs it as well."""
import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

from gpu_util import TOL, GpuLayer, rel_err

pytestmark = pytest.mark.gpu
M = pc.KERNEL_MFMA


def say(*a):
    print("[case]", *a, flush=True)


def run_forms(layer, x, forms, relu=None):
    ref = layer.oracle(x, relu)
    for t in forms:
        say(layer.spec.name, "x", x.shape, "stride", layer.spec.stride, "pad", layer.spec.pad, "form", t)
        try:
            got = layer.run(x, relu, **t)
        except pc.PconvError as e:
            assert e.code == pc.EUNSUPPORTED, t       # a tile shape or split that cannot take the layer says so
            assert t.get("mfma_shape", 0) != 0 or t.get("channel_splits", 0) != 0, \
                "the automatic choice must find a shape or fall back"
            say("  unsupported")
            continue
        err = rel_err(got, ref)
        assert err <= TOL["f16"], (layer.spec, t, err)


SHAPES = [  # N, C, F, H, W, stride, pad
    (3, 40, 70, 13, 28, 1, 1),      # 4-pixel loads and stores, 13 rows: tiles cross images
    (2, 33, 130, 9, 12, 1, 1),      # C and F ragged against 16 / 32 / 128
    (5, 16, 64, 7, 7, 1, 1),        # odd width: 1-pixel loads and stores; several images per tile
    (33, 24, 40, 7, 7, 1, 1),       # more images than one tile holds
    (2, 20, 33, 14, 14, 1, 1),      # 2-pixel loads and stores
    (2, 31, 13, 15, 18, 2, 1),      # stride 2, odd height
    (3, 8, 8, 16, 16, 2, 0),        # stride 2, no padding
    (1, 7, 9, 5, 130, 1, 0),        # no padding, a row wider than a 128-pixel operand group
    (2, 64, 10, 8, 8, 1, 0),
    (1, 5, 3, 1, 1, 1, 1),          # a single pixel
    (2, 3, 64, 30, 224, 1, 1),      # a first layer at full width: one or two rows per tile
    (2, 48, 96, 20, 56, 2, 1),
]


@pytest.mark.parametrize("case", SHAPES, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}s{c[5]}p{c[6]}" for c in SHAPES])
def test_every_tile_shape(case):
    N, C, F, H, W, stride, pad = case
    spec = L.LayerSpec(cfg=20, idx=SHAPES.index(case), name="mfma", N=N, C=C, F=F, H=H, W=W, stride=stride, pad=pad,
                       dtype="f16", K=8, keep=0.4)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    forms = [dict()] + [dict(kernel=M, mfma_shape=sh) for sh in (1, 2, 3, 4)]
    forms += [dict(kernel=M, mfma_shape=sh, rows=r) for sh in (1, 4) for r in (1, 3)]
    # the channel blocks of every tile split over two or four workgroups (refused where there are fewer blocks)
    forms += [dict(kernel=M, mfma_shape=sh, channel_splits=ks) for sh in (1, 2, 4) for ks in (2, 4)]
    forms += [dict(kernel=M, channel_splits=2), dict(kernel=M, mfma_shape=3, channel_splits=2, slot_walk=1)]
    # ... with the parts added by the second kernel instead of by the last arriver
    forms += [dict(kernel=M, mfma_shape=sh, channel_splits=ks, split_reduce=2) for sh in (1, 2, 3, 4) for ks in (2, 4)]
    run_forms(layer, x, forms)
    run_forms(layer, x, [dict(kernel=M)], relu=True)
    layer.free()


def test_library_that_leaves_taps_unused():
    """Two patterns over taps {0,1,2,3} and {0,1,2,4}: four of the nine taps carry no weight and are skipped."""
    spec = L.LayerSpec(cfg=21, idx=0, name="taps", N=2, C=24, F=40, H=12, W=20, dtype="f16", K=2, keep=0.5,
                       lib_kind="all126", assign="uniform", conn="bernoulli")
    layer = GpuLayer(spec)
    assert sorted(int(m) for m in layer.lib) == [0x00F, 0x017]
    x = L.gen_activations(spec)
    run_forms(layer, x, [dict(kernel=M, mfma_shape=sh) for sh in (0, 1, 2, 3, 4)])
    layer.free()


def test_nothing_kept_and_no_bias():
    spec = L.LayerSpec(cfg=21, idx=1, name="none", N=2, C=16, F=32, H=8, W=8, dtype="f16", K=8, keep=0.0)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    y = layer.run(x, kernel=M)
    assert np.array_equal(y, np.broadcast_to(layer.bias[None, :, None, None], y.shape).astype(np.float16))
    layer.free()
    layer = GpuLayer(L.shrink(spec, keep=0.5, idx=2), use_bias=False)
    run_forms(layer, x, [dict(kernel=M)])
    layer.free()


def test_unaligned_pointers_and_fp32_refusal():
    spec = L.LayerSpec(cfg=21, idx=3, name="shift", N=2, C=20, F=24, H=12, W=16, dtype="f16", K=8, keep=0.5)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    ref = layer.oracle(x)
    for xs, ys in ((1, 0), (0, 1), (3, 5), (2, 4)):
        say("x shifted by", xs, "elements, y by", ys)
        assert rel_err(layer.run(x, x_shift=xs, y_shift=ys, kernel=M), ref) <= TOL["f16"]
    layer.free()
    spec32 = L.shrink(spec, dtype="f32", idx=4)
    layer = GpuLayer(spec32)
    with pytest.raises(pc.PconvError) as e:
        layer.run(L.gen_activations(spec32), kernel=M)
    assert e.value.code == pc.EUNSUPPORTED
    layer.free()


def test_runs_are_bit_reproducible():
    spec = L.LayerSpec(cfg=21, idx=5, name="repro", N=4, C=64, F=128, H=28, W=28, dtype="f16", K=8, keep=0.28)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    first = layer.run(x)
    for _ in range(5):
        assert np.array_equal(layer.run(x).view(np.uint16), first.view(np.uint16))
    layer.free()


def test_split_channel_blocks_are_bit_reproducible_and_match_the_oracle():
    """Small maps with many channels: few tiles, so the channel blocks of a tile go to several workgroups and the one
    that arrives last adds the parts in a fixed order.  200 launches must be bit-identical (the order of arrival
    varies from launch to launch), and the forced and the automatic choice must meet the oracle."""
    spec = L.LayerSpec(cfg=21, idx=6, name="splitk", N=8, C=256, F=192, H=7, W=7, dtype="f16", K=8, keep=0.3)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    ref = layer.oracle(x)
    for t in (dict(kernel=M, mfma_shape=4, channel_splits=4), dict(kernel=M, mfma_shape=2, channel_splits=8),
              dict(kernel=M, channel_splits=16), dict(kernel=M), dict()):
        say("split", t)
        first = layer.run(x, **t)
        assert rel_err(first, ref) <= TOL["f16"], t
        for _ in range(40):
            assert np.array_equal(layer.run(x, canary=False, **t).view(np.uint16), first.view(np.uint16)), t
    layer.free()


def test_parts_added_by_a_second_kernel_equal_the_last_arrivers_sum_bit_for_bit():
    """Both ways of adding the parts of a split tile add them in the order of the parts, starting from the part that
    started from the bias: equal outputs bit for bit, with and without ReLU, channel-major and channel-minor; and the
    oracle is met."""
    import torch
    spec = L.LayerSpec(cfg=21, idx=7, name="splitk2", N=9, C=256, F=136, H=7, W=14, dtype="f16", K=8, keep=0.3)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    for relu in (False, True):
        ref = layer.oracle(x, relu)
        for sh, ks in ((1, 2), (2, 8), (3, 4), (4, 16), (4, 3)):
            say("second pass", sh, ks, relu)
            a = layer.run(x, relu, kernel=M, mfma_shape=sh, channel_splits=ks, split_reduce=1)
            b = layer.run(x, relu, kernel=M, mfma_shape=sh, channel_splits=ks, split_reduce=2)
            assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), (sh, ks, relu)
            assert rel_err(b, ref) <= TOL["f16"]
    # channel-minor outputs of the second kernel
    s = spec
    dx = torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1))).cuda()
    dy = torch.full((s.N, s.Ho, s.Wo, s.F), -7.0, dtype=torch.float16, device="cuda")
    pc.conv3x3_tuned(dx, dy, layer.packed, layer.d_bias, s.N, s.H, s.W, 1, 1, pc.FLAG_NHWC | pc.FLAG_RELU,
                     torch.cuda.current_stream().cuda_stream, kernel=M, mfma_shape=4, channel_splits=4, split_reduce=2)
    torch.cuda.synchronize()
    assert rel_err(dy.cpu().numpy().transpose(0, 3, 1, 2), layer.oracle(x, True)) <= TOL["f16"]
    with pytest.raises(pc.PconvError):
        layer.run(x, kernel=M, split_reduce=3)
    layer.free()


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
def test_dense_baseline_on_the_matrix_cores_and_direct(stride, pad):
    import torch
    spec = L.LayerSpec(cfg=22, idx=stride * 2 + pad, name="dense16", N=3, C=40, F=72, H=14, W=20, stride=stride,
                       pad=pad, dtype="f16")
    w, x, b = L.gen_weights(spec), L.gen_activations(spec), L.gen_bias(spec)
    dx, dw, db = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
    ref = oracle.conv3x3(x, w, b, stride, pad, relu=True)
    for flags in (pc.FLAG_RELU, pc.FLAG_RELU | pc.FLAG_DENSE_DIRECT):
        say("dense fp16", stride, pad, "flags", flags)
        dy = torch.full((3, 72, spec.Ho, spec.Wo), -7.0, dtype=torch.float16, device="cuda")
        pc.dense_conv3x3(dx, dy, dw, db, pc.F16, 3, 40, 72, 14, 20, stride, pad, flags,
                         torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert rel_err(dy.cpu().numpy(), ref) <= TOL["f16"]
