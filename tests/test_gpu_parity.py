"""GPU parity: libpconv (through its C ABI) against the CPU oracle, element by element, on the same seeded bytes.

Tolerances (max relative error, see gpu_util.rel_err): 1e-4 for fp32, 2e-3 for fp16 storage with fp32 accumulation.
Pattern assignment, connectivity selection and packing are compared bit for bit (gpu_util.sparsity and
test_host_logic).  Every test prints the case it is about to run, flushed, before touching the GPU.
"""
import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L
from workloads import rng

from gpu_util import TOL, GpuLayer, rel_err

pytestmark = pytest.mark.gpu

T, G = pc.KERNEL_TILED, pc.KERNEL_GENERIC
TILED_TUNINGS = [dict(kernel=T, rows=7, filters_per_wave=nf, waves=w, channels_per_wave=cpw)
                 for nf, w, cpw in [(1, 8, 2), (2, 8, 2), (1, 16, 1), (1, 4, 4), (2, 16, 1), (1, 8, 4),
                                    (2, 16, 2), (1, 16, 2)]]
# two chunk buffers in LDS (one barrier per chunk)
DB_TUNINGS = [dict(kernel=T, rows=7, filters_per_wave=nf, waves=w, channels_per_wave=cpw, buffers=2)
              for nf, w, cpw in [(2, 16, 1), (1, 16, 1), (1, 8, 2), (2, 8, 2)]]
ALL_TUNINGS = [dict(kernel=G)] + TILED_TUNINGS + DB_TUNINGS + [dict()]


def say(*a):
    print("[case]", *a, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _built():
    pc.ensure_built()


def check(layer: GpuLayer, x, tunings, relu=None, tol=None):
    ref = layer.oracle(x, relu)
    tol = TOL[layer.spec.dtype] if tol is None else tol
    for t in tunings:
        say(layer.spec.name, layer.spec.dtype, "x", x.shape, "tuning", t)
        got = layer.run(x, relu, **t)
        assert got.shape == ref.shape
        err = rel_err(got, ref)
        assert err <= tol, (layer.spec, t, err)
    return ref


# ------------------------------------------------------------------------------------------------------------------
# config 0: the small case, every kernel variant
# ------------------------------------------------------------------------------------------------------------------

def test_config0_every_kernel_variant():
    spec = L.config0()
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    assert abs(layer.mask.mean() - 0.5) < 0.1 and set(np.unique(layer.pid)) == {0, 1, 2, 3}
    check(layer, x, ALL_TUNINGS)
    check(layer, x, [dict(), dict(kernel=G)], relu=True)
    layer.free()


def test_every_one_of_the_126_patterns():
    spec = L.LayerSpec(cfg=9, idx=0, name="all126", N=2, C=126, F=20, H=9, W=12, K=126, keep=0.6, lib_kind="all126",
                       assign="uniform", conn="bernoulli")
    layer = GpuLayer(spec)
    assert len(np.unique(layer.pid[layer.mask != 0])) == 126
    check(layer, L.gen_activations(spec), [dict(), dict(kernel=G), TILED_TUNINGS[1], TILED_TUNINGS[6], DB_TUNINGS[0]])
    layer.free()


# ------------------------------------------------------------------------------------------------------------------
# ragged shapes, both pads, both strides, both storage types, several images
# ------------------------------------------------------------------------------------------------------------------

RAGGED = [  # N, C, F, H, W, stride, pad
    (1, 5, 3, 1, 1, 1, 1), (2, 33, 17, 9, 11, 1, 1), (3, 40, 20, 13, 70, 1, 1), (1, 7, 9, 5, 130, 1, 0),
    (2, 64, 10, 8, 8, 1, 0), (2, 16, 8, 3, 3, 1, 0), (2, 31, 13, 15, 17, 2, 1), (1, 8, 8, 8, 8, 2, 0),
    (5, 12, 6, 7, 7, 1, 1), (2, 3, 64, 30, 62, 1, 1), (1, 96, 130, 6, 63, 1, 1), (2, 20, 5, 16, 9, 2, 1),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("case", RAGGED, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}s{c[5]}p{c[6]}" for c in RAGGED])
def test_ragged_shapes(case, dtype):
    N, C, F, H, W, stride, pad = case
    spec = L.LayerSpec(cfg=10, idx=RAGGED.index(case), name="ragged", N=N, C=C, F=F, H=H, W=W, stride=stride, pad=pad,
                       dtype=dtype, K=8, keep=0.4)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    # stride 2 reaches the tiled kernels through the parity-plane form of the layer
    tunings = [dict(), dict(kernel=G), TILED_TUNINGS[0], TILED_TUNINGS[3], TILED_TUNINGS[6], TILED_TUNINGS[7],
               DB_TUNINGS[0], DB_TUNINGS[2]]
    check(layer, x, tunings)
    check(layer, x, [dict()], relu=True)
    layer.free()


def test_no_bias_negative_inputs_and_empty_filters():
    spec = L.LayerSpec(cfg=11, idx=0, name="nobias", N=2, C=48, F=24, H=14, W=14, K=8, keep=0.1)
    w = L.gen_weights(spec)
    layer = GpuLayer(spec, w=w, use_bias=False)
    assert (layer.mask.sum(axis=1) == 0).any() or layer.mask.sum() < 0.11 * layer.mask.size
    x = (rng.normal(77, 2 * 48 * 14 * 14).astype(np.float32) * 3).reshape(2, 48, 14, 14)   # signed, not rectified
    check(layer, x, [dict(), dict(kernel=G), TILED_TUNINGS[1]])
    layer.free()
    # a layer with nothing kept computes the bias alone
    spec0 = L.shrink(spec, keep=0.0, idx=1)
    layer0 = GpuLayer(spec0)
    assert layer0.mask.sum() == 0
    y = layer0.run(x)
    assert np.array_equal(y, np.broadcast_to(layer0.bias[None, :, None, None], y.shape))
    layer0.free()
    # ... with every kernel (the quad kernel needs a width that is a multiple of four)
    spec1 = L.LayerSpec(cfg=11, idx=2, name="nothing", N=3, C=40, F=24, H=10, W=16, K=8, keep=0.0)
    layer1 = GpuLayer(spec1)
    assert layer1.mask.sum() == 0
    x1 = L.gen_activations(spec1)
    for t in (dict(kernel=pc.KERNEL_QUAD), dict(kernel=pc.KERNEL_QUAD, filters_per_wave=1, channel_splits=2),
              dict(kernel=T, channel_splits=2), dict(kernel=G)):
        say(spec1.name, t)
        y1 = layer1.run(x1, **t)
        assert np.array_equal(y1, np.broadcast_to(layer1.bias[None, :, None, None], y1.shape)), t
    layer1.free()


def test_batch_zero_is_a_no_op_and_runs_are_deterministic():
    spec = L.shrink(L.config1(), C=64, F=32, H=28, W=28)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    a = layer.run(x)
    b = layer.run(x)
    assert a.tobytes() == b.tobytes()
    # also with channels split over workgroups (the partial sums are added in a fixed order), in both kernels
    for t in (dict(kernel=T, channel_splits=2), dict(kernel=pc.KERNEL_QUAD, channel_splits=2)):
        assert layer.run(x, **t).tobytes() == layer.run(x, **t).tobytes(), t
    import torch
    dummy = torch.zeros(4, device="cuda")
    pc.conv3x3(dummy, dummy, layer.packed, None, 0, 28, 28)
    layer.free()


def test_channel_splits_agree_and_leave_the_workspace_reusable():
    """Input channels of a tile split over 1..8 workgroups: every split count matches the oracle, the same launch
    repeated gives the same bytes (fixed summation order, counters back at zero), and a larger shape after a smaller
    one (workspace grows) and a smaller one after it (workspace reused) are still right."""
    spec = L.shrink(L.config1(), C=160, F=72, H=20, W=33)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    ref = layer.oracle(x)
    for nf, wv, cpw, nbuf in [(2, 16, 2, 1), (1, 16, 2, 1), (1, 8, 4, 1), (2, 8, 2, 1), (1, 8, 2, 1), (2, 16, 1, 2),
                              (1, 8, 2, 2)]:
        nch = -(-spec.C // (wv * cpw))
        for ks in sorted({1, 2, 3, nch}):
            t = dict(kernel=T, rows=7, filters_per_wave=nf, waves=wv, channels_per_wave=cpw, channel_splits=ks,
                     buffers=nbuf)
            say("splits", t)
            a = layer.run(x, **t)
            assert rel_err(a, ref) <= TOL[spec.dtype], t
            b = layer.run(x, **t)
            assert a.tobytes() == b.tobytes(), t
        with pytest.raises(pc.PconvError):
            layer.run(x, kernel=T, rows=7, filters_per_wave=nf, waves=wv, channels_per_wave=cpw,
                      channel_splits=nch + 1, buffers=nbuf)
    # a larger problem on the same handle, then the first one again; ReLU and fp16 output through the split path
    big = L.gen_activations(L.shrink(spec, N=3))
    t = dict(kernel=T, rows=7, filters_per_wave=2, waves=16, channels_per_wave=2, channel_splits=4)
    assert rel_err(layer.run(big, **t), layer.oracle(big)) <= TOL[spec.dtype]
    assert rel_err(layer.run(x, relu=True, **t), layer.oracle(x, True)) <= TOL[spec.dtype]
    layer.free()
    spec16 = L.shrink(spec, dtype="f16", idx=3)
    layer16 = GpuLayer(spec16)
    x16 = L.gen_activations(spec16)
    check(layer16, x16, [dict(), dict(t, channel_splits=2), dict(t, channel_splits=5)])
    layer16.free()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("pad", [0, 1])
def test_stride2_both_staging_paths(pad, dtype):
    """Stride 2 with even H and W reads the parity planes straight from the input (paired staging); with the balanced
    channel order, or odd sizes, a separate pass splits the input first.  Both against the oracle, several images,
    more channels than one chunk, a filter count that leaves waves without a filter."""
    spec = L.LayerSpec(cfg=14, idx=pad, name="s2paths", N=3, C=20, F=40, H=18, W=26, stride=2, pad=pad, dtype=dtype,
                       K=8, keep=0.45)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    paired = [dict(), dict(kernel=T, rows=7, filters_per_wave=2, waves=16, channels_per_wave=2),
              dict(kernel=T, rows=7, filters_per_wave=1, waves=16, channels_per_wave=2, channel_splits=2)]
    split_first = [dict(kernel=T, rows=7, filters_per_wave=2, waves=16, channels_per_wave=2,
                        channel_order=pc.ORDER_BALANCED),
                   dict(kernel=T, rows=7, filters_per_wave=1, waves=8, channels_per_wave=4)]
    check(layer, x, paired + split_first + [dict(kernel=G)])
    check(layer, x, [dict()], relu=True)
    layer.free()


QUAD_SHAPES = [  # N, C, F, H, W, pad
    (1, 16, 16, 32, 32, 1), (3, 40, 20, 13, 68, 1), (2, 20, 33, 9, 12, 0), (1, 5, 3, 4, 4, 1), (5, 12, 6, 7, 8, 1),
    (2, 33, 17, 6, 256, 1), (1, 64, 40, 56, 56, 1), (9, 24, 16, 5, 4, 1), (2, 17, 70, 11, 28, 0),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("case", QUAD_SHAPES, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}p{c[5]}" for c in QUAD_SHAPES])
def test_quad_kernel(case, dtype):
    """The kernel with four columns per lane (W a multiple of four, unit stride): one and two filters per wave,
    ragged row blocks, waves that span images, channel counts that are not a multiple of the chunk, ReLU."""
    N, C, F, H, W, pad = case
    spec = L.LayerSpec(cfg=15, idx=QUAD_SHAPES.index(case), name="quad", N=N, C=C, F=F, H=H, W=W, stride=1, pad=pad,
                       dtype=dtype, K=8, keep=0.4)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    Q = pc.KERNEL_QUAD
    check(layer, x, [dict(kernel=Q, filters_per_wave=nf, channel_order=o) for nf in (1, 2)
                     for o in (pc.ORDER_PLAIN, pc.ORDER_BALANCED)])
    # channels split over several workgroups per tile (more splits than chunks are cut down to the chunks)
    check(layer, x, [dict(kernel=Q, filters_per_wave=nf, channel_splits=ks) for nf in (1, 2) for ks in (2, 3, 8)])
    check(layer, x, [dict(kernel=Q, channel_splits=2)], relu=True)
    check(layer, x, [dict(kernel=Q)], relu=True)
    layer.free()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_quad_kernel_with_an_output_pointer_that_is_not_16_byte_aligned(dtype):
    """The 128-bit stores of the quad kernel need an aligned output; otherwise it stores element by element."""
    spec = L.LayerSpec(cfg=15, idx=50, name="quadshift", N=2, C=24, F=20, H=10, W=16, stride=1, pad=1, dtype=dtype,
                       K=8, keep=0.5)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    ref = layer.oracle(x)
    for shift in (1, 2, 3):
        for t in (dict(kernel=pc.KERNEL_QUAD), dict(kernel=pc.KERNEL_QUAD, channel_splits=2)):
            say(spec.name, dtype, "shift", shift, t)
            assert rel_err(layer.run(x, y_shift=shift, **t), ref) <= TOL[dtype]
    layer.free()


def test_an_input_pointer_aligned_to_one_element_only():
    """fp16 activations at an odd element offset: the kernels that load two or four elements at a time are not
    chosen (and refuse when asked for), the result is the same."""
    for stride, N in ((1, 40), (2, 3)):
        spec = L.LayerSpec(cfg=15, idx=60 + stride, name="xshift", N=N, C=20, F=36, H=12, W=16, stride=stride, pad=1,
                           dtype="f16", K=8, keep=0.5)
        layer = GpuLayer(spec)
        x = L.gen_activations(spec)
        ref = layer.oracle(x)
        say(spec.name, "stride", stride, "x shifted by one element")
        assert rel_err(layer.run(x, x_shift=1), ref) <= TOL["f16"]
        assert rel_err(layer.run(x, x_shift=1, kernel=T), ref) <= TOL["f16"]
        if stride == 1:
            with pytest.raises(pc.PconvError) as ei:
                layer.run(x, x_shift=1, kernel=pc.KERNEL_QUAD)
            assert ei.value.code == pc.EUNSUPPORTED
        layer.free()


def test_quad_kernel_refuses_what_it_cannot_do():
    spec = L.LayerSpec(cfg=15, idx=99, name="quadno", N=1, C=8, F=8, H=8, W=10, K=8, keep=0.5)
    layer = GpuLayer(spec)
    with pytest.raises(pc.PconvError) as ei:
        layer.run(L.gen_activations(spec), kernel=pc.KERNEL_QUAD)
    assert ei.value.code == pc.EUNSUPPORTED
    layer.free()


WALK_SHAPES = [  # N, C, F, H, W: one chunk of channels (C <= 16), pad 1
    (3, 3, 64, 32, 32), (2, 3, 20, 9, 12), (5, 16, 16, 7, 8), (70, 1, 5, 6, 4), (4, 12, 33, 13, 68),
    (2, 3, 64, 30, 256), (9, 5, 3, 5, 4),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("case", WALK_SHAPES, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}" for c in WALK_SHAPES])
def test_quad_kernel_that_walks_over_the_tiles(case, dtype):
    """First-layer shapes through the workgroups that keep their filters and walk over the output tiles: tile counts
    that are and are not a multiple of the number of workgroups, fewer tiles than workgroups, waves without a filter,
    a ragged last row block, several images per wave; against the oracle and against one workgroup per tile."""
    N, C, F, H, W = case
    spec = L.LayerSpec(cfg=17, idx=WALK_SHAPES.index(case), name="walk", N=N, C=C, F=F, H=H, W=W, pad=1, dtype=dtype,
                       K=8, keep=1.0 if C <= 3 else 0.6)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    for nf in (1, 2) if dtype == "f16" else (1,):      # two filters per wave: fp16 storage only
        walk = dict(kernel=pc.KERNEL_QUAD, filters_per_wave=nf, slot_walk=2)
        ref = check(layer, x, [walk, dict(walk, channel_order=pc.ORDER_PLAIN)])
        check(layer, x, [walk], relu=True)
        got_walk = layer.run(x, **walk)
        got_tile = layer.run(x, kernel=pc.KERNEL_QUAD, filters_per_wave=nf, slot_walk=1, channel_splits=1)
        assert np.array_equal(got_walk, got_tile)       # same sums in the same order
        assert got_walk.shape == ref.shape
    layer.free()


STREAM_SHAPES = [  # N, C, F, H, W: several chunks of channels, pad 1
    (3, 40, 64, 32, 32), (2, 20, 20, 9, 12), (5, 33, 16, 7, 8), (70, 17, 5, 6, 4), (4, 64, 33, 13, 68), (9, 100, 40, 5, 4),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("case", STREAM_SHAPES, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}" for c in STREAM_SHAPES])
def test_quad_kernel_that_walks_over_tiles_of_several_chunks(case, dtype):
    """Layers of more than one chunk through the workgroups that run the chunks of all their tiles as one sequence:
    against the oracle, and bit for bit against one workgroup per tile; a ragged last chunk, tile counts that are
    not a multiple of the number of workgroups, fewer tiles than workgroups, waves without a filter."""
    N, C, F, H, W = case
    spec = L.LayerSpec(cfg=18, idx=STREAM_SHAPES.index(case), name="stream", N=N, C=C, F=F, H=H, W=W, pad=1, dtype=dtype,
                       K=8, keep=0.5)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    for nf in (1, 2) if dtype == "f16" else (1,):      # two filters per wave: fp16 storage only
        walk = dict(kernel=pc.KERNEL_QUAD, filters_per_wave=nf, slot_walk=2)
        check(layer, x, [walk, dict(walk, channel_order=pc.ORDER_PLAIN)])
        check(layer, x, [walk], relu=True)
        for order in (pc.ORDER_PLAIN, pc.ORDER_BALANCED):
            got_walk = layer.run(x, channel_order=order, **walk)
            got_tile = layer.run(x, kernel=pc.KERNEL_QUAD, filters_per_wave=nf, slot_walk=1, channel_order=order,
                                 channel_splits=1)
            assert np.array_equal(got_walk, got_tile)       # same sums in the same order
    layer.free()


def test_walking_kernels_without_a_bias_and_with_empty_filters():
    """The walking forms with no bias vector, and with filters that keep nothing (their outputs are zero, or the
    bias), for one chunk and for several."""
    for C, dtype in ((8, "f16"), (40, "f16"), (40, "f32")):
        spec = L.LayerSpec(cfg=19, idx=C, name="walkedge", N=6, C=C, F=24, H=12, W=16, pad=1, dtype=dtype, K=8, keep=0.5)
        w = L.gen_weights(spec)
        layer = GpuLayer(spec, w=w, use_bias=False)
        x = L.gen_activations(spec)
        for nf in (1, 2) if dtype == "f16" else (1,):
            check(layer, x, [dict(kernel=pc.KERNEL_QUAD, filters_per_wave=nf, slot_walk=2)])
        layer.free()
        layer = GpuLayer(spec, w=w)
        layer.mask[::3, :] = 0                     # every third filter keeps no kernel at all
        layer.packed.free()
        layer.packed = pc.pack(layer.w, layer.lib, layer.pid, layer.mask)
        layer.wm = oracle.mask_weights(layer.w, layer.pid, layer.mask, layer.lib)
        for nf in (1, 2) if dtype == "f16" else (1,):
            t = dict(kernel=pc.KERNEL_QUAD, filters_per_wave=nf, slot_walk=2)
            check(layer, x, [t])
            got = layer.run(x, **t)[:, ::3]
            assert np.array_equal(got, np.broadcast_to(layer.bias[None, ::3, None, None], got.shape).astype(got.dtype))
        layer.free()


def test_walking_is_refused_where_it_does_not_apply():
    for kw, shape in [(dict(filters_per_wave=2), dict(dtype="f32")), (dict(filters_per_wave=1, channel_splits=2), dict(C=40)),
                      (dict(filters_per_wave=1), dict(pad=0))]:
        spec = L.LayerSpec(**{**dict(cfg=17, idx=50, name="walkno", N=2, C=8, F=16, H=8, W=8, K=8, keep=0.5), **shape})
        layer = GpuLayer(spec)
        with pytest.raises(pc.PconvError) as ei:
            layer.run(L.gen_activations(spec), kernel=pc.KERNEL_QUAD, slot_walk=2, **kw)
        assert ei.value.code == pc.EUNSUPPORTED, (kw, shape)
        layer.free()
    # a number of filters per wave for which the four-column kernel is not built, with and without walking
    for dtype in ("f32", "f16"):
        spec = L.LayerSpec(cfg=17, idx=52, name="quadnf", N=2, C=8, F=48, H=8, W=8, K=8, keep=0.5, dtype=dtype)
        layer = GpuLayer(spec)
        for walk in (0, 1, 2):
            with pytest.raises(pc.PconvError) as ei:
                layer.run(L.gen_activations(spec), kernel=pc.KERNEL_QUAD, filters_per_wave=3, slot_walk=walk)
            assert ei.value.code == pc.EUNSUPPORTED, (dtype, walk)
        layer.free()
    # an output pointer that is not 16-byte aligned
    spec = L.LayerSpec(cfg=17, idx=51, name="walkno", N=2, C=8, F=16, H=8, W=8, K=8, keep=0.5)
    layer = GpuLayer(spec)
    with pytest.raises(pc.PconvError) as ei:
        layer.run(L.gen_activations(spec), y_shift=1, kernel=pc.KERNEL_QUAD, filters_per_wave=1, slot_walk=2)
    assert ei.value.code == pc.EUNSUPPORTED
    layer.free()


def test_hip_graph_replays_match_eager_launches():
    """Two layers (the first splits its channels over workgroups, the second runs at stride 2 through the parity
    form) and a max-pool, captured into one HIP graph: every replay, with eager work and synchronisations in between
    and with fresh input values, gives the bytes of the eager launches."""
    import torch
    s1 = L.shrink(L.config1(), C=64, F=32, H=28, W=28, relu=True)
    s2 = L.LayerSpec(cfg=13, idx=0, name="g2", N=1, C=32, F=24, H=14, W=14, stride=2, pad=1, K=8, keep=0.4)
    l1, l2 = GpuLayer(s1), GpuLayer(s2)
    x = torch.from_numpy(L.gen_activations(s1)).cuda()
    y1 = torch.empty((1, 32, 28, 28), device="cuda")
    p1 = torch.empty((1, 32, 14, 14), device="cuda")
    y2 = torch.empty((1, 24, 7, 7), device="cuda")

    def run(st):
        pc.conv3x3(x, y1, l1.packed, l1.d_bias, 1, 28, 28, 1, 1, pc.FLAG_RELU, st)
        pc.maxpool2x2(y1, p1, pc.F32, 1, 32, 28, 28, st)
        pc.conv3x3(p1, y2, l2.packed, l2.d_bias, 1, 14, 14, 2, 1, 0, st)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run(side.cuda_stream)            # allocates workspaces and the parity form outside the capture
        side.synchronize()
        eager = y2.clone()
        ref = l2.oracle(oracle.maxpool2x2(l1.oracle(x.cpu().numpy(), True)).astype(np.float32))
        assert rel_err(eager.cpu().numpy(), ref) <= 2 * TOL["f32"]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            run(side.cuda_stream)
        for rep in range(4):
            say("graph replay", rep)
            if rep == 2:                 # new input values: the graph reads the same buffers
                x.mul_(0.5)
                run(side.cuda_stream)
                side.synchronize()
                eager = y2.clone()
            y2.fill_(-1.0)
            torch.cuda.synchronize()
            g.replay()
            side.synchronize()
            assert torch.equal(y2, eager), rep
    l1.free()
    l2.free()


# ------------------------------------------------------------------------------------------------------------------
# config 1: VGG-16 conv3_x-shaped layer at full size (the benchmark workload)
# ------------------------------------------------------------------------------------------------------------------

def test_config1_full_size():
    spec = L.config1()
    layer = GpuLayer(spec)
    assert layer.packed.n_kept == 18350
    x = L.gen_activations(spec)
    ref = check(layer, x, [dict(), dict(kernel=G)] + TILED_TUNINGS[:7] + DB_TUNINGS +
                [dict(kernel=pc.KERNEL_QUAD, filters_per_wave=1), dict(kernel=pc.KERNEL_QUAD, filters_per_wave=2)])
    # invariant on the GPU side as well: a removed kernel contributes nothing
    f, c = np.argwhere(layer.mask == 0)[0]
    w2 = layer.w.copy()
    w2[f, c] += 100.0
    layer2 = GpuLayer(spec, w=w2)
    if np.array_equal(layer2.mask, layer.mask) and np.array_equal(layer2.pid[layer.mask != 0], layer.pid[layer.mask != 0]):
        assert layer2.run(x).tobytes() == layer.run(x).tobytes()
    layer2.free()
    layer.free()
    assert np.isfinite(ref).all()


# ------------------------------------------------------------------------------------------------------------------
# config 2: the 13 VGG-16 layers in sequence, ReLU fused, 2x2 max-pool between stages
# ------------------------------------------------------------------------------------------------------------------

def test_config2_vgg16_chain():
    import torch
    specs = L.config2()
    layers = [GpuLayer(s) for s in specs]
    assert [l.packed.n_kept for l in layers] == [192, 1434, 2867, 5734, 9175, 18350, 18350, 26214] + [52429] * 5
    x = L.gen_activations(specs[0])
    # oracle chain; every layer of the GPU path is also checked on the oracle's own input for that layer
    xo = x
    for s, layer in zip(specs, layers):
        say("chain layer", s.name, xo.shape)
        yo = layer.oracle(xo).astype(np.float32)
        got = layer.run(xo)
        assert rel_err(got, yo) <= TOL["f32"], s.name
        xo = oracle.maxpool2x2(yo) if s.pool_after else yo
    # the GPU chain end to end (its own activations all the way): rounding differences compound over 13 layers, so
    # the end result is held to 13x the single-layer tolerance
    st = torch.cuda.current_stream().cuda_stream
    cur = torch.from_numpy(x).cuda()
    for s, layer in zip(specs, layers):
        y = torch.empty((1, s.F, s.Ho, s.Wo), dtype=torch.float32, device="cuda")
        pc.conv3x3(cur, y, layer.packed, layer.d_bias, 1, s.H, s.W, 1, 1, pc.FLAG_RELU, st)
        if s.pool_after:
            z = torch.empty((1, s.F, s.Ho // 2, s.Wo // 2), dtype=torch.float32, device="cuda")
            pc.maxpool2x2(y, z, pc.F32, 1, s.F, s.Ho, s.Wo, st)
            y = z
        cur = y
    torch.cuda.synchronize()
    assert tuple(cur.shape) == (1, 512, 7, 7) and xo.shape == (1, 512, 7, 7)
    assert rel_err(cur.cpu().numpy(), xo) <= 13 * TOL["f32"]
    for l in layers:
        l.free()


def test_channel_split_repeats_bit_for_bit_300_times():
    """The channel split of both vector kernels orders its partial sums without a fence (device-scope stores, a wait
    for them, a workgroup barrier, one relaxed atomic, device-scope loads by the last arriver, sums in split order).
    Arrival order changes from launch to launch; 300 launches of each must give the bits of the first, on a layer
    whose automatic choice splits (config 1) and on the four-column kernel with a forced split."""
    import torch
    spec = L.config1()
    layer = GpuLayer(spec)
    dx = torch.from_numpy(L.gen_activations(spec)).cuda()
    st = torch.cuda.current_stream().cuda_stream
    for t in (dict(kernel=T), dict(kernel=T, rows=7, filters_per_wave=2, waves=16, channels_per_wave=2, channel_splits=4),
              dict(kernel=pc.KERNEL_QUAD, filters_per_wave=1, channel_splits=4),
              dict(kernel=pc.KERNEL_QUAD, filters_per_wave=2, channel_splits=2)):
        say("300 launches", t)
        first = None
        for it in range(300):
            dy = torch.empty((1, spec.F, spec.Ho, spec.Wo), dtype=torch.float32, device="cuda")
            pc.conv3x3_tuned(dx, dy, layer.packed, layer.d_bias, 1, spec.H, spec.W, 1, 1, 0, st, **t)
            if first is None:
                first = dy
                torch.cuda.synchronize()
                assert rel_err(first.cpu().numpy(), layer.oracle(dx.cpu().numpy())) <= TOL["f32"]
            elif it % 25 == 24 or it == 299:
                assert bool((dy == first).all()), (t, it)      # (stops at the first block of launches that differs)
            else:
                first_ok = dy                                   # keep the launches back to back between checks
    layer.free()


# ------------------------------------------------------------------------------------------------------------------
# config 3: ResNet-50 bottleneck 3x3 shapes, fp16 storage, batch 1 and batch 32
# ------------------------------------------------------------------------------------------------------------------

def sampled_coords(seed, N, F, Ho, Wo, npts=65536):
    r = rng.raw_u64(seed, 4 * npts).reshape(npts, 4)
    return np.stack([r[:, 0] % N, r[:, 1] % F, r[:, 2] % Ho, r[:, 3] % Wo], axis=1).astype(np.int32)


def check_batched(layer: GpuLayer, x, tunings=(dict(),)):
    """Whole first and last image against the oracle, plus 65,536 sampled outputs over the batch."""
    s = layer.spec
    N = x.shape[0]
    coords = sampled_coords(1000 + s.idx, N, s.F, s.Ho, s.Wo)
    ref_pts = layer.oracle_at(x, coords)
    ref_first, ref_last = layer.oracle(x[:1]), layer.oracle(x[N - 1:])
    for t in tunings:
        say(s.name, s.dtype, "batch", N, "tuning", t)
        got = layer.run(x, **t)
        tol = TOL[s.dtype]
        assert rel_err(got[0], ref_first[0]) <= tol and rel_err(got[N - 1], ref_last[0]) <= tol
        pts = got[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]]
        rms = float(np.sqrt(np.mean(ref_first ** 2)))
        assert np.max(np.abs(pts.astype(np.float64) - ref_pts) / np.maximum(np.abs(ref_pts), rms)) <= tol


@pytest.mark.parametrize("N", [1, 32])
def test_config3_resnet50_shapes(N):
    for spec in L.config3(N):
        layer = GpuLayer(spec)
        x = L.gen_activations(spec)
        if N == 1:
            tun = [dict(), dict(kernel=G), TILED_TUNINGS[1], TILED_TUNINGS[5], DB_TUNINGS[1]]
            check(layer, x, tun)
        else:
            check_batched(layer, x)
        layer.free()


# ------------------------------------------------------------------------------------------------------------------
# config 4: VGG-16 shapes at batch 64, fp16 storage; library sizes 4/8/12, keep fractions 0.5/0.28/0.15
# ------------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("K,keep", [(4, 0.5), (4, 0.15), (8, 0.28), (12, 0.5), (12, 0.15)])
def test_config4_sweep_points_small_batch(K, keep):
    for spec in L.config4(K, keep, N=2):
        if spec.name not in ("conv1_1", "conv1_2", "conv3_2", "conv5_1"):
            continue
        layer = GpuLayer(spec)
        check(layer, L.gen_activations(spec), [dict()])
        layer.free()


_BATCH64 = {}


def batch64_activations(spec):
    """The 64 seeded images of a config-4 layer; they depend on the layer only, not on the sweep point, so the
    sweep-point tests generate them once per layer."""
    key = (spec.cfg, spec.idx, spec.N)
    if key not in _BATCH64:
        say("generating", spec.name, "batch", spec.N)
        _BATCH64[key] = L.gen_activations(spec)
    return _BATCH64[key]


# every explicit kernel form that takes the layer at this size, next to the library's own choice
def full_batch_tunings(spec):
    forms = [dict(), dict(kernel=T)]
    if spec.W % 4 == 0:
        forms.append(dict(kernel=pc.KERNEL_QUAD))
    return forms


@pytest.mark.parametrize("name", [L.VGG16_NAMES[i] for i in L.vgg_distinct_shapes()])
def test_config4_full_batch(name):
    """All nine distinct VGG-16 shapes at batch 64 at the sweep's centre point (K = 8, keep 0.28)."""
    spec = [s for s in L.config4(8, 0.28, N=64) if s.name == name][0]
    layer = GpuLayer(spec)
    check_batched(layer, batch64_activations(spec), full_batch_tunings(spec))
    layer.free()


@pytest.mark.parametrize("K,keep", [(8, 0.5), (8, 0.15), (4, 0.28), (12, 0.28), (4, 0.5), (12, 0.15)])
@pytest.mark.parametrize("name", ["conv1_2", "conv3_2", "conv4_2", "conv5_1"])
def test_config4_sweep_points_full_batch(name, K, keep):
    """The other sweep points at batch 64, in the launch configuration the bench times: the kept fraction and the
    batch decide between one workgroup per tile, walking workgroups and the channel split."""
    spec = [s for s in L.config4(K, keep, N=64) if s.name == name][0]
    layer = GpuLayer(spec)
    check_batched(layer, batch64_activations(spec), full_batch_tunings(spec))
    layer.free()


@pytest.mark.parametrize("stride", [1, 2])
def test_input_and_output_beyond_4_gib(stride):
    """2800 images of 64 x 112 x 112 in fp16: x is 4.5 GB and so is y at stride 1, so element offsets pass 2^31 and
    byte offsets 2^32 (stride 2: in x only).  The batch repeats four generated images (copied on the device), every output image is compared on the
    device with the first of its kind, and the first four, the last four and the four around the 4 GiB mark with
    the oracle."""
    import torch
    N, reps = 2800, 700
    spec = L.shrink([s for s in L.config4(8, 0.28, N=4) if s.name == "conv1_2"][0], H=112, W=112, stride=stride)
    layer = GpuLayer(spec)
    x4 = L.gen_activations(spec)
    ref4 = layer.oracle(x4)
    per_img = spec.F * spec.Ho * spec.Wo
    assert (N * per_img * 2 > 1 << 32 or stride == 2) and N * spec.C * spec.H * spec.W * 2 > 1 << 32
    dx = torch.from_numpy(x4).cuda().repeat(reps, 1, 1, 1).contiguous()
    assert dx.shape[0] == N
    pad = 4096
    buf = torch.empty(N * per_img + 2 * pad, dtype=torch.float16, device="cuda")
    dy = buf[pad:pad + N * per_img]
    st = torch.cuda.current_stream().cuda_stream
    mark = (1 << 32) // (spec.C * spec.H * spec.W * 2)      # the image in which byte 2^32 of x falls (y: stride 1)
    first = mark - mark % 4
    tol = TOL["f16"]
    tunings = [dict(), dict(kernel=pc.KERNEL_QUAD, filters_per_wave=1), dict(kernel=T), dict(kernel=G)]
    if stride == 2:    # paired staging (automatic), the separate pass that splits x into parity planes, generic
        tunings = [dict(), dict(kernel=T, rows=7, filters_per_wave=1, waves=8, channels_per_wave=4), dict(kernel=G)]
    for t in tunings:
        say(spec.name, "112x112 stride", stride, "batch", N, "tuning", t)
        buf.fill_(-777.0)
        if t:
            pc.conv3x3_tuned(dx, dy, layer.packed, layer.d_bias, N, spec.H, spec.W, stride, 1, 0, st, **t)
        else:
            pc.conv3x3(dx, dy, layer.packed, layer.d_bias, N, spec.H, spec.W, stride, 1, 0, st)
        torch.cuda.synchronize()
        assert bool((buf[:pad] == -777.0).all()) and bool((buf[pad + N * per_img:] == -777.0).all())
        got = dy.view(reps, 4, spec.F, spec.Ho, spec.Wo)
        for r0 in range(0, reps, 100):           # in slices: the comparison's temporaries stay small
            assert bool((got[r0:r0 + 100] == got[0:1]).all()), (t, r0)
        for n0 in (0, first, N - 4):
            g = dy.view(N, spec.F, spec.Ho, spec.Wo)[n0:n0 + 4].cpu().numpy()
            assert rel_err(g, ref4) <= tol, (t, n0)
    del dx, buf, dy
    torch.cuda.empty_cache()
    layer.free()


# ------------------------------------------------------------------------------------------------------------------
# the comparison kernels: dense 3x3 baseline and max-pool
# ------------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0)])
def test_dense_baseline(dtype, stride, pad):
    import torch
    spec = L.LayerSpec(cfg=12, idx=stride * 2 + pad, name="dense", N=2, C=24, F=10, H=17, W=19, stride=stride, pad=pad,
                       dtype=dtype)
    w, x, b = L.gen_weights(spec), L.gen_activations(spec), L.gen_bias(spec)
    say("dense", dtype, stride, pad)
    tdt = torch.float16 if dtype == "f16" else torch.float32
    dx, dw, db = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
    dy = torch.empty((2, 10, spec.Ho, spec.Wo), dtype=tdt, device="cuda")
    pc.dense_conv3x3(dx, dy, dw, db, pc.F16 if dtype == "f16" else pc.F32, 2, 24, 10, 17, 19, stride, pad, pc.FLAG_RELU,
                     torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ref = oracle.conv3x3(x, w, b, stride, pad, relu=True)
    assert rel_err(dy.cpu().numpy(), ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_maxpool(dtype):
    import torch
    x = L.gen_activations(L.LayerSpec(cfg=13, idx=0, name="pool", N=3, C=5, F=1, H=14, W=10, dtype=dtype))
    x = x - x.dtype.type(0.3)
    say("maxpool", dtype)
    dx = torch.from_numpy(x).cuda()
    dy = torch.empty((3, 5, 7, 5), dtype=dx.dtype, device="cuda")
    pc.maxpool2x2(dx, dy, pc.F16 if dtype == "f16" else pc.F32, 3, 5, 14, 10, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert np.array_equal(dy.cpu().numpy().astype(np.float32), oracle.maxpool2x2(x))
