"""The channel-minor form of the matrix-core kernel (PCONV_FLAG_NHWC: x [N][H][W][C], y [N][Ho][Wo][F]) against the
oracle: every tile shape and channel splits, tiles that run from one image into the next, a ragged last tile, both
strides and paddings, widths that make the 64-position pieces of the staging straddle rows, a library that leaves taps
unused; and what the form refuses."""
import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

from gpu_util import TOL, GpuLayer, rel_err

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)


def run_nhwc(layer, x_nchw, relu, **tuning):
    import torch
    s = layer.spec
    N = x_nchw.shape[0]
    dx = torch.from_numpy(np.ascontiguousarray(x_nchw.transpose(0, 2, 3, 1))).cuda()
    n_out = N * s.F * s.Ho * s.Wo
    buf = torch.full((n_out + 8192,), -777.0, dtype=torch.float16, device="cuda")
    dy = buf[4096:4096 + n_out]
    flags = pc.FLAG_NHWC | (pc.FLAG_RELU if relu else 0)
    st = torch.cuda.current_stream().cuda_stream
    if tuning:
        pc.conv3x3_tuned(dx, dy, layer.packed, layer.d_bias, N, s.H, s.W, s.stride, s.pad, flags, st, **tuning)
    else:
        pc.conv3x3(dx, dy, layer.packed, layer.d_bias, N, s.H, s.W, s.stride, s.pad, flags, st)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:4096] == -777.0) and np.all(out[4096 + n_out:] == -777.0), "write outside the output buffer"
    return out[4096:4096 + n_out].reshape(N, s.Ho, s.Wo, s.F).transpose(0, 3, 1, 2)


SHAPES = [  # N, C, F, H, W, stride, pad
    (3, 40, 72, 13, 28, 1, 1),      # 13 rows: tiles cross images; F ragged against 32 and 128
    (2, 32, 136, 9, 12, 1, 1),      # two filter tiles of 128, the second nearly empty
    (5, 16, 64, 7, 7, 1, 1),        # several images per tile
    (33, 24, 40, 7, 7, 1, 1),       # more images than one tile holds
    (2, 24, 32, 14, 14, 1, 1),
    (2, 32, 16, 15, 18, 2, 1),      # stride 2, odd height
    (3, 8, 8, 16, 16, 2, 0),        # stride 2, no padding
    (1, 8, 16, 5, 130, 1, 0),       # no padding, a row wider than a 128-pixel operand group
    (2, 64, 8, 8, 8, 1, 0),
    (1, 8, 8, 1, 1, 1, 1),          # a single pixel
    (2, 8, 64, 30, 224, 1, 1),      # a first layer (channels padded to eight) at full width
    (2, 48, 96, 20, 56, 2, 1),
    (4, 128, 128, 28, 28, 1, 1),
]


@pytest.mark.parametrize("case", SHAPES, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}s{c[5]}p{c[6]}" for c in SHAPES])
def test_channel_minor_form(case):
    N, C, F, H, W, stride, pad = case
    spec = L.LayerSpec(cfg=50, idx=SHAPES.index(case), name="nhwc", N=N, C=C, F=F, H=H, W=W, stride=stride, pad=pad,
                       dtype="f16", K=8, keep=0.4)
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    ref = layer.oracle(x, True)
    forms = [{}] + [dict(mfma_shape=s, channel_splits=k) for s in (1, 2, 3, 4) for k in (1, 2)]
    ran = 0
    for t in forms:
        say(case, t)
        try:
            got = run_nhwc(layer, x, True, **t)
        except pc.PconvError as e:
            assert e.code == pc.EUNSUPPORTED and t, (case, t, e.code)
            say("  unsupported")
            continue
        ran += 1
        err = rel_err(got, ref)
        assert err <= TOL["f16"], (case, t, err)
    assert ran >= 3
    assert rel_err(run_nhwc(layer, x, False), layer.oracle(x, False)) <= TOL["f16"]
    layer.free()


def test_unused_taps_and_equality_with_the_channel_major_form():
    # a library whose masks all lie in the upper two kernel rows: three tap slots are never staged
    spec = L.LayerSpec(cfg=50, idx=40, name="nhwc", N=3, C=32, F=64, H=12, W=20, dtype="f16", K=4, keep=0.5,
                       lib_kind="fixed4")
    spec = L.LayerSpec(**{**spec.__dict__, "K": 2})
    layer = GpuLayer(spec)
    x = L.gen_activations(spec)
    got = run_nhwc(layer, x, False)
    assert rel_err(got, layer.oracle(x, False)) <= TOL["f16"]
    # both forms multiply the same operands in the same order: equal bit for bit
    assert np.array_equal(got, layer.run(x, False))
    layer.free()


def test_what_the_form_refuses():
    import torch
    one = torch.zeros(4096, dtype=torch.float16, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    def refused(spec, **kw):
        layer = GpuLayer(spec)
        with pytest.raises(pc.PconvError) as e:
            pc.conv3x3(one, one[2048:], layer.packed, None, 1, 4, 4, 1, 1, pc.FLAG_NHWC, st)
        assert e.value.code == pc.EUNSUPPORTED
        layer.free()
    refused(L.LayerSpec(cfg=50, idx=60, name="nhwc", N=1, C=12, F=16, H=4, W=4, dtype="f16", K=8, keep=0.5))   # C % 8
    refused(L.LayerSpec(cfg=50, idx=61, name="nhwc", N=1, C=16, F=12, H=4, W=4, dtype="f16", K=8, keep=0.5))   # F % 8
    refused(L.LayerSpec(cfg=50, idx=62, name="nhwc", N=1, C=16, F=16, H=4, W=4, dtype="f32", K=8, keep=0.5))   # fp32
    layer = GpuLayer(L.LayerSpec(cfg=50, idx=63, name="nhwc", N=1, C=16, F=16, H=4, W=4, dtype="f16", K=8, keep=0.5))
    with pytest.raises(pc.PconvError) as e:                                          # a pointer that is not 16-byte aligned
        pc.conv3x3(one[1:], one[2048:], layer.packed, None, 1, 4, 4, 1, 1, pc.FLAG_NHWC, st)
    assert e.value.code == pc.EUNSUPPORTED
    layer.free()
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["conv1_2", "conv3_2", "conv5_1"])
def test_channel_minor_form_at_benchmark_shapes(name):
    # config 4 at batch 64 (K = 8, keep 0.28), as bench.py --nhwc launches it: the first and the last image whole,
    # and 65,536 outputs sampled over the batch
    spec = [s for s in L.config4(8, 0.28, 64) if s.name == name][0]
    say("nhwc full", name)
    layer = GpuLayer(spec)
    base = L.gen_activations(spec, images=[0, 1, 2, 3])
    x = np.concatenate([base] * (spec.N // 4), axis=0)
    x[spec.N - 1] = L.gen_image(spec, spec.N - 1)
    got = run_nhwc(layer, x, spec.relu)
    ref_first, ref_last = layer.oracle(x[:1]), layer.oracle(x[spec.N - 1:])
    tol = TOL["f16"]
    assert rel_err(got[0], ref_first[0]) <= tol and rel_err(got[spec.N - 1], ref_last[0]) <= tol
    rng = np.random.default_rng(77 + spec.idx)
    coords = np.stack([rng.integers(0, spec.N, 65536), rng.integers(0, spec.F, 65536), rng.integers(0, spec.Ho, 65536),
                       rng.integers(0, spec.Wo, 65536)], axis=1).astype(np.int32)
    ref_pts = layer.oracle_at(x, coords)
    pts = got[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]].astype(np.float64)
    rms = float(np.sqrt(np.mean(ref_first ** 2)))
    assert np.max(np.abs(pts - ref_pts) / np.maximum(np.abs(ref_pts), rms)) <= tol
    layer.free()
