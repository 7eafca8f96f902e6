"""Channel lists of the matrix-core kernel against the oracle: layers whose connectivity is clustered (similar filters
keep the same channels), packed in the order that pconv_filter_similarity_order gives, so that a filter tile stages
and multiplies only the channels it keeps.  Every tile shape, channel splits, both strides, ragged channel counts, a
tile that keeps nothing, a list whose last block is not full; and the same layer in its own filter order must give
the same outputs."""
import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

from gpu_util import TOL, rel_err

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)


def run(torch, packed, x, bias, spec, relu, **tuning):
    dx, db = torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda()
    n_out = spec.N * spec.F * spec.Ho * spec.Wo
    buf = torch.full((n_out + 8192,), -777.0, dtype=torch.float16, device="cuda")
    dy = buf[4096:4096 + n_out]
    st = torch.cuda.current_stream().cuda_stream
    flags = pc.FLAG_RELU if relu else 0
    if tuning:
        pc.conv3x3_tuned(dx, dy, packed, db, spec.N, spec.H, spec.W, spec.stride, spec.pad, flags, st, **tuning)
    else:
        pc.conv3x3(dx, dy, packed, db, spec.N, spec.H, spec.W, spec.stride, spec.pad, flags, st)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:4096] == -777.0) and np.all(out[4096 + n_out:] == -777.0), "write outside the output buffer"
    return out[4096:4096 + n_out].reshape(spec.N, spec.F, spec.Ho, spec.Wo)


CASES = [  # N, C, F, H, W, stride, pad, clusters, share, group
    (3, 128, 256, 14, 28, 1, 1, 4, 0.30, 64),
    (2, 200, 256, 9, 12, 1, 1, 2, 0.25, 128),     # C not a multiple of 16; lists whose last block is not full
    (2, 96, 192, 20, 56, 2, 1, 3, 0.30, 64),      # stride 2
    (5, 64, 128, 7, 7, 1, 0, 2, 0.40, 64),        # no padding, odd width
    (2, 512, 256, 14, 14, 1, 1, 4, 0.20, 64),     # many blocks per tile: channel splits have room
]


@pytest.mark.parametrize("case", CASES, ids=[f"n{c[0]}c{c[1]}f{c[2]}h{c[3]}w{c[4]}s{c[5]}p{c[6]}" for c in CASES])
def test_clustered_layer_in_similarity_order(case):
    import torch
    N, C, F, H, W, stride, pad, clusters, share, group = case
    i = CASES.index(case)
    spec = L.LayerSpec(cfg=41, idx=i, name="clustered", N=N, C=C, F=F, H=H, W=W, stride=stride, pad=pad, dtype="f16",
                       K=8, keep=0.8 * share)
    w, _ = L.gen_clustered_weights(spec, clusters, share)
    if i == 0:
        w[:5] = 0                                  # (with the zero scores' ties these filters keep nothing)
    x, bias, lib = L.gen_activations(spec), L.gen_bias(spec), spec.library()
    w32 = w.astype(np.float32)
    pid = pc.assign_patterns(w32, lib)
    mask = pc.select_connectivity(w32, lib, pid, spec.keep)
    if i == 0:
        mask[:5] = 0
    order = pc.filter_similarity_order(mask, group)
    assert np.array_equal(order, oracle.filter_similarity_order(mask, group))
    wo, po, mo, bo = w[order], pid[order], mask[order], bias[order]
    packed = pc.pack(wo, lib, po, mo)
    listed, dense = pc.packed_mfma_blocks(packed, group)
    say(case, "blocks", listed, "of", dense)
    assert listed * 10 <= dense * 7, "the re-ordered layer should have channel lists"
    ref = oracle.conv3x3(x, oracle.mask_weights(wo, po, mo, lib), bo, stride, pad, True)
    forms = [{}] + [dict(kernel=pc.KERNEL_MFMA, mfma_shape=s, channel_splits=k) for s in (1, 2, 3, 4) for k in (1, 2, 3)]
    ran = 0
    for t in forms:
        say("  form", t)
        try:
            got = run(torch, packed, x, bo, spec, True, **t)
        except pc.PconvError as e:
            assert e.code == pc.EUNSUPPORTED and t, t
            continue
        ran += 1
        err = rel_err(got, ref)
        assert err <= TOL["f16"], (case, t, err)
    assert ran >= 4
    # the layer in its own filter order: the same outputs, filter order[i] at place i
    natural = pc.pack(w, lib, pid, mask)
    got_nat = run(torch, natural, x, bias, spec, True)
    got_ord = run(torch, packed, x, bo, spec, True)
    assert rel_err(got_nat[:, order], got_ord.astype(np.float64)) <= 2 * TOL["f16"]
    if i == 0:
        assert np.all(got_nat[:, :5] == np.maximum(bias[:5], 0).astype(np.float16)[None, :, None, None])
    natural.free()
    packed.free()


def test_transposed_and_non_allocating_calls_on_a_layer_with_channel_lists():
    # the input gradient of a clustered layer runs on its transposed layer, whose tiles (of the original channels) have
    # lists of their own or none; the entry point that allocates nothing takes a layer with lists like any other
    import torch
    spec = L.LayerSpec(cfg=41, idx=9, name="clustered", N=2, C=128, F=256, H=14, W=14, dtype="f16", K=8, keep=0.24)
    w, _ = L.gen_clustered_weights(spec, 4, 0.30)
    lib, w32 = spec.library(), w.astype(np.float32)
    pid = pc.assign_patterns(w32, lib)
    mask = pc.select_connectivity(w32, lib, pid, spec.keep)
    order = pc.filter_similarity_order(mask, 64)
    wo, po, mo = w[order], pid[order], mask[order]
    packed = pc.pack(wo, lib, po, mo)
    assert pc.packed_mfma_blocks(packed, 64)[0] < pc.packed_mfma_blocks(packed, 64)[1]
    wm = oracle.mask_weights(wo, po, mo, lib)
    st = torch.cuda.current_stream().cuda_stream
    # input gradient
    dy = np.random.default_rng(3).standard_normal((spec.N, spec.F, spec.H, spec.W)).astype(np.float16)
    t = pc.packed_transpose(packed)
    d_dy = torch.from_numpy(dy).cuda()
    d_dx = torch.full((spec.N, spec.C, spec.H, spec.W), -777.0, dtype=torch.float16, device="cuda")
    pc.conv3x3_grad_input(d_dy, d_dx, t, spec.N, spec.H, spec.W, st)
    torch.cuda.synchronize()
    assert rel_err(d_dx.cpu().numpy(), oracle.conv3x3_grad_input(dy, wm, spec.H, spec.W, 1, 1)) <= TOL["f16"]
    # the non-allocating entry point: bit-equal to the allocating one
    x = L.gen_activations(spec)
    d_x = torch.from_numpy(x).cuda()
    y0 = torch.empty((spec.N, spec.F, spec.H, spec.W), dtype=torch.float16, device="cuda")
    y1 = torch.empty_like(y0)
    pc.conv3x3(d_x, y0, packed, None, spec.N, spec.H, spec.W, 1, 1, 0, st)
    pc.conv3x3_noalloc(d_x, y1, packed, None, spec.N, spec.H, spec.W, 1, 1, 0, st)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    assert rel_err(y0.cpu().numpy(), oracle.conv3x3(x, wm, None, 1, 1)) <= TOL["f16"]
    t.free()
    packed.free()


def test_clustered_layer_at_a_benchmark_shape():
    # 512 -> 512 channels at 28 x 28, batch 64, as bench.py --clustered launches it in similarity order: the first and
    # the last image whole, 65,536 outputs sampled over the batch
    import torch
    spec = [s for s in L.config4(8, 0.28, 64) if s.name == "conv4_2"][0]
    say("clustered full", spec.name)
    w, _ = L.gen_clustered_weights(spec, spec.F // 128, 1.25 * spec.keep)
    lib, w32 = spec.library(), w.astype(np.float32)
    pid = pc.assign_patterns(w32, lib)
    mask = pc.select_connectivity(w32, lib, pid, spec.keep)
    order = pc.filter_similarity_order(mask, 128)
    wo, po, mo, bo = w[order], pid[order], mask[order], L.gen_bias(spec)[order]
    packed = pc.pack(wo, lib, po, mo)
    listed, dense = pc.packed_mfma_blocks(packed, 128)
    assert listed * 2 <= dense
    base = L.gen_activations(spec, images=[0, 1, 2, 3])
    x = np.concatenate([base] * (spec.N // 4), axis=0)
    x[spec.N - 1] = L.gen_image(spec, spec.N - 1)
    got = run(torch, packed, x, bo, spec, True)
    wm = oracle.mask_weights(wo, po, mo, lib)
    tol = TOL["f16"]
    ref_first, ref_last = oracle.conv3x3(x[:1], wm, bo, 1, 1, True), oracle.conv3x3(x[spec.N - 1:], wm, bo, 1, 1, True)
    assert rel_err(got[0], ref_first[0]) <= tol and rel_err(got[spec.N - 1], ref_last[0]) <= tol
    rng = np.random.default_rng(5)
    coords = np.stack([rng.integers(0, spec.N, 65536), rng.integers(0, spec.F, 65536), rng.integers(0, spec.Ho, 65536),
                       rng.integers(0, spec.Wo, 65536)], axis=1).astype(np.int32)
    ref_pts = oracle.conv3x3_at(x, wm, coords, bo, 1, 1, True)
    pts = got[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]].astype(np.float64)
    rms = float(np.sqrt(np.mean(ref_first ** 2)))
    assert np.max(np.abs(pts - ref_pts) / np.maximum(np.abs(ref_pts), rms)) <= tol
    packed.free()
