"""Pins for the CPU oracle: facts the paper prints, closed forms, brute force and library routines.

Each test is chosen so that a plausible slip in the oracle (dropped term, wrong sign or index, transposed or flipped
kernel, off-by-one in padding or stride, mask bit order) fails at least one of them.  None of them calls the HIP path.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from workloads import layers as L
from workloads import rng

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------------------------------------------------------
# brute force: second, independent implementation.  Explicit zero padding, explicit zeros in the weights, seven
# nested loops, nothing skipped.
# ------------------------------------------------------------------------------------------------------------------

def brute_masked_weights(w, pid, mask, lib):
    F, C = w.shape[:2]
    out = np.zeros((F, C, 3, 3), dtype=np.float64)
    for f in range(F):
        for c in range(C):
            if not mask[f][c]:
                continue
            m = int(lib[int(pid[f][c])])
            for ky in range(3):
                for kx in range(3):
                    if (m >> (3 * ky + kx)) & 1:
                        out[f, c, ky, kx] = float(w[f, c, ky, kx])
    return out


def brute_dense_conv(x, wd, bias, stride, pad, relu=False):
    N, C, H, W = x.shape
    F = wd.shape[0]
    Ho = (H + 2 * pad - 3) // stride + 1
    Wo = (W + 2 * pad - 3) // stride + 1
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    y = np.zeros((N, F, max(Ho, 0), max(Wo, 0)), dtype=np.float64)
    for n in range(N):
        for f in range(F):
            for oy in range(Ho):
                for ox in range(Wo):
                    acc = float(bias[f]) if bias is not None else 0.0
                    for c in range(C):
                        for ky in range(3):
                            for kx in range(3):
                                acc += float(wd[f, c, ky, kx]) * float(xp[n, c, oy * stride + ky, ox * stride + kx])
                    y[n, f, oy, ox] = max(acc, 0.0) if relu else acc
    return y


def rand_case(seed, N, C, F, H, W, K=None, lib=None, keep=0.6):
    r = np.random.default_rng(seed)
    if lib is None:
        lib = np.asarray(r.choice(L.all_masks_4of9(), size=K, replace=False), dtype=np.uint16)
    K = len(lib)
    w = r.standard_normal((F, C, 3, 3)).astype(np.float32)
    x = np.maximum(r.standard_normal((N, C, H, W)), 0).astype(np.float32)
    b = r.standard_normal(F).astype(np.float32)
    pid = r.integers(0, K, size=(F, C)).astype(np.uint8)
    mask = (r.random((F, C)) < keep).astype(np.uint8)
    return x, w, b, pid, mask, lib


def ulp_close(a, b, ulps=1):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    tol = ulps * np.spacing(np.maximum(np.abs(a), np.abs(b)))
    return np.all(np.abs(a - b) <= tol)


# ------------------------------------------------------------------------------------------------------------------
# counts the paper prints (sections 5.1, 7.1, 7.3, table 1)
# ------------------------------------------------------------------------------------------------------------------

def _counts():
    out = {}
    with open(os.path.join(GOLDEN, "paper_counts.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if len(line) == 2:
                out[line[0]] = float(line[1])
    return out


def test_counts_from_the_paper():
    g = _counts()
    masks = L.all_masks_4of9()
    assert len(masks) == g["initial_library_size"] == math.comb(9, 4)
    assert all(oracle.library_bits([m]).sum() == g["kept_per_kernel"] for m in masks)
    assert len(L.centre_masks()) == math.comb(8, 3) == 56
    assert 9 / g["kept_per_kernel"] == g["pattern_compression"]
    assert sum(c * f for c, f, _, _ in L.VGG16) == 1634496 > g["vgg16_kernels_more_than"]
    # keep fraction 0.28 on top of the 2.25x of the patterns is the 8x operating point of table 1
    assert abs(g["pattern_compression"] / 0.28 - g["vgg16_overall_compression"]) < 0.05
    # masked tensor of a pattern-only layer keeps exactly 4/9 of its entries
    x, w, b, pid, mask, lib = rand_case(1, 1, 6, 5, 4, 4, K=8, keep=1.1)
    wm = oracle.mask_weights(w, pid, mask, lib)
    assert np.count_nonzero(wm) * 9 == wm.size * 4


def test_library_rejects_bad_masks():
    for bad in ([0x00F, 0x1FF], [0x007], [512 + 15], []):
        with pytest.raises(ValueError):
            oracle.library_bits(bad)


# ------------------------------------------------------------------------------------------------------------------
# the paper's worked example: four masks interpolate to the binomial Gaussian (section 4.2)
# ------------------------------------------------------------------------------------------------------------------

def test_gaussian_worked_example():
    G = np.loadtxt(os.path.join(GOLDEN, "gaussian_3x3.txt"))
    assert np.array_equal(np.outer([1, 2, 1], [1, 2, 1]), G)
    assert np.array_equal(np.convolve([1, 1], [1, 1]), [1, 2, 1])
    lib = np.asarray(L.FIXED4, dtype=np.uint16)
    # the four 2x2-block masks add up to the printed matrix
    assert np.array_equal(oracle.library_bits(lib).sum(axis=0).reshape(3, 3), G)
    # and through the convolution: filter j = all-ones kernel pruned to mask j; a unit impulse in the middle of a
    # 5x5 image; the sum over the four filters of the response is the matrix (it is symmetric, so correlation and
    # convolution agree), and each single response is the point-reflected mask
    w = np.ones((4, 1, 3, 3), dtype=np.float32)
    pid = np.arange(4, dtype=np.uint8).reshape(4, 1)
    mask = np.ones((4, 1), dtype=np.uint8)
    x = np.zeros((1, 1, 5, 5), dtype=np.float32)
    x[0, 0, 2, 2] = 1.0
    y = oracle.pattern_conv3x3(x, w, pid, mask, lib, None, 1, 1)
    assert np.array_equal(y[0].sum(axis=0)[1:4, 1:4], G)
    assert np.count_nonzero(y) == 16
    for j in range(4):
        mj = oracle.library_bits(lib)[j].reshape(3, 3)
        assert np.array_equal(y[0, j, 1:4, 1:4], mj[::-1, ::-1])


# ------------------------------------------------------------------------------------------------------------------
# orientation: which tap reads which input (a flipped or transposed kernel fails here)
# ------------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("t", range(9))
def test_single_tap_orientation(t):
    ky, kx = divmod(t, 3)
    others = [u for u in range(9) if u != t][:3]
    m = (1 << t) | sum(1 << u for u in others)
    lib = np.asarray([m], dtype=np.uint16)
    w = np.zeros((1, 1, 3, 3), dtype=np.float32)
    w[0, 0, ky, kx] = 3.0
    x = np.zeros((1, 1, 6, 7), dtype=np.float32)
    iy, ix = 2, 4
    x[0, 0, iy, ix] = 2.0
    pid = np.zeros((1, 1), np.uint8)
    mask = np.ones((1, 1), np.uint8)
    for stride, pad in ((1, 1), (1, 0), (2, 1), (2, 0)):
        y = oracle.pattern_conv3x3(x, w, pid, mask, lib, None, stride, pad)
        exp = np.zeros_like(y)
        # input (iy, ix) is read by output (oy, ox) through tap (ky, kx) when oy*s + ky - p = iy, ox*s + kx - p = ix
        ny, nx = iy - ky + pad, ix - kx + pad
        if ny % stride == 0 and nx % stride == 0:
            oy, ox = ny // stride, nx // stride
            if 0 <= oy < y.shape[2] and 0 <= ox < y.shape[3]:
                exp[0, 0, oy, ox] = 6.0
        assert np.array_equal(y, exp), (t, stride, pad)


def test_output_size_formula():
    for H, W, s, p in itertools.product([1, 2, 3, 4, 7, 8], [1, 3, 5, 6], [1, 2], [0, 1]):
        Ho, Wo = oracle.out_hw(H, W, s, p)
        x = torch.zeros(1, 1, H, W, dtype=torch.float64)
        if H + 2 * p < 3 or W + 2 * p < 3:
            assert Ho <= 0 or Wo <= 0
            continue
        ref = torch.nn.functional.conv2d(x, torch.zeros(1, 1, 3, 3, dtype=torch.float64), stride=s, padding=p)
        assert tuple(ref.shape[2:]) == (Ho, Wo)


# ------------------------------------------------------------------------------------------------------------------
# brute force on tiny inputs, every mask, random masks
# ------------------------------------------------------------------------------------------------------------------

def _tiny_grid():
    r = np.random.default_rng(7)
    combos = [c for c in itertools.product([1, 2, 3, 5], [1, 2, 3, 5], [1, 2, 3, 4, 7], [1, 2, 3, 4, 7], [1, 2], [0, 1],
                                           [1, 2]) if c[2] + 2 * c[5] >= 3 and c[3] + 2 * c[5] >= 3]
    pick = r.choice(len(combos), size=90, replace=False)
    return [combos[i] for i in sorted(pick)]


@pytest.mark.parametrize("F,C,H,W,stride,pad,N", _tiny_grid())
def test_oracle_equals_brute_force(F, C, H, W, stride, pad, N):
    x, w, b, pid, mask, lib = rand_case(F * 1000 + C * 100 + H * 10 + W, N, C, F, H, W, K=6)
    wd = brute_masked_weights(w, pid, mask, lib)
    assert np.array_equal(wd, oracle.mask_weights(w, pid, mask, lib).astype(np.float64))
    for relu in (False, True):
        y = oracle.pattern_conv3x3(x, w, pid, mask, lib, b, stride, pad, relu)
        yb = brute_dense_conv(x, wd, b, stride, pad, relu)
        assert y.shape == yb.shape
        assert ulp_close(y, yb, 1)


def test_every_one_of_the_126_masks_against_brute_force():
    masks = L.all_masks_4of9()
    lib = np.asarray(masks, dtype=np.uint16)
    r = np.random.default_rng(3)
    F, C = 126, 2
    w = r.standard_normal((F, C, 3, 3)).astype(np.float32)
    x = r.standard_normal((1, C, 4, 5)).astype(np.float32)
    pid = np.repeat(np.arange(126, dtype=np.uint8)[:, None], C, axis=1)
    mask = np.ones((F, C), np.uint8)
    y = oracle.pattern_conv3x3(x, w, pid, mask, lib, None, 1, 1)
    yb = brute_dense_conv(x, brute_masked_weights(w, pid, mask, lib), None, 1, 1)
    assert ulp_close(y, yb, 1)


def test_points_variant_matches_full():
    x, w, b, pid, mask, lib = rand_case(11, 3, 7, 6, 9, 8, K=8)
    wm = oracle.mask_weights(w, pid, mask, lib)
    for stride, pad, relu in ((1, 1, False), (2, 1, True), (1, 0, False), (2, 0, True)):
        y = oracle.conv3x3(x, wm, b, stride, pad, relu)
        coords = np.asarray(list(np.ndindex(*y.shape)), dtype=np.int32)
        yp = oracle.conv3x3_at(x, wm, coords, b, stride, pad, relu)
        assert np.array_equal(yp.reshape(y.shape), y)
    with pytest.raises(ValueError):
        oracle.conv3x3_at(x, wm, np.asarray([[0, 0, 99, 0]]), b, 1, 1)


# ------------------------------------------------------------------------------------------------------------------
# library routine: the pruned layer is a dense convolution with explicit zeros
# ------------------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0), (2, 0)])
def test_against_float64_conv2d(stride, pad):
    x, w, b, pid, mask, lib = rand_case(21 + stride * 2 + pad, 2, 19, 23, 17, 13, K=8, keep=0.3)
    wm = oracle.mask_weights(w, pid, mask, lib)
    y = oracle.conv3x3(x, wm, b, stride, pad)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(wm).double(),
                                     torch.from_numpy(b).double(), stride=stride, padding=pad).numpy()
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_maxpool_against_library():
    r = np.random.default_rng(5)
    for H, W in ((4, 4), (7, 9), (2, 2), (14, 14)):
        x = r.standard_normal((2, 3, H, W)).astype(np.float32)
        ref = torch.nn.functional.max_pool2d(torch.from_numpy(x), 2, 2).numpy()
        assert np.array_equal(oracle.maxpool2x2(x), ref)


# ------------------------------------------------------------------------------------------------------------------
# invariants: exactly four kept entries inside the library pattern; removed kernels and pruned taps contribute nothing
# ------------------------------------------------------------------------------------------------------------------

def test_invariants_pruned_entries_do_not_matter():
    x, w, b, pid, mask, lib = rand_case(31, 2, 9, 8, 6, 7, K=8, keep=0.5)
    bits = oracle.library_bits(lib)
    assert np.all(bits.sum(axis=1) == 4)
    wm = oracle.mask_weights(w, pid, mask, lib)
    F, C = w.shape[:2]
    for f in range(F):
        for c in range(C):
            nz = (wm[f, c].reshape(9) != 0)
            if mask[f, c]:
                assert np.all(bits[pid[f, c]][nz] == 1) and nz.sum() == 4   # Gaussian weights are never exactly 0
            else:
                assert not nz.any()
    y0 = oracle.pattern_conv3x3(x, w, pid, mask, lib, b, 1, 1)
    # perturb every weight the masks remove, and the pattern ids of removed kernels
    keep_sel = oracle.mask_weights(np.ones_like(w), pid, mask, lib) != 0
    w2 = np.where(keep_sel, w, w + 123.0).astype(np.float32)
    pid2 = np.where(mask != 0, pid, (pid + 3) % len(lib)).astype(np.uint8)
    y1 = oracle.pattern_conv3x3(x, w2, pid2, mask, lib, b, 1, 1)
    assert np.array_equal(y0, y1)
    # and a kept weight does matter
    f, c = np.argwhere(mask != 0)[0]
    t = int(np.nonzero(bits[pid[f, c]])[0][0])
    w3 = w.copy()
    w3[f, c, t // 3, t % 3] += 1.0
    y2 = oracle.pattern_conv3x3(x, w3, pid, mask, lib, b, 1, 1)
    assert not np.array_equal(y0[:, f], y2[:, f])
    others = [g for g in range(F) if g != f]
    assert np.array_equal(y0[:, others], y2[:, others])


# ------------------------------------------------------------------------------------------------------------------
# closed forms
# ------------------------------------------------------------------------------------------------------------------

def test_delta_kernel_is_identity_plus_bias():
    r = np.random.default_rng(41)
    C, F = 5, 5
    lib = np.asarray(L.FIXED4, np.uint16)
    w = np.zeros((F, C, 3, 3), np.float32)
    a = r.standard_normal(F).astype(np.float32)
    for f in range(F):
        w[f, f, 1, 1] = a[f]
    mask = np.eye(F, dtype=np.uint8)
    pid = r.integers(0, 4, (F, C)).astype(np.uint8)
    x = r.standard_normal((2, C, 6, 5)).astype(np.float32)
    b = r.standard_normal(F).astype(np.float32)
    y = oracle.pattern_conv3x3(x, w, pid, mask, lib, b, 1, 1)
    exp = a.astype(np.float64)[None, :, None, None] * x.astype(np.float64) + b.astype(np.float64)[None, :, None, None]
    assert ulp_close(y, exp, 1)


def test_all_ones_input_closed_form():
    x0, w, b, pid, mask, lib = rand_case(51, 1, 6, 4, 7, 8, K=8, keep=0.7)
    x = np.ones_like(x0)
    wm = oracle.mask_weights(w, pid, mask, lib).astype(np.float64)
    y = oracle.pattern_conv3x3(x, w, pid, mask, lib, b, 1, 1)
    H, W = x.shape[2:]
    for f in range(w.shape[0]):
        for oy in range(H):
            for ox in range(W):
                kys = [ky for ky in range(3) if 0 <= oy + ky - 1 < H]
                kxs = [kx for kx in range(3) if 0 <= ox + kx - 1 < W]
                exp = math.fsum([float(b[f])] + [wm[f, c, ky, kx] for c in range(w.shape[1]) for ky in kys for kx in kxs])
                assert abs(y[0, f, oy, ox] - exp) <= 1e-13 * max(1.0, abs(exp))


def test_linearity_and_shift():
    x, w, b, pid, mask, lib = rand_case(61, 1, 4, 3, 9, 9, K=5)
    x2 = np.random.default_rng(62).standard_normal(x.shape).astype(np.float32)
    f = lambda xx, ww, bb: oracle.pattern_conv3x3(xx, ww, pid, mask, lib, bb, 1, 1)
    ya, yb = f(x, w, None), f(x2, w, None)
    ysum = f((x.astype(np.float64) + x2).astype(np.float32), w, None)   # fp32 sum is rounded: compare loosely
    assert np.max(np.abs(ysum - (ya + yb))) < 1e-5
    assert np.max(np.abs(f(x, 2 * w, None) - 2 * ya)) == 0.0            # scaling by two is exact
    assert np.max(np.abs(f(x, w, b) - (ya + b.astype(np.float64)[None, :, None, None]))) < 1e-12
    # shift-equivariance away from the border
    xs = np.zeros_like(x)
    xs[:, :, 1:, 2:] = x[:, :, :-1, :-2]
    ys = f(xs, w, None)
    assert np.max(np.abs(ys[:, :, 3:-1, 4:-1] - ya[:, :, 2:-2, 2:-3])) < 1e-12


# ------------------------------------------------------------------------------------------------------------------
# assignment and connectivity selection against exact rational arithmetic
# ------------------------------------------------------------------------------------------------------------------

def _exact_energy(kernel9, m):
    return sum(Fraction(float(kernel9[t])) ** 2 for t in range(9) if (m >> t) & 1)


def test_assignment_is_the_projection_onto_the_library():
    r = np.random.default_rng(71)
    for K in (4, 8, 12, 126):
        lib = np.asarray(r.choice(L.all_masks_4of9(), size=K, replace=False), np.uint16)
        w = r.standard_normal((6, 7, 3, 3)).astype(np.float32)
        pid = oracle.assign_patterns(w, lib)
        assert pid.dtype == np.uint8 and pid.shape == (6, 7)
        for f in range(6):
            for c in range(7):
                k9 = w[f, c].reshape(9)
                e = [_exact_energy(k9, int(m)) for m in lib]
                best = max(e)
                assert e[pid[f, c]] == best or float(e[pid[f, c]]) == float(best)
                # projection property: the chosen mask minimises ||W - W o M||^2
                total = sum(Fraction(float(v)) ** 2 for v in k9)
                assert all(total - e[pid[f, c]] <= total - ej or float(ej) == float(e[pid[f, c]]) for ej in e)


def test_assignment_ties_go_to_the_lowest_index():
    lib = np.asarray(L.FIXED4, np.uint16)
    w = np.ones((1, 1, 3, 3), np.float32)                      # every mask keeps the same energy
    assert oracle.assign_patterns(w, lib)[0, 0] == 0
    w = np.zeros((1, 1, 3, 3), np.float32)
    w[0, 0, 2, 2] = 1.0                                         # only mask 3 (down-right block) keeps it
    assert oracle.assign_patterns(w, lib)[0, 0] == 3
    w[0, 0, 0, 2] = -1.0                                        # masks 1 and 3 tie
    assert oracle.assign_patterns(w, lib)[0, 0] == 1


def test_connectivity_topk_against_exact_sort():
    r = np.random.default_rng(81)
    lib = np.asarray(r.choice(L.centre_masks(), size=8, replace=False), np.uint16)
    F, C = 5, 9
    w = r.standard_normal((F, C, 3, 3)).astype(np.float32)
    w[1, 2] = w[3, 4]                                           # an exact tie
    pid = oracle.assign_patterns(w, lib)
    for keep in (0.0, 0.1, 0.28, 0.5, 0.9, 1.0):
        mask = oracle.select_connectivity(w, lib, pid, keep)
        k = int(math.floor(keep * F * C + 0.5))
        assert mask.sum() == k
        score = [(-_exact_energy(w[i // C, i % C].reshape(9), int(lib[pid[i // C, i % C]])), i) for i in range(F * C)]
        exp = np.zeros(F * C, np.uint8)
        for _, i in sorted(score)[:k]:
            exp[i] = 1
        assert np.array_equal(mask.reshape(-1), exp)


def test_rounding_of_k_is_floor_of_x_plus_half():
    w = np.random.default_rng(91).standard_normal((2, 5, 3, 3)).astype(np.float32)   # 10 kernels
    lib = np.asarray(L.FIXED4, np.uint16)
    pid = oracle.assign_patterns(w, lib)
    assert oracle.select_connectivity(w, lib, pid, 0.25).sum() == 3    # 2.5 -> 3 (banker's rounding would give 2)
    assert oracle.select_connectivity(w, lib, pid, 0.45).sum() == 5    # 4.5 -> 5
    assert oracle.select_connectivity(w, lib, pid, 0.28).sum() == 3


# ------------------------------------------------------------------------------------------------------------------
# canonical packing
# ------------------------------------------------------------------------------------------------------------------

def test_pack_hand_example():
    # two filters, three channels, library {up-left block, down-right block}
    lib = np.asarray([0x01B, 0x1B0], np.uint16)
    w = np.arange(2 * 3 * 9, dtype=np.float32).reshape(2, 3, 3, 3)
    pid = np.asarray([[1, 0, 0], [0, 1, 0]], np.uint8)
    mask = np.asarray([[1, 0, 0], [1, 1, 1]], np.uint8)
    fo, gp, cin, w4 = oracle.pack_canonical(w, pid, mask, lib)
    assert fo.tolist() == [1, 0]                       # filter 1 keeps three kernels, filter 0 one
    assert gp.tolist() == [0, 2, 3, 3, 4]              # (f1,m0): c0,c2   (f1,m1): c1   (f0,m0): -   (f0,m1): c0
    assert cin.tolist() == [0, 2, 1, 0]
    base = lambda f, c: (f * 3 + c) * 9
    assert w4.tolist() == [[base(1, 0) + t for t in (0, 1, 3, 4)], [base(1, 2) + t for t in (0, 1, 3, 4)],
                           [base(1, 1) + t for t in (4, 5, 7, 8)], [base(0, 0) + t for t in (4, 5, 7, 8)]]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_pack_round_trip_and_structure(dtype):
    x, w, b, pid, mask, lib = rand_case(101, 1, 37, 29, 3, 3, K=8, keep=0.3)
    w = w.astype(dtype)
    w[0, 0, 1, 1] = dtype(-0.0)
    mask[0, 0] = 1
    fo, gp, cin, w4 = oracle.pack_canonical(w, pid, mask, lib)
    F, C, K = 29, 37, 8
    assert sorted(fo.tolist()) == list(range(F))
    counts = (mask != 0).sum(axis=1)
    assert all((counts[fo[i]], -int(fo[i])) >= (counts[fo[i + 1]], -int(fo[i + 1])) for i in range(F - 1))
    assert gp[0] == 0 and gp[-1] == mask.sum() == len(cin) == len(w4) and np.all(np.diff(gp.astype(np.int64)) >= 0)
    for i in range(F):
        for j in range(K):
            seg = cin[gp[i * K + j]:gp[i * K + j + 1]].astype(np.int64)
            assert np.all(np.diff(seg) > 0)
            assert np.all(pid[fo[i], seg] == j) and np.all(mask[fo[i], seg] == 1)
    back = oracle.unpack_canonical(fo, gp, cin, w4, lib, F, C)
    wm = oracle.mask_weights(w, pid, mask, lib)
    assert back.dtype == wm.dtype
    assert np.array_equal(back.view(np.uint16 if dtype == np.float16 else np.uint32),
                          wm.view(np.uint16 if dtype == np.float16 else np.uint32))   # bit for bit, -0.0 included


# ------------------------------------------------------------------------------------------------------------------
# the input recipe (not the oracle, but everything downstream leans on it)
# ------------------------------------------------------------------------------------------------------------------

def test_input_recipe_statistics():
    s = L.config1()
    w = L.gen_weights(s)
    x = L.gen_image(s, 0)
    b = L.gen_bias(L.shrink(s, F=4096))
    assert abs(w.std() / math.sqrt(2.0 / (9 * s.C)) - 1) < 0.01
    assert abs((x == 0).mean() - 0.5) < 0.005 and x.min() == 0
    assert abs(x[x > 0].mean() - math.sqrt(2 / math.pi)) < 0.01        # mean of a half-normal
    assert abs(b.std() - 0.1) < 0.005
    assert np.array_equal(L.gen_weights(s), w)                          # seeded: same bytes again
    lib4, lib8, lib12 = (L.drawn_library(4, K) for K in (4, 8, 12))
    assert lib8[:4].tolist() == lib4.tolist() and lib12[:8].tolist() == lib8.tolist()
    assert all((int(m) >> 4) & 1 for m in lib12) and len(set(lib12.tolist())) == 12
    assert rng.raw_u64(1234567, 3).tolist() == [int(v) for v in rng.raw_u64(1234567, 5)[:3]]
    # SplitMix64 reference values for seed 1234567 (first outputs of the published generator)
    assert rng.raw_u64(1234567, 2).tolist() == [6457827717110365317, 3203168211198807973]
    assert [s.n_keep_target() for s in L.config2()] == [192, 1434, 2867, 5734, 9175, 18350, 18350, 26214] + [52429] * 5
