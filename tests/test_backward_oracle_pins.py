"""Pins of the backward-pass oracle and of the grouped 1x1 oracle (oracle/backward_oracle.py) to things other than
themselves: brute-force loops on tiny inputs, the adjoint identities that tie both gradients to the forward oracle
(C code, pinned on its own), float64 autograd of the library convolution, closed forms, and for the 1x1 layer the
3x3 forward oracle on centre-tap kernels.  CPU only."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from oracle import backward_oracle as B

RNG = np.random.default_rng(20010771)


def _case(N, C, F, H, W, s, p):
    Ho, Wo = B._out_hw(H, W, s, p)
    x = RNG.standard_normal((N, C, H, W))
    w = RNG.standard_normal((F, C, 3, 3))
    dy = RNG.standard_normal((N, F, Ho, Wo))
    return x, w, dy, Ho, Wo


TINY = [(1, 1, 1, 3, 3, 1, 1), (2, 2, 3, 4, 5, 1, 1), (1, 3, 2, 5, 4, 1, 0), (2, 2, 2, 6, 7, 2, 1), (1, 2, 3, 7, 5, 2, 0),
        (1, 1, 2, 4, 4, 2, 1)]


@pytest.mark.parametrize("shape", TINY)
def test_gradients_equal_brute_force_loops(shape):
    N, C, F, H, W, s, p = shape
    x, w, dy, Ho, Wo = _case(*shape)
    dx = np.zeros((N, C, H, W))
    G = np.zeros((F, C, 3, 3))
    for n, f, c, oy, ox, ky, kx in itertools.product(range(N), range(F), range(C), range(Ho), range(Wo), range(3), range(3)):
        iy, ix = oy * s + ky - p, ox * s + kx - p
        if 0 <= iy < H and 0 <= ix < W:
            dx[n, c, iy, ix] += w[f, c, ky, kx] * dy[n, f, oy, ox]
            G[f, c, ky, kx] += dy[n, f, oy, ox] * x[n, c, iy, ix]
    np.testing.assert_allclose(B.conv3x3_grad_input(dy, w, H, W, s, p), dx, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(B.conv3x3_grad_weight(x, dy, s, p), G, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("shape", [(2, 5, 4, 9, 8, 1, 1), (1, 4, 6, 8, 8, 1, 0), (2, 3, 5, 9, 11, 2, 1), (1, 6, 3, 10, 7, 2, 0)])
def test_adjoint_identities_with_the_forward_oracle(shape):
    # y is bilinear in (x, w): <y, dy> = <x, dx> = <w, G>, with y from the C forward oracle (float32 inputs, so the
    # operands are rounded to float32 first and all three sides see the same numbers)
    N, C, F, H, W, s, p = shape
    x, w, dy, _, _ = _case(*shape)
    x, w = x.astype(np.float32), w.astype(np.float32)
    y = oracle.conv3x3(x, w, None, s, p)
    lhs = float(np.sum(y * dy))
    assert abs(lhs - float(np.sum(B.conv3x3_grad_input(dy, w, H, W, s, p) * x))) <= 1e-9 * max(1.0, abs(lhs))
    assert abs(lhs - float(np.sum(B.conv3x3_grad_weight(x, dy, s, p) * w))) <= 1e-9 * max(1.0, abs(lhs))


@pytest.mark.parametrize("shape", [(2, 3, 4, 8, 9, 1, 1), (1, 2, 3, 7, 7, 1, 0), (2, 3, 2, 9, 8, 2, 1), (1, 2, 2, 8, 6, 2, 0)])
def test_gradients_equal_float64_autograd(shape):
    N, C, F, H, W, s, p = shape
    x, w, dy, _, _ = _case(*shape)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    ty = torch.nn.functional.conv2d(tx, tw, None, stride=s, padding=p)
    ty.backward(torch.tensor(dy, dtype=torch.float64))
    np.testing.assert_allclose(B.conv3x3_grad_input(dy, w, H, W, s, p), tx.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(B.conv3x3_grad_weight(x, dy, s, p), tw.grad.numpy(), rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("shape", [(2, 3, 4, 6, 7, 1, 1), (1, 2, 3, 7, 6, 2, 1), (2, 2, 2, 5, 5, 1, 0)])
def test_weight_gradient_at_listed_coordinates_equals_the_full_one(shape):
    N, C, F, H, W, s, p = shape
    x, _, dy, _, _ = _case(*shape)
    G = B.conv3x3_grad_weight(x, dy, s, p)
    coords = [(f, c, ky, kx) for f in range(F) for c in range(C) for ky in range(3) for kx in range(3)]
    got = B.conv3x3_grad_weight_at(x, dy, coords, s, p)
    np.testing.assert_allclose(got, G.reshape(-1), rtol=1e-12, atol=1e-12)


def test_closed_forms():
    # a centre-only kernel of value a: dx = a * dy (stride 1, pad 1); its weight gradient is <dy, x>
    x, _, dy, _, _ = _case(2, 1, 1, 6, 5, 1, 1)
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 1, 1] = -1.75
    np.testing.assert_allclose(B.conv3x3_grad_input(dy, w, 6, 5), -1.75 * dy, rtol=0, atol=1e-14)
    G = B.conv3x3_grad_weight(x, dy)
    assert abs(G[0, 0, 1, 1] - np.sum(dy * x)) < 1e-12
    # the tap above the centre reads the row above: its gradient pairs dy row r with x row r - 1
    assert abs(G[0, 0, 0, 1] - np.sum(dy[:, :, 1:, :] * x[:, :, :-1, :])) < 1e-12
    assert abs(G[0, 0, 1, 0] - np.sum(dy[:, :, :, 1:] * x[:, :, :, :-1])) < 1e-12
    # a single tap at the left column hands dy to the input one column to the LEFT of the output's own column
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 1, 0] = 1.0
    dx = B.conv3x3_grad_input(dy, w, 6, 5)
    np.testing.assert_allclose(dx[:, :, :, :-1], dy[:, :, :, 1:], atol=1e-14)
    assert np.all(dx[:, :, :, -1] == 0)


def test_masked_weight_gradient_is_the_dense_one_under_the_mask():
    F, C = 5, 7
    x, _, dy, _, _ = _case(2, C, F, 6, 6, 1, 1)
    lib = np.array([0x01B, 0x036, 0x0D8, 0x1B0], dtype=np.uint16)
    pid = RNG.integers(0, 4, size=(F, C)).astype(np.uint8)
    mask = (RNG.random((F, C)) < 0.5).astype(np.uint8)
    G = B.conv3x3_grad_weight(x, dy)
    Gm = B.masked_grad_weight(x, dy, pid, mask, lib)
    bits = oracle.library_bits(lib)
    for f in range(F):
        for c in range(C):
            sel = bits[pid[f, c]].reshape(3, 3).astype(bool) & bool(mask[f, c])
            assert np.array_equal(Gm[f, c][sel], G[f, c][sel]) and np.all(Gm[f, c][~sel] == 0)
    assert int(np.count_nonzero(Gm)) == 4 * int(mask.sum())


def test_group_mask_of_the_1x1_layer():
    lib = np.array([0x01B, 0x1B0], dtype=np.uint16)       # taps {0,1,3,4} and {4,5,7,8}
    F, C = 2, 21                                          # groups of 9, 9 and 3 channels
    pid = np.array([[0, 1, 1], [1, 0, 0]], dtype=np.uint8)
    mask = np.array([[1, 1, 1], [0, 1, 1]], dtype=np.uint8)
    m = B.group_mask_1x1(pid, mask, lib, F, C)
    assert m.shape == (F, C)
    assert list(np.nonzero(m[0])[0]) == [0, 1, 3, 4, 9 + 4, 9 + 5, 9 + 7, 9 + 8]      # tail group: taps 4.. do not exist
    assert list(np.nonzero(m[1])[0]) == [9 + 0, 9 + 1, 9 + 3, 9 + 4, 18 + 0, 18 + 1]  # taps 3, 4 of the tail do not exist
    with pytest.raises(ValueError):
        B.group_mask_1x1(np.full((F, 3), 2, np.uint8), mask, lib, F, C)


@pytest.mark.parametrize("stride", [1, 2])
def test_conv1x1_equals_loops_library_and_centre_tap_3x3(stride):
    N, C, F, H, W = 2, 21, 4, 5, 6
    lib = np.array([0x01B, 0x036, 0x0D8, 0x1B0], dtype=np.uint16)
    G = (C + 8) // 9
    x = RNG.standard_normal((N, C, H, W)).astype(np.float32)
    w = RNG.standard_normal((F, C)).astype(np.float32)
    b = RNG.standard_normal(F).astype(np.float32)
    pid = RNG.integers(0, 4, size=(F, G)).astype(np.uint8)
    mask = (RNG.random((F, G)) < 0.7).astype(np.uint8)
    y = B.conv1x1(x, w, pid, mask, lib, b, stride)
    m = B.group_mask_1x1(pid, mask, lib, F, C)
    # loops
    ref = np.zeros_like(y)
    for n, f, oy, ox in itertools.product(range(N), range(F), range(y.shape[2]), range(y.shape[3])):
        acc = float(b[f])
        for c in range(C):
            if m[f, c]:
                acc += float(w[f, c]) * float(x[n, c, oy * stride, ox * stride])
        ref[n, f, oy, ox] = acc
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    # the library's 1x1 convolution in float64 over the masked weights
    t = torch.nn.functional.conv2d(torch.tensor(x, dtype=torch.float64),
                                   torch.tensor((w * m).reshape(F, C, 1, 1), dtype=torch.float64),
                                   torch.tensor(b, dtype=torch.float64), stride=stride)
    np.testing.assert_allclose(y, t.numpy(), rtol=1e-12, atol=1e-12)
    # a 1x1 kernel is a 3x3 kernel with only its centre tap, at padding 1: the pinned forward oracle
    w9 = np.zeros((F, C, 3, 3), dtype=np.float32)
    w9[:, :, 1, 1] = w * m
    np.testing.assert_allclose(y, oracle.conv3x3(x, w9, b, stride, 1), rtol=1e-12, atol=1e-12)
    assert np.all(B.conv1x1(x, w, pid, mask, lib, b, stride, relu=True) == np.maximum(y, 0))
