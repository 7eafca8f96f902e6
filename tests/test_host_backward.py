"""CPU-side tests of the entry points of pconv_backward.h: the library exports what the header declares; the
transposed layer and the packed 1x1 layer match the oracle bit for bit; the claim behind the transposed layer (its
forward pass is the input gradient) holds between two oracle functions; argument checks."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
RNG = np.random.default_rng(77100120)
LIB8 = np.array([0x01B, 0x036, 0x0D8, 0x1B0, 0x03A, 0x0B8, 0x0B2, 0x09A], dtype=np.uint16)


def rotate(m: int) -> int:
    return int(format(int(m), "09b")[::-1], 2)


def test_library_exports_every_symbol_of_the_header():
    hdr = open(os.path.join(ROOT, "include", "pconv_backward.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(pconv_[a-z0-9_]+)\s*\(", hdr))
    assert {"pconv_packed_transpose", "pconv_conv3x3_grad_input", "pconv_conv3x3_grad_weight",
            "pconv_conv3x3_grad_weight_workspace", "pconv_pack_1x1", "pconv_conv1x1"} <= names
    lib = ctypes.CDLL(pc.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in pconv_backward.h but not exported"


def _layer(F, C, dtype, keep=0.4):
    w = (RNG.standard_normal((F, C, 3, 3)) * 0.1).astype(dtype)
    pid = oracle.assign_patterns(w.astype(np.float32), LIB8)
    mask = (RNG.random((F, C)) < keep).astype(np.uint8)
    return w, pid, mask


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("fc", [(5, 7), (33, 20), (64, 64)])
def test_transposed_layer_is_the_oracles_pack_of_the_rotated_layer(dtype, fc):
    F, C = fc
    w, pid, mask = _layer(F, C, dtype)
    p = pc.pack(w, LIB8, pid, mask, pc.PACK_HOST_ONLY)
    t = pc.packed_transpose(p, pc.PACK_HOST_ONLY)
    assert pc.packed_stats(t)[:3] == (C, F, 8)
    lib_t = np.array([rotate(m) for m in LIB8], dtype=np.uint16)
    assert np.array_equal(pc.packed_library(t), lib_t)
    w_t = np.ascontiguousarray(w.transpose(1, 0, 2, 3)[:, :, ::-1, ::-1])
    ref = oracle.pack_canonical(w_t, pid.T, mask.T, lib_t)
    got = pc.packed_export(t)
    for a, b in zip(got, ref):
        assert a.dtype == b.dtype and a.tobytes() == b.tobytes()
    t.free()
    p.free()


def test_forward_pass_of_the_rotated_layer_is_the_input_gradient():
    # what pconv_conv3x3_grad_input relies on, checked between the forward oracle and the gradient oracle
    F, C, N, H, W = 6, 5, 2, 7, 9
    w, pid, mask = _layer(F, C, np.float32)
    wm = oracle.mask_weights(w, pid, mask, LIB8)
    dy = RNG.standard_normal((N, F, H, W)).astype(np.float32)
    lib_t = np.array([rotate(m) for m in LIB8], dtype=np.uint16)
    w_t = np.ascontiguousarray(w.transpose(1, 0, 2, 3)[:, :, ::-1, ::-1])
    wm_t = oracle.mask_weights(w_t, pid.T, mask.T, lib_t)
    np.testing.assert_allclose(oracle.conv3x3(dy, wm_t, None, 1, 1), oracle.conv3x3_grad_input(dy, wm, H, W, 1, 1),
                               rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("fc", [(4, 21), (9, 9), (17, 100), (3, 5)])
def test_packed_1x1_layer_lists_the_oracles_kept_weights(dtype, fc):
    F, C = fc
    G = (C + 8) // 9
    w = (RNG.standard_normal((F, C)) * 0.1).astype(dtype)
    w[0, 0] = -0.0
    pid = RNG.integers(0, 8, size=(F, G)).astype(np.uint8)
    mask = (RNG.random((F, G)) < 0.6).astype(np.uint8)
    p = pc.pack_1x1(w, LIB8, pid, mask, pc.PACK_HOST_ONLY)
    m = oracle.group_mask_1x1(pid, mask, LIB8, F, C)
    fo, gp, cin, w4 = pc.packed_export(p)
    assert pc.packed_stats(p)[:3] == (F, C, 1) and p.n_kept == int(m.sum())
    counts = m.sum(axis=1).astype(np.int64)
    assert np.array_equal(fo, np.lexsort((np.arange(F), -counts)).astype(np.uint32))
    for i, f in enumerate(fo):
        a, b = int(gp[i]), int(gp[i + 1])
        kept = np.nonzero(m[f])[0]
        assert np.array_equal(cin[a:b], kept.astype(np.uint16))
        assert w4[a:b, 0].tobytes() == w[f, kept].tobytes()          # bit for bit, -0.0 included
        assert not np.any(w4[a:b, 1:].view(np.uint16 if dtype == np.float16 else np.uint32))
    assert list(pc.packed_library(p)) == [0x010]
    p.free()


def test_argument_checks():
    lib = pc._load()
    w, pid, mask = _layer(4, 4, np.float32)
    p = pc.pack(w, LIB8, pid, mask, pc.PACK_HOST_ONLY)
    out = ctypes.c_void_p(None)
    assert lib.pconv_packed_transpose(None, 0, ctypes.byref(out)) == pc.EINVAL
    assert lib.pconv_packed_transpose(p.handle, 8, ctypes.byref(out)) == pc.EINVAL
    par = pc.packed_parity_form(p, 1)
    assert lib.pconv_packed_transpose(par.handle, 1, ctypes.byref(out)) == pc.EUNSUPPORTED
    n = ctypes.c_size_t(0)
    f = lib.pconv_conv3x3_grad_weight_workspace
    assert f(p.handle, 1, 8, 8, 1, 1, ctypes.byref(n)) == pc.EUNSUPPORTED          # fp32 storage
    wh, pidh, maskh = _layer(4, 4, np.float16)
    ph = pc.pack(wh, LIB8, pidh, maskh, pc.PACK_HOST_ONLY)
    assert f(ph.handle, 1, 8, 8, 2, 1, ctypes.byref(n)) == pc.EUNSUPPORTED         # stride 2
    assert f(ph.handle, 1, 8, 8, 1, 0, ctypes.byref(n)) == pc.EUNSUPPORTED         # padding 0
    assert f(ph.handle, 1, 0, 8, 1, 1, ctypes.byref(n)) == pc.ESHAPE
    assert f(ph.handle, 2, 8, 8, 1, 1, ctypes.byref(n)) == pc.OK and n.value > 0
    one = ctypes.c_void_p(4096)
    g = lib.pconv_conv3x3_grad_weight
    assert g(one, one, ph.handle, one, 1, 8, 8, 1, 1, one, n.value, None) == pc.ESTATE   # host-only handle
    assert g(None, one, ph.handle, one, 1, 8, 8, 1, 1, one, n.value, None) == pc.EINVAL
    w1 = np.zeros((2, 9), np.float32)
    bad = np.full((2, 1), 9, np.uint8)
    assert lib.pconv_pack_1x1(w1.ctypes.data, pc.F32, 2, 9, LIB8.ctypes.data, 8, bad.ctypes.data,
                              np.ones((2, 1), np.uint8).ctypes.data, pc.PACK_HOST_ONLY, ctypes.byref(out)) == pc.EPATTERN
    assert lib.pconv_conv1x1(one, one, p.handle, None, 1, 8, 8, 1, 0, None) == pc.ESTATE     # not a 1x1 layer
    for h in (par, ph, p):
        h.free()
