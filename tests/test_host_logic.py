"""CPU-side tests of libpconv: the library loads and exports what include/pconv.h declares; pattern assignment,
connectivity selection and packing agree bit for bit with the oracle; bad arguments give the documented codes.
No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    pc.ensure_built()


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "pconv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(pconv_[a-z0-9_]+)\s*\(", hdr))
    assert {"pconv_pack", "pconv_conv3x3", "pconv_assign_patterns", "pconv_select_connectivity", "pconv_free",
            "pconv_packed_export", "pconv_dense_conv3x3", "pconv_maxpool2x2", "pconv_conv3x3_tuned"} <= names
    lib = ctypes.CDLL(pc.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in pconv.h but not exported"


def test_peaks_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "pconv_peaks.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(pconv_peak_[a-z0-9_]+)\s*\(", hdr))
    assert len(names) == 7
    lib = ctypes.CDLL(pc.PEAKS_LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in pconv_peaks.h but not exported"


def test_admm_entry_points_are_exported_and_refuse_bad_arguments_without_a_gpu():
    hdr = open(os.path.join(ROOT, "include", "pconv_admm.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(pconv_[a-z0-9_]+)\s*\(", hdr))
    assert names == {"pconv_admm_proximal", "pconv_admm_binarize", "pconv_assign_patterns_device",
                     "pconv_select_connectivity_device"}
    lib = ctypes.CDLL(pc.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in pconv_admm.h but not exported"
    # argument checks come before any device call (no compute here: every call below returns before a launch)
    vp, ll, i = ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int
    lib.pconv_admm_proximal.argtypes = [vp, vp, ctypes.c_float, ll, i, vp, vp, vp]
    lib.pconv_admm_binarize.argtypes = [vp, ll, i, vp, vp]
    lib.pconv_assign_patterns_device.argtypes = [vp, i, ll, vp, i, vp, vp]
    fake = 4096                                             # never dereferenced by the calls below
    assert lib.pconv_admm_proximal(None, None, 1.0, 4, 8, fake, None, None) == pc.EINVAL
    assert lib.pconv_admm_proximal(fake, None, 0.0, 4, 8, fake, None, None) == pc.EINVAL
    assert lib.pconv_admm_proximal(fake, None, float("nan"), 4, 8, fake, None, None) == pc.EINVAL
    assert lib.pconv_admm_proximal(fake, None, 1.0, 4, 33, fake, None, None) == pc.EINVAL
    assert lib.pconv_admm_proximal(fake, None, 1.0, -1, 8, fake, None, None) == pc.EINVAL
    assert lib.pconv_admm_proximal(fake, None, 1.0, 0, 8, fake, None, None) == pc.OK       # nothing to do
    assert lib.pconv_admm_binarize(fake, 4, 0, fake, None) == pc.EINVAL
    assert lib.pconv_admm_binarize(fake, 0, 8, fake, None) == pc.OK
    good = np.array([0x01B, 0x036], dtype=np.uint16)
    bad = np.array([0x01B, 0x007], dtype=np.uint16)
    assert lib.pconv_assign_patterns_device(fake, pc.F32, 4, bad.ctypes.data, 2, fake, None) == pc.EPATTERN
    assert lib.pconv_assign_patterns_device(fake, pc.F32, 4, good.ctypes.data, 0, fake, None) == pc.EPATTERN
    assert lib.pconv_assign_patterns_device(fake, 7, 4, good.ctypes.data, 2, fake, None) == pc.EINVAL
    assert lib.pconv_assign_patterns_device(fake, pc.F32, 0, good.ctypes.data, 2, fake, None) == pc.OK


def _layer(spec):
    w = L.gen_weights(spec)
    lib = spec.library()
    return w, lib


@pytest.mark.parametrize("spec", [L.config0(), L.shrink(L.config1(), C=64, F=48), L.config2()[0],
                                  L.shrink(L.config3(1)[0], C=32, F=40), L.shrink(L.config4(12, 0.15)[3], C=24, F=56)],
                         ids=["cfg0", "cfg1s", "cfg2_conv1_1", "cfg3s_f16", "cfg4s_K12"])
def test_assign_select_pack_bit_exact(spec):
    w, lib = _layer(spec)
    w32 = w.astype(np.float32)
    if spec.assign == "uniform":
        pid = L.gen_uniform_pattern_ids(spec)
    else:
        pid = pc.assign_patterns(w32, lib)
        assert np.array_equal(pid, oracle.assign_patterns(w32, lib))
    if spec.conn == "bernoulli":
        mask = L.gen_bernoulli_mask(spec)
    else:
        mask = pc.select_connectivity(w32, lib, pid, spec.keep)
        assert np.array_equal(mask, oracle.select_connectivity(w32, lib, pid, spec.keep))
        assert mask.sum() == spec.n_keep_target()
    p = pc.pack(w, lib, pid, mask, pc.PACK_HOST_ONLY)
    assert pc.packed_stats(p) == (spec.F, spec.C, spec.K, pc.F16 if spec.dtype == "f16" else pc.F32, int(mask.sum()))
    got = pc.packed_export(p)
    exp = oracle.pack_canonical(w, pid, mask, lib)
    for g, e, name in zip(got, exp, ("filter_order", "grp_ptr", "cin", "w4")):
        assert g.dtype == e.dtype and g.shape == e.shape, name
        assert g.tobytes() == e.tobytes(), name
    # round trip: unpack(pack(W)) == W o M, bit for bit
    back = oracle.unpack_canonical(*got, lib, spec.F, spec.C)
    assert back.tobytes() == oracle.mask_weights(w, pid, mask, lib).tobytes()
    p.free()


def test_full_size_config1_assignment_and_selection():
    spec = L.config1()
    w, lib = _layer(spec)
    pid = pc.assign_patterns(w, lib)
    assert np.array_equal(pid, oracle.assign_patterns(w, lib))
    mask = pc.select_connectivity(w, lib, pid, spec.keep)
    assert np.array_equal(mask, oracle.select_connectivity(w, lib, pid, spec.keep))
    assert mask.sum() == 18350
    # every library pattern is in use, roughly uniformly (the draw is from one family of masks)
    hist = np.bincount(pid.reshape(-1), minlength=8)
    assert hist.min() > 0.05 * pid.size


def test_ties_and_special_values():
    lib = np.asarray(L.FIXED4, np.uint16)
    w = np.ones((3, 4, 3, 3), np.float32)
    assert np.all(pc.assign_patterns(w, lib) == 0)
    w[1, 2] = 0
    w[1, 2, 2, 2] = 5
    assert pc.assign_patterns(w, lib)[1, 2] == 3
    # equal scores: the lowest linear index wins
    pid = pc.assign_patterns(np.ones((3, 4, 3, 3), np.float32), lib)
    mask = pc.select_connectivity(np.ones((3, 4, 3, 3), np.float32), lib, pid, 5 / 12)
    assert mask.reshape(-1).tolist() == [1] * 5 + [0] * 7
    # -0.0 and NaN payloads survive packing
    wh = np.zeros((1, 1, 3, 3), np.float16)
    wh.view(np.uint16)[0, 0, 0, 0] = 0x8000
    wh.view(np.uint16)[0, 0, 0, 1] = 0x7E01
    p = pc.pack(wh, lib, np.zeros((1, 1), np.uint8), np.ones((1, 1), np.uint8), pc.PACK_HOST_ONLY)
    w4 = pc.packed_export(p)[3]
    assert w4.view(np.uint16).reshape(-1).tolist() == [0x8000, 0x7E01, 0, 0]


def test_empty_and_full_masks():
    spec = L.shrink(L.config1(), C=10, F=6)
    w, lib = _layer(spec)
    pid = pc.assign_patterns(w, lib)
    for mask in (np.zeros((6, 10), np.uint8), np.ones((6, 10), np.uint8)):
        p = pc.pack(w, lib, pid, mask, pc.PACK_HOST_ONLY)
        got = pc.packed_export(p)
        exp = oracle.pack_canonical(w, pid, mask, lib)
        assert all(g.tobytes() == e.tobytes() for g, e in zip(got, exp))
        assert p.n_kept == int(mask.sum())
    assert pc.select_connectivity(w, lib, pid, 0.0).sum() == 0
    assert pc.select_connectivity(w, lib, pid, 1.0).sum() == 60


def test_error_codes():
    lib = np.asarray(L.FIXED4, np.uint16)
    w = np.zeros((2, 3, 3, 3), np.float32)
    pid = np.zeros((2, 3), np.uint8)
    mask = np.ones((2, 3), np.uint8)

    def code(fn, *a, **k):
        with pytest.raises(pc.PconvError) as ei:
            fn(*a, **k)
        return ei.value.code

    assert code(pc.assign_patterns, w, np.asarray([0x00F, 0x007], np.uint16)) == pc.EPATTERN        # three bits
    assert code(pc.assign_patterns, w, np.asarray([0x20F], np.uint16)) == pc.EPATTERN               # bit above the ninth
    assert code(pc.assign_patterns, w, np.zeros(0, np.uint16)) == pc.EPATTERN                       # K = 0
    assert code(pc.assign_patterns, w, np.asarray([0x01B] * 127, np.uint16)) == pc.EPATTERN          # K > 126
    bad_pid = pid.copy()
    bad_pid[1, 1] = 4
    assert code(pc.pack, w, lib, bad_pid, mask, pc.PACK_HOST_ONLY) == pc.EPATTERN
    mask0 = mask.copy()
    mask0[1, 1] = 0                                                                                  # ... ignored when removed
    pc.pack(w, lib, bad_pid, mask0, pc.PACK_HOST_ONLY).free()
    assert code(pc.select_connectivity, w, lib, bad_pid, 0.5) == pc.EPATTERN
    assert code(pc.select_connectivity, w, lib, pid, 1.5) == pc.EINVAL
    assert code(pc.pack, w, lib, pid, mask, 2) == pc.EINVAL
    raw = pc._load()
    assert raw.pconv_pack(None, 0, 2, 3, lib.ctypes.data, 4, pid.ctypes.data, mask.ctypes.data, 1,
                          ctypes.byref(ctypes.c_void_p())) == pc.EINVAL
    assert raw.pconv_pack(w.ctypes.data, 7, 2, 3, lib.ctypes.data, 4, pid.ctypes.data, mask.ctypes.data, 1,
                          ctypes.byref(ctypes.c_void_p())) == pc.EINVAL
    assert raw.pconv_pack(w.ctypes.data, 0, 0, 3, lib.ctypes.data, 4, pid.ctypes.data, mask.ctypes.data, 1,
                          ctypes.byref(ctypes.c_void_p())) == pc.ESHAPE
    assert raw.pconv_pack(w.ctypes.data, 0, 2, 65536, lib.ctypes.data, 4, pid.ctypes.data, mask.ctypes.data, 1,
                          ctypes.byref(ctypes.c_void_p())) == pc.ESHAPE
    # argument checks of the device entry points come before any HIP call, so they can be exercised here
    p = pc.pack(w, lib, pid, mask, pc.PACK_HOST_ONLY)
    one = ctypes.c_void_p(16)
    f = raw.pconv_conv3x3
    assert f(None, one, p.handle, None, 1, 8, 8, 1, 1, 0, None) == pc.EINVAL
    assert f(one, one, p.handle, None, 1, 8, 8, 3, 1, 0, None) == pc.EUNSUPPORTED
    assert f(one, one, p.handle, None, 1, 8, 8, 1, 2, 0, None) == pc.EUNSUPPORTED
    assert f(one, one, p.handle, None, 1, 0, 8, 1, 1, 0, None) == pc.ESHAPE
    assert f(one, one, p.handle, None, 1, 2, 2, 1, 0, 0, None) == pc.ESHAPE           # no output
    assert f(one, one, p.handle, None, 1, 8, 8, 1, 1, 64, None) == pc.EINVAL          # unknown flag
    assert f(one, one, p.handle, None, 1, 8, 8, 1, 1, pc.FLAG_NHWC, None) in (pc.EUNSUPPORTED, pc.ESTATE)   # fp32 layer
    assert f(one, one, p.handle, None, 1, 8, 8, 1, 1, 0, None) == pc.ESTATE           # host-only handle
    assert f(one, one, None, None, 1, 8, 8, 1, 1, 0, None) == pc.EINVAL
    assert raw.pconv_maxpool2x2(one, one, 0, 1, 1, 1, 8, None) == pc.ESHAPE
    assert raw.pconv_dense_conv3x3(one, one, None, None, 0, 1, 1, 1, 8, 8, 1, 1, 0, None) == pc.EINVAL
    assert "pattern" in pc.strerror(pc.EPATTERN)
    p.free()
    raw.pconv_free(None)


def test_balanced_staging_order_evens_out_the_waves():
    spec = L.shrink(L.config1(), C=128, F=64)
    w, lib = _layer(spec)
    pid = pc.assign_patterns(w, lib)
    mask = pc.select_connectivity(w, lib, pid, spec.keep)
    p = pc.pack(w, lib, pid, mask, pc.PACK_HOST_ONLY)
    for waves, nf in ((16, 2), (16, 1), (8, 1)):
        mean_plain, max_plain = pc.packed_balance(p, waves, nf, False)
        mean_bal, max_bal = pc.packed_balance(p, waves, nf, True)
        # same kernels, same number of wave-chunks: the mean cannot move; the slowest wave per chunk gets faster
        assert abs(mean_plain - mean_bal) < 1e-9
        assert max_bal <= max_plain and max_bal >= mean_bal
        assert mean_bal / max_bal > 0.8
    with pytest.raises(pc.PconvError):
        pc.packed_balance(p, 4, 1, True)
    p.free()


@pytest.mark.parametrize("pad", [0, 1])
@pytest.mark.parametrize("hw", [(9, 11), (8, 6)])
def test_parity_form_of_a_stride2_layer_computes_the_same_function(pad, hw):
    """The re-packed layer that the stride-2 path runs, checked on the CPU against the definition: the oracle's
    stride-2 convolution of x equals its stride-1 convolution of the four parity planes of x with the re-packed
    weights."""
    H, W = hw
    spec = L.LayerSpec(cfg=12, idx=pad, name="s2", N=2, C=10, F=12, H=H, W=W, stride=2, pad=pad, K=8, keep=0.5)
    w, lib = _layer(spec)
    pid = pc.assign_patterns(w, lib)
    mask = pc.select_connectivity(w, lib, pid, spec.keep)
    p = pc.pack(w, lib, pid, mask, pc.PACK_HOST_ONLY)
    q = pc.packed_parity_form(p, pad)
    F, C4, K2, _, n2 = pc.packed_stats(q)
    assert (F, C4) == (spec.F, 4 * spec.C) and 1 <= K2 <= 255
    lib2 = pc.packed_library(q)
    assert np.all(np.diff(lib2.astype(int)) > 0)
    bits = np.array([[(int(m) >> t) & 1 for t in range(9)] for m in lib2])
    assert np.all((bits.sum(axis=1) >= 1) & (bits.sum(axis=1) <= 4)) and np.all(bits[:, [2, 5, 6, 7, 8]] == 0)
    fo, gp, cin, w4 = pc.packed_export(q)
    w2 = np.zeros((F, C4, 9), np.float32)
    n_taps = 0
    for i in range(F):
        for j in range(K2):
            taps = np.nonzero(bits[j])[0]
            for e in range(int(gp[i * K2 + j]), int(gp[i * K2 + j + 1])):
                w2[int(fo[i]), int(cin[e]), taps] = w4[e][:len(taps)]
                assert np.all(w4[e][len(taps):] == 0)
                n_taps += len(taps)
    assert n_taps == 4 * int(mask.sum())          # every kept tap went to exactly one plane kernel
    x = L.gen_activations(spec)
    Hs, Ws = (H + 1) // 2, (W + 1) // 2
    planes = np.zeros((spec.N, spec.C, 4, Hs + 1, Ws + 1), np.float32)   # one spare zero row/column for pad 0
    for a in range(2):
        for b in range(2):
            sub = x[:, :, a::2, b::2]
            planes[:, :, 2 * a + b, :sub.shape[2], :sub.shape[3]] = sub
    planes = planes.reshape(spec.N, C4, Hs + 1, Ws + 1)
    ref = oracle.pattern_conv3x3(x, w, pid, mask, lib, None, 2, pad)
    via = oracle.conv3x3(planes, w2.reshape(F, C4, 3, 3), None, 1, pad)[:, :, :ref.shape[2], :ref.shape[3]]
    assert via.shape == ref.shape
    assert np.max(np.abs(via - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    q.free()
    p.free()
