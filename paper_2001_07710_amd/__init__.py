"""Python binding of libpconv (pattern-sparse 3x3 convolution for MI355X).

Argument marshalling only: every step of the path runs inside the C-ABI library declared in include/pconv.h; the
functions here have the same names minus the `pconv_` prefix.  Host arrays are numpy arrays; device buffers are
anything with a `data_ptr()` (torch tensors on the GPU), used only for their address.  There is no CPU fallback: a
missing or broken library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

F32, F16 = 0, 1
FLAG_RELU = 1
FLAG_DENSE_DIRECT = 2
FLAG_NHWC = 4
PACK_HOST_ONLY = 1
KERNEL_AUTO, KERNEL_TILED, KERNEL_GENERIC, KERNEL_QUAD, KERNEL_MFMA = 0, 1, 2, 3, 4
ORDER_AUTO, ORDER_PLAIN, ORDER_BALANCED = 0, 1, 2
OK, EINVAL, EPATTERN, ESHAPE, EUNSUPPORTED, ENOMEM, EHIP, ESTATE, ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7, -8

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpconv.so")
PEAKS_LIB_PATH = os.path.join(_HERE, "libpconv_peaks.so")     # measured-peaks kernels, separate from the product
_lib = None


class PconvError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        text = _load().pconv_strerror(code).decode()
        hip = _load().pconv_last_hip_error().decode() if code == EHIP else ""
        super().__init__(f"{where}: {text} (code {code})" + (f" [{hip}]" if hip else ""))


class _Tuning(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int), ("rows", ctypes.c_int), ("filters_per_wave", ctypes.c_int),
                ("waves", ctypes.c_int), ("channels_per_wave", ctypes.c_int), ("channel_order", ctypes.c_int), ("channel_splits", ctypes.c_int), ("buffers", ctypes.c_int),
                ("slot_walk", ctypes.c_int), ("mfma_shape", ctypes.c_int), ("split_reduce", ctypes.c_int)]


def ensure_built() -> str:
    """Build the library if no built one is there (tests, smoke and bench call this; the binding itself never builds)."""
    if not os.path.exists(LIB_PATH) or not os.path.exists(PEAKS_LIB_PATH):
        from .build import build_library
        build_library()
    return LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, u = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint
    lib.pconv_assign_patterns.argtypes = [vp, i, i, vp, i, vp]
    lib.pconv_select_connectivity.argtypes = [vp, i, i, vp, i, vp, ctypes.c_double, vp]
    lib.pconv_pack.argtypes = [vp, i, i, i, vp, i, vp, vp, u, ctypes.POINTER(vp)]
    lib.pconv_packed_export.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_size_t)]
    lib.pconv_packed_import.argtypes = [vp, vp, vp, vp, i, i, i, vp, i, u, ctypes.POINTER(vp)]
    lib.pconv_packed_import.restype = i
    lib.pconv_packed_stats.argtypes = [vp, ctypes.POINTER(i), ctypes.POINTER(i), ctypes.POINTER(i), ctypes.POINTER(i),
                                       ctypes.POINTER(ctypes.c_size_t)]
    lib.pconv_packed_balance.argtypes = [vp, i, i, i, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.pconv_packed_balance.restype = i
    lib.pconv_packed_parity_form.argtypes = [vp, i, ctypes.POINTER(vp)]
    lib.pconv_packed_library.argtypes = [vp, vp]
    lib.pconv_free.argtypes = [vp]
    lib.pconv_free.restype = None
    lib.pconv_conv3x3.argtypes = [vp, vp, vp, vp, i, i, i, i, i, u, vp]
    lib.pconv_conv3x3_noalloc.argtypes = [vp, vp, vp, vp, i, i, i, i, i, u, vp]
    lib.pconv_noalloc_scratch_bytes.argtypes = []
    lib.pconv_noalloc_scratch_bytes.restype = ctypes.c_size_t
    lib.pconv_conv3x3_choice.argtypes = [vp, i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.pconv_conv3x3_choice.restype = i
    lib.pconv_conv3x3_tuned.argtypes = [vp, vp, vp, vp, i, i, i, i, i, u, vp, ctypes.POINTER(_Tuning)]
    lib.pconv_dense_conv3x3.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, i, u, vp]
    lib.pconv_maxpool2x2.argtypes = [vp, vp, i, i, i, i, i, vp]
    ll = ctypes.c_longlong
    lib.pconv_admm_proximal.argtypes = [vp, vp, ctypes.c_float, ll, i, vp, vp, vp]
    lib.pconv_admm_binarize.argtypes = [vp, ll, i, vp, vp]
    lib.pconv_assign_patterns_device.argtypes = [vp, i, ll, vp, i, vp, vp]
    lib.pconv_select_connectivity_device.argtypes = [vp, i, ll, vp, i, vp, ctypes.c_double, vp, vp,
                                                     ctypes.POINTER(ctypes.c_size_t), vp]
    for name in ("pconv_admm_proximal", "pconv_admm_binarize", "pconv_assign_patterns_device",
                 "pconv_select_connectivity_device"):
        getattr(lib, name).restype = i
    for name in ("pconv_assign_patterns", "pconv_select_connectivity", "pconv_pack", "pconv_packed_export",
                 "pconv_packed_stats", "pconv_packed_parity_form", "pconv_packed_library", "pconv_conv3x3", "pconv_conv3x3_noalloc", "pconv_conv3x3_tuned", "pconv_dense_conv3x3",
                 "pconv_maxpool2x2"):
        getattr(lib, name).restype = i
    lib.pconv_packed_transpose.argtypes = [vp, u, ctypes.POINTER(vp)]
    lib.pconv_conv3x3_grad_input.argtypes = [vp, vp, vp, i, i, i, vp]
    lib.pconv_conv3x3_grad_weight_workspace.argtypes = [vp, i, i, i, i, i, ctypes.POINTER(ctypes.c_size_t)]
    lib.pconv_conv3x3_grad_weight.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, ctypes.c_size_t, vp]
    lib.pconv_pack_1x1.argtypes = [vp, i, i, i, vp, i, vp, vp, u, ctypes.POINTER(vp)]
    lib.pconv_conv1x1.argtypes = [vp, vp, vp, vp, i, i, i, i, u, vp]
    for name in ("pconv_packed_transpose", "pconv_conv3x3_grad_input", "pconv_conv3x3_grad_weight_workspace",
                 "pconv_conv3x3_grad_weight", "pconv_pack_1x1", "pconv_conv1x1"):
        getattr(lib, name).restype = i
    lib.pconv_filter_similarity_order.argtypes = [vp, i, i, i, vp]
    lib.pconv_filter_similarity_order.restype = i
    lib.pconv_packed_mfma_blocks.argtypes = [vp, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.pconv_packed_mfma_blocks.restype = i
    lib.pconv_strerror.argtypes = [i]
    lib.pconv_strerror.restype = ctypes.c_char_p
    lib.pconv_last_hip_error.argtypes = []
    lib.pconv_last_hip_error.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(rc: int, where: str):
    if rc != OK:
        raise PconvError(rc, where)


def _host(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _dp(t):
    return None if t is None else int(t.data_ptr())


def _dtype_code(np_dtype) -> int:
    if np.dtype(np_dtype) == np.float32:
        return F32
    if np.dtype(np_dtype) == np.float16:
        return F16
    raise TypeError("storage type must be float32 or float16")


def peaks() -> dict:
    """Measured peaks of the current GPU (libpconv_peaks.so; see include/pconv_peaks.h)."""
    lib = ctypes.CDLL(PEAKS_LIB_PATH)
    d, i = ctypes.c_double, ctypes.c_int
    for name in ("pconv_peak_copy_gbs", "pconv_peak_fma_tflops", "pconv_peak_lds_read_bytes_per_clk",
                 "pconv_peak_vmem_clk_per_load", "pconv_peak_vmem_clk_per_store", "pconv_peak_mfma_f16_tflops"):
        getattr(lib, name).argtypes = [i]
        getattr(lib, name).restype = d
    lib.pconv_peak_device.argtypes = [ctypes.POINTER(i), ctypes.POINTER(d)]
    lib.pconv_peak_device.restype = i
    cus, mhz = i(0), d(0.0)
    if lib.pconv_peak_device(ctypes.byref(cus), ctypes.byref(mhz)) != 0:
        raise RuntimeError("pconv_peak_device failed")
    return {
        "compute_units": cus.value, "nominal_clock_MHz": mhz.value,
        "copy_GBs": {f"{m}MiB": lib.pconv_peak_copy_gbs(m) for m in (256, 1024)},
        "fp32_fma_TFLOPs": {f"{w}_waves_per_simd": lib.pconv_peak_fma_tflops(w) for w in (1, 2, 4)},
        "lds_read_b128_bytes_per_clk_per_cu": {f"{w}_waves": lib.pconv_peak_lds_read_bytes_per_clk(w) for w in (4, 8, 16)},
        "vmem_clk_per_wave_load": {f"{b}B_per_lane": lib.pconv_peak_vmem_clk_per_load(b) for b in (4, 16)},
        "vmem_clk_per_wave_store_16B_per_lane": {f"{w}_waves": lib.pconv_peak_vmem_clk_per_store(w) for w in (4, 16)},
        "mfma_f16_TFLOPs": {f"{w}_waves_per_simd": lib.pconv_peak_mfma_f16_tflops(w) for w in (1, 2)},
    }


def strerror(code: int) -> str:
    return _load().pconv_strerror(code).decode()


def assign_patterns(w_oihw, lib) -> np.ndarray:
    w = _host(w_oihw, np.float32)
    F, C = w.shape[:2]
    lb = _host(lib, np.uint16)
    pid = np.empty((F, C), dtype=np.uint8)
    _check(_load().pconv_assign_patterns(_hp(w), F, C, _hp(lb), int(lb.size), _hp(pid)), "pconv_assign_patterns")
    return pid


def select_connectivity(w_oihw, lib, pid, keep: float) -> np.ndarray:
    w = _host(w_oihw, np.float32)
    F, C = w.shape[:2]
    lb = _host(lib, np.uint16)
    pd = _host(pid, np.uint8)
    mask = np.empty((F, C), dtype=np.uint8)
    _check(_load().pconv_select_connectivity(_hp(w), F, C, _hp(lb), int(lb.size), _hp(pd), float(keep), _hp(mask)),
           "pconv_select_connectivity")
    return mask


class Packed:
    """Owner of a pconv_packed handle."""

    def __init__(self, handle: int, F: int, C: int, K: int, np_dtype):
        self.handle, self.F, self.C, self.K, self.np_dtype = handle, F, C, K, np.dtype(np_dtype)

    @property
    def n_kept(self) -> int:
        n = ctypes.c_size_t(0)
        _check(_load().pconv_packed_stats(self.handle, None, None, None, None, ctypes.byref(n)), "pconv_packed_stats")
        return int(n.value)

    def free(self):
        if self.handle:
            _load().pconv_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def pack(w_oihw, lib, pid, mask, flags: int = 0) -> Packed:
    w = np.ascontiguousarray(w_oihw)
    code = _dtype_code(w.dtype)
    F, C = w.shape[:2]
    lb = _host(lib, np.uint16)
    pd = _host(pid, np.uint8)
    mk = _host(mask, np.uint8)
    out = ctypes.c_void_p(None)
    _check(_load().pconv_pack(_hp(w), code, F, C, _hp(lb), int(lb.size), _hp(pd), _hp(mk), int(flags),
                              ctypes.byref(out)), "pconv_pack")
    return Packed(out.value, F, C, int(lb.size), w.dtype)


def packed_stats(p: Packed):
    F, C, K, dt = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    n = ctypes.c_size_t()
    _check(_load().pconv_packed_stats(p.handle, ctypes.byref(F), ctypes.byref(C), ctypes.byref(K), ctypes.byref(dt),
                                      ctypes.byref(n)), "pconv_packed_stats")
    return F.value, C.value, K.value, dt.value, int(n.value)


def packed_balance(p: Packed, waves: int, filters_per_wave: int, balanced: bool):
    """(mean kept kernels per wave and chunk, mean over chunks of the maximum over the waves)."""
    a, b = ctypes.c_double(), ctypes.c_double()
    _check(_load().pconv_packed_balance(p.handle, waves, filters_per_wave, int(balanced), ctypes.byref(a),
                                        ctypes.byref(b)), "pconv_packed_balance")
    return a.value, b.value


def packed_parity_form(p: Packed, pad: int) -> Packed:
    """The layer as the stride-2 path runs it (4*C parity-plane channels, kernels of one to four taps), host only."""
    out = ctypes.c_void_p(None)
    _check(_load().pconv_packed_parity_form(p.handle, int(pad), ctypes.byref(out)), "pconv_packed_parity_form")
    q = Packed(out.value, p.F, 4 * p.C, 0, p.np_dtype)
    q.K = packed_stats(q)[2]
    return q


def packed_library(p: Packed) -> np.ndarray:
    lib = np.empty(p.K, dtype=np.uint16)
    _check(_load().pconv_packed_library(p.handle, _hp(lib)), "pconv_packed_library")
    return lib


def packed_export(p: Packed):
    n = p.n_kept
    fo = np.empty(p.F, dtype=np.uint32)
    gp = np.empty(p.F * p.K + 1, dtype=np.uint32)
    cin = np.empty(n, dtype=np.uint16)
    w4 = np.empty((n, 4), dtype=p.np_dtype)
    nk = ctypes.c_size_t(0)
    _check(_load().pconv_packed_export(p.handle, _hp(fo), _hp(gp), _hp(cin), _hp(w4), ctypes.byref(nk)),
           "pconv_packed_export")
    assert nk.value == n
    return fo, gp, cin, w4


def packed_import(filter_order, grp_ptr, cin, w4, F: int, C: int, lib, flags: int = 0) -> Packed:
    """A packed layer from the arrays packed_export returns; w4's dtype (float32 or float16) is the layer's."""
    fo = np.ascontiguousarray(filter_order, dtype=np.uint32)
    gp = np.ascontiguousarray(grp_ptr, dtype=np.uint32)
    ci = np.ascontiguousarray(cin, dtype=np.uint16)
    w4 = np.ascontiguousarray(w4)
    lb = np.ascontiguousarray(lib, dtype=np.uint16)
    code = _dtype_code(w4.dtype)
    if fo.size != F or gp.size != F * lb.size + 1 or ci.size < int(gp[-1]) or w4.size < 4 * int(gp[-1]):
        raise ValueError("array sizes do not fit F, K and grp_ptr's last entry")
    out = ctypes.c_void_p(None)
    _check(_load().pconv_packed_import(_hp(fo), _hp(gp), _hp(ci) if ci.size else None, _hp(w4) if w4.size else None,
                                       code, F, C, _hp(lb), int(lb.size), flags, ctypes.byref(out)),
           "pconv_packed_import")
    return Packed(out.value, F, C, int(lb.size), w4.dtype)


def conv3x3(x, y, wp: Packed, bias, N: int, H: int, W: int, stride: int = 1, pad: int = 1, flags: int = 0,
            stream: int = 0):
    _check(_load().pconv_conv3x3(_dp(x), _dp(y), wp.handle, _dp(bias), N, H, W, stride, pad, flags, stream or None),
           "pconv_conv3x3")


def conv3x3_noalloc(x, y, wp: Packed, bias, N: int, H: int, W: int, stride: int = 1, pad: int = 1, flags: int = 0,
                    stream: int = 0):
    _check(_load().pconv_conv3x3_noalloc(_dp(x), _dp(y), wp.handle, _dp(bias), N, H, W, stride, pad, flags,
                                         stream or None), "pconv_conv3x3_noalloc")


def conv3x3_choice(wp: Packed, N: int, H: int, W: int, stride: int = 1, pad: int = 1):
    """(kernel family, tile shape of the matrix-core kernel or 0) that conv3x3 takes for this shape."""
    k, sh = ctypes.c_int(0), ctypes.c_int(0)
    _check(_load().pconv_conv3x3_choice(wp.handle, N, H, W, stride, pad, ctypes.byref(k), ctypes.byref(sh)),
           "pconv_conv3x3_choice")
    return k.value, sh.value


def noalloc_scratch_bytes() -> int:
    return int(_load().pconv_noalloc_scratch_bytes())


def conv3x3_tuned(x, y, wp: Packed, bias, N: int, H: int, W: int, stride: int = 1, pad: int = 1, flags: int = 0,
                  stream: int = 0, kernel: int = 0, rows: int = 0, filters_per_wave: int = 0, waves: int = 0,
                  channels_per_wave: int = 0, channel_order: int = 0, channel_splits: int = 0, buffers: int = 0,
                  slot_walk: int = 0, mfma_shape: int = 0, split_reduce: int = 0):
    t = _Tuning(kernel, rows, filters_per_wave, waves, channels_per_wave, channel_order, channel_splits, buffers,
                slot_walk, mfma_shape, split_reduce)
    _check(_load().pconv_conv3x3_tuned(_dp(x), _dp(y), wp.handle, _dp(bias), N, H, W, stride, pad, flags,
                                       stream or None, ctypes.byref(t)), "pconv_conv3x3_tuned")


def dense_conv3x3(x, y, w_oihw_dev, bias, dtype: int, N: int, C: int, F: int, H: int, W: int, stride: int = 1,
                  pad: int = 1, flags: int = 0, stream: int = 0):
    _check(_load().pconv_dense_conv3x3(_dp(x), _dp(y), _dp(w_oihw_dev), _dp(bias), dtype, N, C, F, H, W, stride, pad,
                                       flags, stream or None), "pconv_dense_conv3x3")


def maxpool2x2(x, y, dtype: int, N: int, C: int, H: int, W: int, stream: int = 0):
    _check(_load().pconv_maxpool2x2(_dp(x), _dp(y), dtype, N, C, H, W, stream or None), "pconv_maxpool2x2")


# ---- the selection-variable steps of the pruning framework (include/pconv_admm.h); device tensors in, device tensors out

def admm_proximal(z, mu, rho: float, n: int, K: int, u=None, mu_out=None, stream: int = 0):
    _check(_load().pconv_admm_proximal(_dp(z), _dp(mu), float(rho), n, K, _dp(u), _dp(mu_out), stream),
           "pconv_admm_proximal")


def admm_binarize(z, n: int, K: int, pid, stream: int = 0):
    _check(_load().pconv_admm_binarize(_dp(z), n, K, _dp(pid), stream), "pconv_admm_binarize")


def assign_patterns_device(w, dtype: int, n: int, lib, pid, stream: int = 0):
    lib_h = _host(lib, np.uint16)
    _check(_load().pconv_assign_patterns_device(_dp(w), dtype, n, _hp(lib_h), int(lib_h.size), _dp(pid), stream),
           "pconv_assign_patterns_device")


def select_connectivity_device_workspace(n: int) -> int:
    """Bytes of device scratch pconv_select_connectivity_device needs for n kernels."""
    need = ctypes.c_size_t(0)
    _check(_load().pconv_select_connectivity_device(None, F32, n, None, 0, None, 0.0, None, None, ctypes.byref(need), None),
           "pconv_select_connectivity_device (size query)")
    return int(need.value)


def select_connectivity_device(w, dtype: int, n: int, lib, pid, keep: float, mask, workspace, workspace_bytes: int,
                               stream: int = 0):
    lib_h = _host(lib, np.uint16)
    have = ctypes.c_size_t(workspace_bytes)
    _check(_load().pconv_select_connectivity_device(_dp(w), dtype, n, _hp(lib_h), int(lib_h.size), _dp(pid), float(keep),
                                                    _dp(mask), _dp(workspace), ctypes.byref(have), stream),
           "pconv_select_connectivity_device")


# ---- pconv_backward.h: backward pass of the pruned layer, 1x1 layers grouped into 3x3 patterns

def packed_transpose(p: Packed, flags: int = 0) -> Packed:
    out = ctypes.c_void_p(None)
    _check(_load().pconv_packed_transpose(p.handle, int(flags), ctypes.byref(out)), "pconv_packed_transpose")
    return Packed(out.value, p.C, p.F, p.K, p.np_dtype)


def conv3x3_grad_input(dy, dx, wpt: Packed, N: int, H: int, W: int, stream: int = 0):
    _check(_load().pconv_conv3x3_grad_input(_dp(dy), _dp(dx), wpt.handle, N, H, W, stream or None),
           "pconv_conv3x3_grad_input")


def conv3x3_grad_weight_workspace(p: Packed, N: int, H: int, W: int, stride: int = 1, pad: int = 1) -> int:
    n = ctypes.c_size_t(0)
    _check(_load().pconv_conv3x3_grad_weight_workspace(p.handle, N, H, W, stride, pad, ctypes.byref(n)),
           "pconv_conv3x3_grad_weight_workspace")
    return int(n.value)


def conv3x3_grad_weight(x, dy, p: Packed, dw4, N: int, H: int, W: int, stride: int = 1, pad: int = 1, workspace=None,
                        workspace_bytes: int = 0, stream: int = 0):
    _check(_load().pconv_conv3x3_grad_weight(_dp(x), _dp(dy), p.handle, _dp(dw4), N, H, W, stride, pad,
                                             _dp(workspace), int(workspace_bytes), stream or None),
           "pconv_conv3x3_grad_weight")


def pack_1x1(w_fc, lib, pid, mask, flags: int = 0) -> Packed:
    w = np.ascontiguousarray(w_fc)
    code = _dtype_code(w.dtype)
    F, C = w.shape
    lb = _host(lib, np.uint16)
    pd = _host(pid, np.uint8)
    mk = _host(mask, np.uint8)
    out = ctypes.c_void_p(None)
    _check(_load().pconv_pack_1x1(_hp(w), code, F, C, _hp(lb), int(lb.size), _hp(pd), _hp(mk), int(flags),
                                  ctypes.byref(out)), "pconv_pack_1x1")
    return Packed(out.value, F, C, 1, w.dtype)


def conv1x1(x, y, wp: Packed, bias, N: int, H: int, W: int, stride: int = 1, flags: int = 0, stream: int = 0):
    _check(_load().pconv_conv1x1(_dp(x), _dp(y), wp.handle, _dp(bias), N, H, W, stride, flags, stream or None),
           "pconv_conv1x1")


def filter_similarity_order(mask, group: int) -> np.ndarray:
    mk = _host(mask, np.uint8)
    F, C = mk.shape
    out = np.empty(F, dtype=np.uint32)
    _check(_load().pconv_filter_similarity_order(_hp(mk), F, C, int(group), _hp(out)), "pconv_filter_similarity_order")
    return out


def packed_mfma_blocks(p: Packed, tile_filters: int):
    """(channel blocks that the matrix-core kernel multiplies over all filter tiles, what it would be without lists)."""
    a, b = ctypes.c_int(), ctypes.c_int()
    _check(_load().pconv_packed_mfma_blocks(p.handle, int(tile_filters), ctypes.byref(a), ctypes.byref(b)),
           "pconv_packed_mfma_blocks")
    return a.value, b.value
