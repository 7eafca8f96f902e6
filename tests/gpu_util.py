"""Helpers shared by the GPU parity tests: run a layer through libpconv and through the oracle on the same bytes."""
from __future__ import annotations

import numpy as np

import oracle
import paper_2001_07710_amd as pc
from workloads import layers as L

TOL = {"f32": 1e-4, "f16": 2e-3}   # max relative error asked for fp32, and for fp16 storage with fp32 accumulation


def rel_err(g, r) -> float:
    """max_i |g_i - r_i| / max(|r_i|, rms(r)): element-relative for large outputs, rms-relative near zero crossings."""
    g = np.asarray(g, np.float64).reshape(-1)
    r = np.asarray(r, np.float64).reshape(-1)
    if r.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(r * r)))
    den = np.maximum(np.abs(r), max(rms, 1e-30))
    return float(np.max(np.abs(g - r) / den))


def sparsity(spec: L.LayerSpec, w):
    """Pattern ids and connectivity mask of a layer, by the library (product path) and by the oracle; both must agree
    bit for bit.  Returns (lib, pid, mask)."""
    lib = spec.library()
    w32 = np.asarray(w, np.float32)
    if spec.assign == "uniform":
        pid = L.gen_uniform_pattern_ids(spec)
    else:
        pid = pc.assign_patterns(w32, lib)
        assert np.array_equal(pid, oracle.assign_patterns(w32, lib)), "pattern assignment differs from the oracle"
    if spec.conn == "bernoulli":
        mask = L.gen_bernoulli_mask(spec)
    else:
        mask = pc.select_connectivity(w32, lib, pid, spec.keep)
        assert np.array_equal(mask, oracle.select_connectivity(w32, lib, pid, spec.keep)), "connectivity differs"
    return lib, pid, mask


class GpuLayer:
    """A packed layer resident on the GPU plus the host copies the oracle needs."""

    def __init__(self, spec: L.LayerSpec, w=None, bias=None, use_bias=True):
        import torch
        self.torch = torch
        self.spec = spec
        self.w = L.gen_weights(spec) if w is None else w
        self.bias = (L.gen_bias(spec) if bias is None else bias) if use_bias else None
        self.lib, self.pid, self.mask = sparsity(spec, self.w)
        self.packed = pc.pack(self.w, self.lib, self.pid, self.mask)
        self.d_bias = torch.from_numpy(self.bias).cuda() if self.bias is not None else None
        self.wm = oracle.mask_weights(self.w, self.pid, self.mask, self.lib)
        self.tdtype = torch.float16 if spec.dtype == "f16" else torch.float32

    def run(self, x_np, relu=None, canary=True, y_shift=0, x_shift=0, **tuning):
        """x_np [N][C][H][W] in the storage dtype -> numpy y [N][F][Ho][Wo] (storage dtype).  y_shift moves the
        output buffer by that many elements (an output pointer that is not 16-byte aligned), x_shift the input."""
        torch, s = self.torch, self.spec
        N = x_np.shape[0]
        relu = s.relu if relu is None else relu
        dx = torch.from_numpy(np.ascontiguousarray(x_np)).cuda()
        if x_shift:
            xbuf = torch.zeros(dx.numel() + x_shift, dtype=dx.dtype, device="cuda")
            xbuf[x_shift:] = dx.reshape(-1)
            dx = xbuf[x_shift:]
        n_out = N * s.F * s.Ho * s.Wo
        pad = (4096 if canary else 0) + y_shift
        buf = torch.full((n_out + 2 * pad,), -777.0, dtype=self.tdtype, device="cuda")
        dy = buf[pad:pad + n_out]
        flags = pc.FLAG_RELU if relu else 0
        st = torch.cuda.current_stream().cuda_stream
        if tuning:
            pc.conv3x3_tuned(dx, dy, self.packed, self.d_bias, N, s.H, s.W, s.stride, s.pad, flags, st, **tuning)
        else:
            pc.conv3x3(dx, dy, self.packed, self.d_bias, N, s.H, s.W, s.stride, s.pad, flags, st)
        torch.cuda.synchronize()
        out = buf.cpu().numpy()
        if canary:
            assert np.all(out[:pad] == -777.0) and np.all(out[pad + n_out:] == -777.0), "write outside the output buffer"
        return out[pad:pad + n_out].reshape(N, s.F, s.Ho, s.Wo)

    def oracle(self, x_np, relu=None):
        s = self.spec
        relu = s.relu if relu is None else relu
        return oracle.conv3x3(x_np, self.wm, self.bias, s.stride, s.pad, relu)

    def oracle_at(self, x_np, coords, relu=None):
        s = self.spec
        relu = s.relu if relu is None else relu
        return oracle.conv3x3_at(x_np, self.wm, coords, self.bias, s.stride, s.pad, relu)

    def free(self):
        self.packed.free()
