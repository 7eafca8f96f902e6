"""CPU oracle for the backward pass of the pruned 3x3 layer and for the 1x1 layer whose kernels are grouped into
3x3 patterns.

TEST INFRASTRUCTURE ONLY: imported by tests and the bench's cpu_baseline leg, never by the product path, with which
it shares no code.  Plain numpy, float64, the definitions written out tap by tap; no blocking or reordering.

The primal step of the pruning framework (section 5.1 of the paper) trains the weights through the pruned layer
y = conv(x, W o M): the loss reaches W only through W o M, so dL/dW = G o M with G the weight gradient of the dense
convolution, and dL/dx is the adjoint of the convolution with the masked weights.  With
    y[n,f,oy,ox] = sum_{c,ky,kx} Wm[f,c,ky,kx] * x[n,c,oy*s+ky-p, ox*s+kx-p]        (zero outside the image)
the two gradients for a given dy = dL/dy are
    dx[n,c,iy,ix]   = sum_{f,ky,kx} Wm[f,c,ky,kx] * dy[n,f,oy,ox]   over the (oy,ox) with oy*s+ky-p = iy, ox*s+kx-p = ix
    G[f,c,ky,kx]    = sum_{n,oy,ox} dy[n,f,oy,ox] * x[n,c,oy*s+ky-p, ox*s+kx-p]

Section 3 of the paper handles 1x1 layers by grouping 1x1 kernels into 3x3 ones and applying the patterns to those;
the reading taken here: for filter f the input channels 9g .. 9g+8 are the nine positions (tap t = c - 9g) of group
g, a pattern keeps four of them, connectivity pruning removes whole groups, and a last group that C does not fill
keeps only the taps that exist.
"""
from __future__ import annotations

import numpy as np


def _out_hw(H: int, W: int, stride: int, pad: int):
    return (H + 2 * pad - 3) // stride + 1, (W + 2 * pad - 3) // stride + 1


def conv3x3_grad_input(dy, wm, H: int, W: int, stride: int = 1, pad: int = 1) -> np.ndarray:
    """dx [N][C][H][W] (float64) from dy [N][F][Ho][Wo] and the masked dense weights wm [F][C][3][3]: every output
    element hands wm * dy back to the input element it read."""
    dy = np.asarray(dy, dtype=np.float64)
    wm = np.asarray(wm, dtype=np.float64)
    N, F, Ho, Wo = dy.shape
    C = wm.shape[1]
    assert wm.shape == (F, C, 3, 3) and (Ho, Wo) == _out_hw(H, W, stride, pad)
    padded = np.zeros((N, C, H + 2 * pad + 2, W + 2 * pad + 2), dtype=np.float64)   # (room for every tap's window)
    for ky in range(3):
        for kx in range(3):
            # input element (oy*s + ky - p, ox*s + kx - p) sits at padded position (oy*s + ky, ox*s + kx)
            contrib = np.einsum("nfhw,fc->nchw", dy, wm[:, :, ky, kx])
            padded[:, :, ky:ky + stride * Ho:stride, kx:kx + stride * Wo:stride] += contrib
    return np.ascontiguousarray(padded[:, :, pad:pad + H, pad:pad + W])


def conv3x3_grad_weight(x, dy, stride: int = 1, pad: int = 1) -> np.ndarray:
    """G [F][C][3][3] (float64), the weight gradient of the dense convolution, from x [N][C][H][W] and
    dy [N][F][Ho][Wo]."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    N, C, H, W = x.shape
    F, Ho, Wo = dy.shape[1:]
    assert dy.shape[0] == N and (Ho, Wo) == _out_hw(H, W, stride, pad)
    padded = np.zeros((N, C, H + 2 * pad + 2, W + 2 * pad + 2), dtype=np.float64)
    padded[:, :, pad:pad + H, pad:pad + W] = x
    G = np.zeros((F, C, 3, 3), dtype=np.float64)
    for ky in range(3):
        for kx in range(3):
            window = padded[:, :, ky:ky + stride * Ho:stride, kx:kx + stride * Wo:stride]   # x at (oy*s+ky-p, ...)
            G[:, :, ky, kx] = np.einsum("nfhw,nchw->fc", dy, window)
    return G


def conv3x3_grad_weight_at(x, dy, coords, stride: int = 1, pad: int = 1) -> np.ndarray:
    """The same sum for the listed weights only: coords [npts][4] = (f, c, ky, kx); float64 [npts].  For layers too
    large to take the whole gradient of."""
    x = np.asarray(x)
    dy = np.asarray(dy)
    N, C, H, W = x.shape
    Ho, Wo = dy.shape[2:]
    out = np.zeros(len(coords), dtype=np.float64)
    for i, (f, c, ky, kx) in enumerate(np.asarray(coords, dtype=np.int64).reshape(-1, 4)):
        # output rows and columns whose tap (ky, kx) lies inside the image
        oy = np.arange(Ho)
        ox = np.arange(Wo)
        oy = oy[(oy * stride + ky - pad >= 0) & (oy * stride + ky - pad < H)]
        ox = ox[(ox * stride + kx - pad >= 0) & (ox * stride + kx - pad < W)]
        a = dy[:, f][:, oy][:, :, ox].astype(np.float64)
        b = x[:, c][:, oy * stride + ky - pad][:, :, ox * stride + kx - pad].astype(np.float64)
        out[i] = np.sum(a * b)
    return out


def masked_grad_weight(x, dy, pid, mask, lib, stride: int = 1, pad: int = 1) -> np.ndarray:
    """G o M: the gradient of the weights that the layer keeps, zero elsewhere (float64 [F][C][3][3])."""
    from .pattern_oracle import mask_weights
    G = conv3x3_grad_weight(x, dy, stride, pad)
    return mask_weights(G, pid, mask, lib)


def group_mask_1x1(pid, mask, lib, F: int, C: int) -> np.ndarray:
    """[F][C] of 0/1: which weights of a 1x1 layer survive when channels 9g..9g+8 of a filter are read as the nine
    positions of a 3x3 kernel with pattern lib[pid[f][g]], and groups with mask[f][g] = 0 are removed."""
    from .pattern_oracle import library_bits
    bits = library_bits(lib)
    G = (C + 8) // 9
    pid = np.asarray(pid).reshape(F, G).astype(np.int64)
    keep = np.asarray(mask).reshape(F, G) != 0
    if np.any(pid[keep] >= bits.shape[0]):
        raise ValueError("pattern id outside the library")
    sel = bits[np.where(keep, pid, 0)] * keep[:, :, None]                 # [F][G][9]
    return sel.reshape(F, G * 9)[:, :C].astype(np.uint8)


def conv1x1(x, w, pid, mask, lib, bias=None, stride: int = 1, relu: bool = False) -> np.ndarray:
    """The pruned 1x1 layer: y[n,f,oy,ox] = b[f] + sum_c (w o M)[f,c] * x[n,c,oy*s,ox*s]; float64."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    F, C = w.shape
    wm = w * group_mask_1x1(pid, mask, lib, F, C)
    y = np.einsum("fc,nchw->nfhw", wm, x[:, :, ::stride, ::stride])
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :, None, None]
    return np.maximum(y, 0.0) if relu else y
