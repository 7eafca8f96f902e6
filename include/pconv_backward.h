/*
 * pconv_backward — the backward pass of the pruned 3x3 layer and the 1x1 layer grouped into 3x3 patterns.  C ABI,
 * part of libpconv.so, next to pconv.h (whose conventions, handle type, error codes and pconv_strerror apply).
 *
 * Backward pass.  The pruning framework trains the weights through the pruned layer (paper, section 5.1: the primal
 * step minimises the loss over W o M by SGD, and the non-zero weights go on being trained after the patterns are
 * fixed).  For y = conv(x, W o M), with dy = dL/dy:
 *     dL/dx[n][c][iy][ix]   = sum over f and the kept taps (ky,kx) of kernel (f,c) of
 *                             w[f][c][ky][kx] * dy[n][f][oy][ox],  oy*stride + ky - pad = iy, ox*stride + kx - pad = ix
 *     dL/dW[f][c][ky][kx]   = sum over n, oy, ox of dy[n][f][oy][ox] * x[n][c][oy*stride+ky-pad][ox*stride+kx-pad]
 *                             for the kept taps of kept kernels, zero elsewhere (dL/dW = G o M)
 * At stride 1 and padding 1 the input gradient is itself a pruned 3x3 layer over dy: filters and channels exchanged,
 * every kernel and its mask rotated by 180 degrees.  pconv_packed_transpose builds that layer once per weight
 * update; pconv_conv3x3_grad_input is then the forward kernel.  The weight gradient is a contraction over the
 * pixels; it runs on the matrix cores (fp16 storage) and returns the gradients of the kept weights in the order of
 * the canonical packed form.
 *
 * 1x1 layers.  Section 3 of the paper handles 1x1 layers by grouping 1x1 kernels into 3x3 ones and applying the
 * patterns to those.  Reading taken here: for filter f the input channels 9g .. 9g+8 are the nine positions (tap
 * t = c - 9g) of group g; the group's pattern keeps four of them; connectivity pruning removes whole groups; a last
 * group that C does not fill keeps the kept taps that exist.
 *
 * Device pointers are caller-owned; `stream` is a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef PCONV_BACKWARD_H
#define PCONV_BACKWARD_H

#include <stddef.h>
#include <stdint.h>

#include "pconv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The layer whose forward pass at stride 1, padding 1 is the input gradient of `p` at stride 1, padding 1 (see
 * above): F' = C, C' = F, kernel (c,f) = kernel (f,c) rotated by 180 degrees (tap t -> 8 - t), pattern j of its
 * library = pattern j of p's rotated, same pattern ids, connectivity transposed.  Host work like pconv_pack, same
 * flags, same upload; the caller frees the result with pconv_free.
 * PCONV_EUNSUPPORTED for handles that are not layers from pconv_pack (parity forms, 1x1 layers); PCONV_ESHAPE if
 * F >= 65536.
 */
int pconv_packed_transpose(const pconv_packed* p, unsigned flags, pconv_packed** out);

/*
 * dx = dL/dx from dy at stride 1, padding 1 (section 5.1, primal step): the forward kernels on the transposed layer.
 *   dy   in,  device, [N][F][H][W] in the layer's storage type
 *   dx   out, device, [N][C][H][W], same type; must not overlap dy
 *   wpt  pconv_packed_transpose(layer)
 * Errors, asynchrony and hidden allocations are those of pconv_conv3x3.
 */
int pconv_conv3x3_grad_input(const void* dy, void* dx, const pconv_packed* wpt, int N, int H, int W, void* stream);

/*
 * dL/dW of the kept weights (section 5.1, primal step; see above), fp16 storage, stride 1, padding 1:
 *   x     in,  device, [N][C][H][W] fp16       the layer's input
 *   dy    in,  device, [N][F][H][W] fp16       gradient of its output
 *   p     the layer (from pconv_pack, with a device copy on the current device)
 *   dw4   out, device, float[n_kept][4]: entry e, slot q = gradient of the weight that the canonical form
 *         (pconv_packed_export) holds at w4[e][q]; fp32 accumulation over all pixels, not rounded to fp16
 *   workspace, workspace_bytes   device scratch of at least pconv_conv3x3_grad_weight_workspace() bytes (partial
 *         sums of the workgroups that share a tile); the call allocates nothing
 * The result is deterministic (fixed summation order).  Asynchronous on `stream`.
 * PCONV_EUNSUPPORTED: fp32 storage, stride 2, padding 0, an image of 2 GiB or more, or a handle that is not a layer
 * from pconv_pack.  PCONV_EINVAL: null or odd pointers, a workspace that is too small.  PCONV_ESTATE: no device copy
 * on the current device.  N = 0 gives zeros.
 */
int pconv_conv3x3_grad_weight_workspace(const pconv_packed* p, int N, int H, int W, int stride, int pad, size_t* bytes);
int pconv_conv3x3_grad_weight(const void* x, const void* dy, const pconv_packed* p, float* dw4, int N, int H, int W,
                              int stride, int pad, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Packs a pruned 1x1 layer (section 3; reading above).
 *   w_fc   host, F*C weights [F][C], storage type `dtype`
 *   lib, K the 3x3 pattern library, as for pconv_pack
 *   pid    host, uint8[F][G], G = ceil(C / 9): pattern of group g of filter f
 *   mask   host, uint8[F][G]: 1 = the group is kept
 * The handle is a 3x3 layer whose kept kernels hold their centre tap only: pconv_packed_export lists, per filter,
 * the kept channels ascending with the weight bit-identical in w4[e][0] (slots 1..3 zero), K = 1.  Errors as
 * pconv_pack.  For fp16 storage and C a multiple of 64 the handle holds the matrix-core kernel's copy of the weights
 * twice (the second time with the channels in four ranges that the kernel walks like taps): 2 * 2 * F * C bytes more
 * on the device.
 */
int pconv_pack_1x1(const void* w_fc, int dtype, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
                   const uint8_t* mask, unsigned flags, pconv_packed** out);

/*
 * The pruned 1x1 layer: y[n][f][oy][ox] = bias[f] + sum over kept weights (f,c) of w[f][c] * x[n][c][oy*stride][ox*stride],
 * Ho = floor((H-1)/stride) + 1, Wo likewise.  Arguments, flags, errors and asynchrony as pconv_conv3x3 (it is that
 * call at padding 1 on the centre-tap layer); PCONV_ESTATE if wp is not from pconv_pack_1x1.
 */
int pconv_conv1x1(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H, int W, int stride,
                  unsigned flags, void* stream);

#ifdef __cplusplus
}
#endif

#endif /* PCONV_BACKWARD_H */
