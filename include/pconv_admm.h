/*
 * pconv_admm — the selection-variable steps of the pattern-aware pruning framework on the GPU.  C ABI, part of
 * libpconv.so, next to pconv.h (whose conventions, error codes and pconv_strerror apply).  These are the per-kernel
 * pieces of the framework that do not need a dataset: everything here is an independent small problem per 3x3
 * kernel, so a layer (or a whole network: VGG-16 has 1.6 million kernels) is one launch, one thread per kernel,
 * bound by HBM.  The training of the weights themselves (the primal step of the iteration, a DNN solver) is not part
 * of this library.
 *
 * Notation (paper, section 5.1): every kernel W_i has a selection vector z in R^K over the K patterns of the library,
 * an auxiliary copy u on the probability simplex, a multiplier mu, and the penalty rho > 0.  Vectors are stored one
 * kernel after the other: v[i*K + j], i < n, j < K; float storage; the arithmetic inside is double.
 *
 * All pointers except `lib` (and the size word of the selection's workspace) are DEVICE pointers, caller-owned;
 * `stream` is a hipStream_t passed as void* (NULL = the default stream); calls are asynchronous on it and allocate
 * nothing.  n = 0 is a no-op.  Non-finite inputs give
 * unspecified values (no fault).
 */
#ifndef PCONV_ADMM_H
#define PCONV_ADMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Proximal step and multiplier update of one ADMM iteration (section 5.1: the problem over u, its analytical
 * solution, and the update of mu):
 *     d      = z + mu / rho
 *     u      = [d - nu 1]_+   with nu the root of 1^T [d - nu 1]_+ = 1     (the point of the simplex nearest to d)
 *     mu_out = mu + rho (z - u)
 *   z, mu    in,  float[n*K]
 *   u        out, float[n*K], or NULL if only the multipliers are wanted
 *   mu_out   out, float[n*K], or NULL; may be the same buffer as mu (each kernel reads its vector before it writes)
 *   K        1..32;  rho > 0
 * With mu_out = NULL and mu a buffer of zeros (or mu = NULL, which means zeros) this is the plain projection of z.
 * PCONV_EINVAL for a null z, K outside 1..32, n < 0 or rho <= 0 (or not a number).
 */
int pconv_admm_proximal(const float* z, const float* mu, float rho, long long n, int K, float* u, float* mu_out,
                        void* stream);

/*
 * Projection of the relaxed selection onto one pattern (section 5.1, last problem: z_binary has its single one at
 * argmax_j z_j): pid[i] = that index; ties go to the lowest index.
 *   z    in,  float[n*K];  pid out, int32[n];  K 1..126
 */
int pconv_admm_binarize(const float* z, long long n, int K, int32_t* pid, void* stream);

/*
 * Pattern assignment on the device: for every 3x3 kernel the library pattern that keeps the most of its squared L2
 * norm -- the Euclidean projection of the kernel onto the kernels of each pattern is the masked kernel W o M_j
 * (sections 4.1, 5.1), so the nearest one is the one that retains the most energy.  Same rule and same arithmetic as
 * the host entry pconv_assign_patterns (squares and sums in double, taps ascending, nothing contracted, ties to the
 * lowest pattern id): the two agree bit for bit on finite weights.
 *   w      in,  device, n kernels of 9 weights each (w[i*9 + t], t = 3*ky + kx), storage type `dtype`
 *          (PCONV_F32 or PCONV_F16)
 *   lib    in,  HOST, uint16[K] 9-bit masks with exactly four bits set, K 1..126 (copied into the launch)
 *   pid    out, device, int32[n]
 * PCONV_EPATTERN for a bad mask or K, PCONV_EINVAL for null pointers, a bad dtype or n < 0.
 */
int pconv_assign_patterns_device(const void* w, int dtype, long long n, const uint16_t* lib, int K, int32_t* pid,
                                 void* stream);

/*
 * Connectivity selection on the device (sections 3 and 6.1: the kernels with the smallest L2 norm are cut): of the
 * n = F*C kernels of a layer, the k = floor(keep*n + 0.5) with the largest squared norm of the pattern-pruned kernel
 * W o M_pid are kept; equal norms go to the lower index f*C + c.  Same rule and arithmetic as the host entry
 * pconv_select_connectivity (norms in double, taps ascending): the two agree bit for bit on finite weights.
 * The selection is a stable radix sort of (norm, index) pairs (the hipCUB device primitive) between two small
 * kernels of this library.
 *   w          in,  device, n kernels of 9 weights, storage type `dtype`
 *   lib        in,  HOST, uint16[K]
 *   pid        in,  device, int32[n], every entry in [0, K) (not checked on the device: an entry outside reads
 *              an arbitrary mask of the library's storage, never outside it)
 *   keep       in [0, 1]
 *   mask       out, device, uint8[n]: 1 = kept
 *   workspace  device scratch of *workspace_bytes bytes, 256-byte aligned.  Called with workspace == NULL the
 *              function only writes the size it needs for this n to *workspace_bytes and returns PCONV_OK; it never
 *              allocates.  A workspace that is too small gives PCONV_ESCRATCH.
 */
int pconv_select_connectivity_device(const void* w, int dtype, long long n, const uint16_t* lib, int K,
                                     const int32_t* pid, double keep, uint8_t* mask, void* workspace,
                                     size_t* workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
