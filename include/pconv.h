/*
 * pconv — pattern-sparse 3x3 convolution for AMD MI355X (gfx950).  C ABI.
 *
 * The operation is the forward 3x3 convolution of a layer pruned with pattern-based sparsity:
 *   - pattern sparsity: every surviving 3x3 kernel keeps exactly four of its nine weights, at the positions of one
 *     binary mask M_j out of a small pattern library {M_1..M_K}; pruning is the element-wise product W o M_j
 *     (paper, sections 3, 4.1 and eq. (1) of section 5.1);
 *   - connectivity sparsity: whole kernels between an input channel c and an output filter f are removed
 *     (paper, sections 3 and 6.1).
 * The result is exactly that of a dense convolution whose weight tensor carries explicit zeros.
 *
 * Conventions used by every entry point
 *   - weights are OIHW, contiguous: w[f][c][ky][kx], F filters, C channels (section 6.1 names them F and C);
 *   - the tap index of a kernel position is t = 3*ky + kx; a pattern mask is a 9-bit integer with bit t set where the
 *     weight is kept; the convolution does not flip the kernel (cross-correlation);
 *   - activations are NCHW, contiguous; Ho = floor((H + 2*pad - 3)/stride) + 1, likewise Wo; positions outside the
 *     image read as zero;
 *   - dtype is the STORAGE type of x, y and w (PCONV_F32 or PCONV_F16); sums are always accumulated in fp32, the
 *     bias is always fp32, fp16 results are rounded to nearest even once, at the store;
 *   - every function returns PCONV_OK (0) or a negative error code; nothing throws; distinct handles may be used
 *     from distinct threads.  Process-wide state is limited to three per-device caches behind mutexes: the number of
 *     compute units, the address of the fixed scratch array of pconv_conv3x3_noalloc, and the weight buffer of
 *     pconv_dense_conv3x3 for fp16 storage;
 *   - "host" / "device" in a parameter comment says where the pointer must point.  Device buffers are owned by the
 *     caller; the library owns what it allocates behind a pconv_packed handle until pconv_free.
 */
#ifndef PCONV_H
#define PCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pconv_packed pconv_packed; /* opaque packed layer */

enum { PCONV_F32 = 0, PCONV_F16 = 1 };

enum {
    PCONV_OK = 0,
    PCONV_EINVAL = -1,       /* null pointer, bad enum or flag */
    PCONV_EPATTERN = -2,     /* library mask without exactly four bits in its low nine, K outside [1,126], pattern id >= K */
    PCONV_ESHAPE = -3,       /* zero or negative extent, C >= 65536, empty output, size overflow */
    PCONV_EUNSUPPORTED = -4, /* stride not 1 or 2, pad not 0 or 1 */
    PCONV_ENOMEM = -5,       /* host or device allocation failed */
    PCONV_EHIP = -6,         /* a HIP call failed (pconv_last_hip_error() has the runtime's text) */
    PCONV_ESTATE = -7,       /* handle was packed host-only and has no device copy, or (pconv_conv3x3_noalloc) lacks
                                a form of the layer that only an allocating call can build */
    PCONV_ESCRATCH = -8      /* pconv_conv3x3_noalloc: the launch needs more scratch than the fixed arena holds */
};

enum { PCONV_FLAG_RELU = 1u,        /* conv flags: y = max(y, 0) after the bias */
       PCONV_FLAG_DENSE_DIRECT = 2u, /* pconv_dense_conv3x3 only: the plain direct kernel also for fp16 storage */
       PCONV_FLAG_NHWC = 4u         /* pconv_conv3x3 and its variants: x is [N][H][W][C], y is [N][Ho][Wo][F] (below) */ };
enum { PCONV_PACK_HOST_ONLY = 1u }; /* pack flags: build the packed form on the host, allocate nothing on the device */

/*
 * Pattern assignment (host).  For every kernel picks the library mask that keeps the largest part of the kernel's
 * squared L2 norm, i.e. the Euclidean projection of the kernel onto the library — the hard one-hot selection that
 * ends section 5.1 of the paper.  Squares and sums are taken in double, taps ascending; ties go to the lowest index.
 *   w_oihw   host, float[F*C*9]
 *   lib      host, uint16[K], each with exactly four of the low nine bits set
 *   pid_out  host, uint8[F*C], written
 * K must be in [1,126].
 */
int pconv_assign_patterns(const float* w_oihw, int F, int C, const uint16_t* lib, int K, uint8_t* pid_out);

/*
 * Connectivity selection (host).  Scores every kernel by the squared L2 norm that its assigned pattern keeps (the
 * connectivity score gamma of section 6.1, squared, on the pattern-pruned kernel) and keeps the
 * k = floor(keep*F*C + 0.5) kernels of the layer with the largest score; ties by ascending index f*C + c.
 *   pid       host, uint8[F*C] (from pconv_assign_patterns or the caller's own)
 *   keep      fraction in [0,1]
 *   mask_out  host, uint8[F*C], written: 1 = kernel kept, 0 = removed
 */
int pconv_select_connectivity(const float* w_oihw, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
                              double keep, uint8_t* mask_out);

/*
 * Pack: dense weights + per-kernel pattern id + connectivity mask -> pattern-grouped compressed weights.  This is
 * the filter/kernel re-ordering and compact weight storage of section 6.2, in this library's own layout: filters
 * ordered by kept-kernel count, and inside a filter the kernels with the same pattern stored together.
 *   w_oihw   host, dtype-typed [F*C*9]; weights are copied bit for bit, entries outside the pattern are ignored
 *   dtype    PCONV_F32 or PCONV_F16: type of w_oihw here and of x and y in pconv_conv3x3
 *   pid      host, uint8[F*C]; entries of removed kernels are ignored
 *   mask     host, uint8[F*C]; non-zero = kept
 *   flags    0, or PCONV_PACK_HOST_ONLY
 *   out      receives the handle; release with pconv_free
 * Unless PCONV_PACK_HOST_ONLY is given, the packed arrays are copied to the current HIP device (synchronously) and
 * the handle is tied to that device.
 */
int pconv_pack(const void* w_oihw, int dtype, int F, int C, const uint16_t* lib, int K, const uint8_t* pid,
               const uint8_t* mask, unsigned flags, pconv_packed** out);

/*
 * Canonical packed form, for inspection, storage and bit-exact comparison (all host pointers, caller-allocated):
 *   filter_order uint32[F]      filters by (kept count descending, filter index ascending)
 *   grp_ptr      uint32[F*K+1]  grp_ptr[i*K+j] .. grp_ptr[i*K+j+1] = entries of filter filter_order[i] with mask j
 *   cin          uint16[n_kept] input channel of each entry, ascending inside a group
 *   w4           dtype[n_kept*4] the four kept weights of each entry, taps ascending, bit-identical to the input
 *   n_kept       receives the number of kept kernels
 * Any array pointer may be NULL to skip it (call once with all NULL to learn n_kept).
 */
int pconv_packed_export(const pconv_packed* p, uint32_t* filter_order, uint32_t* grp_ptr, uint16_t* cin, void* w4,
                        size_t* n_kept);

/*
 * A packed layer from its canonical form (the arrays pconv_packed_export writes, all host pointers, not kept after the
 * call; lib and K as in pconv_pack, dtype the type of w4): the stored form of a pruned layer (section 6.2's compact
 * weight storage) read back.  The handle is the one pconv_pack makes from the weights the arrays describe, so
 * pconv_packed_export of it returns the same arrays bit for bit when they were canonical; filter_order may be any
 * permutation of the filters (it is put into the canonical order).  PCONV_EINVAL for a filter_order that is no
 * permutation, a grp_ptr that does not start at 0 or descends, a channel >= C, channels that do not ascend inside a
 * group or come twice in one filter; the other codes as pconv_pack.  flags: 0 or PCONV_PACK_HOST_ONLY.
 */
int pconv_packed_import(const uint32_t* filter_order, const uint32_t* grp_ptr, const uint16_t* cin, const void* w4,
                        int dtype, int F, int C, const uint16_t* lib, int K, unsigned flags, pconv_packed** out);

/* Shape of a packed layer; any output pointer may be NULL. */
int pconv_packed_stats(const pconv_packed* p, int* F, int* C, int* K, int* dtype, size_t* n_kept);

/*
 * Load balance of the tiled kernel's staging order (introspection, host).  The waves of a workgroup meet at a barrier
 * after every chunk of 32 staged channels, so the wave with the most kept kernels in a chunk sets the pace.  For the
 * tiling (waves, filters_per_wave) this returns the mean number of kept kernels per wave and chunk and the mean,
 * over workgroups and chunks, of the maximum over the waves; their ratio is the share of the multiply phase that an
 * average wave spends working.  balanced = 0: channels staged in their own order; 1: in the balanced order computed
 * at pack time (PCONV_EUNSUPPORTED if the handle has none for this tiling).
 */
int pconv_packed_balance(const pconv_packed* p, int waves, int filters_per_wave, int balanced, double* mean_per_wave,
                         double* mean_of_max);

/*
 * Introspection of the stride-2 path.  A stride-2 layer runs as a stride-1 layer over the four row/column parity
 * planes of its input: input channel 4*c + 2*a + b of that form is the plane x[c][2i+a][2j+b], and tap (ky,kx) of
 * kernel (f,c) becomes tap (ky',kx') of kernel (f, 4*c + 2*a + b) with a = (ky-pad) mod 2, ky' = floor((ky-pad)/2)
 * + pad (columns likewise); a four-tap kernel thus falls apart into up to four kernels of one to four taps, 4*F*C
 * kernels in all.  pconv_packed_parity_form returns that layer as a new host-only handle (the caller frees it with
 * pconv_free); its canonical arrays come from pconv_packed_export, its masks (one to four bits each, ascending, at
 * most 255) from pconv_packed_library.  pad is 0 or 1.
 *   lib_out  host, uint16_t[K] with K from pconv_packed_stats
 */
int pconv_packed_parity_form(const pconv_packed* p, int pad, pconv_packed** out);
int pconv_packed_library(const pconv_packed* p, uint16_t* lib_out);

/*
 * Filter re-ordering by similarity (section 6.2 of the paper: filters with similar kernels are grouped together so that
 * a group's work is compact and regular).  On this chip the unit that matters is the tile of `group` consecutive
 * filters that one workgroup computes (128 or 64 for fp16 storage, 32 or 16 for fp32): a tile only stages the input
 * channels that some filter of it keeps, so filters that keep the same channels belong into one tile.  This returns
 * an order of the filters, group after group of `group` filters: a group starts with the not yet placed filter that
 * keeps the most kernels (lowest index among equals) and then takes, one at a time, the filter that adds the fewest
 * channels to the union of the group's kept channels (among equals the one that shares the most channels with it,
 * then the lowest index).  The caller applies it: row order_out[i] of weights, pattern ids and mask becomes filter i
 * of the layer it packs, output channel i of that layer is the original filter order_out[i] (a renaming that the
 * next layer's input channels absorb, as in the paper's compiler).  Host only; O(F^2 C / 64).
 *   mask       host, uint8[F*C], 1 = kept
 *   order_out  host, uint32[F]: a permutation of 0..F-1
 */
int pconv_filter_similarity_order(const uint8_t* mask, int F, int C, int group, uint32_t* order_out);

/*
 * Introspection of the matrix-core path (fp16 storage).  A workgroup tile of `tile_filters` (128 or 64) filters takes
 * the input channels in blocks of 16.  Where the filters of the layer's tiles keep only part of the channels, pconv_pack
 * gives every tile the list of the channels it keeps, and the kernel stages and multiplies those blocks only:
 * listed_blocks is the number of blocks over all tiles that are multiplied, all_blocks = tiles * ceil(C / 16) what
 * it would be without lists (equal when the layer has none: lists are made where they save a tenth or more).
 * PCONV_EUNSUPPORTED for fp32 storage or another tile height.
 */
int pconv_packed_mfma_blocks(const pconv_packed* p, int tile_filters, int* listed_blocks, int* all_blocks);

/* Releases host and device memory of a handle (NULL is allowed).  The caller makes sure no launch still uses it. */
void pconv_free(pconv_packed* p);

/*
 * The pruned layer (section 3; the computation the paper's inference framework of section 6.2 accelerates):
 *   y[n][f][oy][ox] = bias[f] + sum over kept kernels (f,c), over the four taps t of their pattern, of
 *                     w[f][c][t] * x[n][c][oy*stride + ky - pad][ox*stride + kx - pad]
 * optionally followed by max(.,0).  Asynchronous on `stream`.
 *   x       device, dtype[N*C*H*W], read only; must not overlap y
 *   y       device, dtype[N*F*Ho*Wo], every element written
 *           (x and y need the alignment of one element only; the automatic choice uses the kernels with 64- and
 *           128-bit accesses where x is aligned to 4 bytes -- stride 2: to two elements -- and y to 16 bytes, as
 *           device allocations are)
 *   wp      handle from pconv_pack (with a device copy, on the current device)
 *   bias    device, float[F], or NULL for no bias
 *   stride  1 or 2;  pad 0 or 1
 *   flags   0, PCONV_FLAG_RELU, PCONV_FLAG_NHWC or both
 *   stream  a hipStream_t passed as void* (NULL = the default stream)
 * Launch errors are returned; execution errors surface at the caller's next synchronisation.  N = 0 is a no-op.
 *
 * Channel-minor layout.  With PCONV_FLAG_NHWC x is dtype[N][H][W][C] and y dtype[N][Ho][Wo][F]: the order in which the
 * matrix-core kernel keeps activations on chip, so they travel from memory to LDS without passing registers.  fp16
 * storage only, C and F multiples of 8 (pad a three-channel input to eight), x and y aligned to 16 bytes, and a layer
 * without per-tile channel lists (pconv_packed_mfma_blocks reports equal counts); PCONV_EUNSUPPORTED otherwise.
 *
 * Workspace.  When a layer has too few output tiles to occupy the GPU (small batch, small feature map) the library
 * splits the input channels of each tile over several workgroups, which add their partial sums in a workspace that
 * belongs to the handle; the sum is taken in a fixed order, so results are reproducible run to run.  The workspace
 * is allocated (hipMalloc, which synchronises) the first time a shape needs it and kept until pconv_free; a later
 * call with the same or a smaller shape allocates nothing.  Because of it, calls that share one handle must not
 * overlap in time: issue them on one stream, or order them with events.
 *
 * Other work hidden in a first call.  The first stride-2 call on a handle (per padding) re-packs the layer over the
 * four parity planes of the input on the host and uploads it (hipMalloc and synchronous copies); a stride-2 call with
 * an odd H or W, or with a tiling other than the automatic one, also allocates a buffer for the input split into
 * planes.  When the workspace or that buffer has to grow it is freed and allocated anew (hipFree waits for the
 * device), so addresses recorded in a HIP graph captured before the growth are stale: run every shape once before
 * capturing, or use pconv_conv3x3_noalloc.
 */
int pconv_conv3x3(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H, int W, int stride,
                  int pad, unsigned flags, void* stream);

/*
 * pconv_conv3x3 for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same results bit for bit (with one exception: an fp16 layer whose
 * tiles the library itself chose to split, and whose partial sums do not fit the fixed array, runs unsplit here --
 * the same sums added in another order, within the tolerance of the type); the call makes no hipMalloc, hipFree or
 * other allocating call.  Where pconv_conv3x3 would split the input channels of a tile over several workgroups, the
 * partial sums and arrival counters live in a fixed device array of pconv_noalloc_scratch_bytes() bytes (24 MiB
 * of partial sums and 16384 tile counters) that every GPU the library runs on holds until the process ends, instead
 * of the handle's workspace; the counters the launch uses are cleared by a small kernel on `stream` first.
 *   - a launch whose split needs more than that returns PCONV_ESCRATCH and launches nothing (on the VGG-16 and
 *     ResNet-50 shapes the split is taken at small batch only and needs at most 8 MiB);
 *   - stride 2 needs the layer re-packed over parity planes, which pconv_conv3x3 builds (and allocates) on its first
 *     stride-2 call with that padding on the handle: without it this call returns PCONV_ESTATE; an odd H or W would
 *     also need a plane buffer and returns PCONV_ESCRATCH unless an earlier allocating call left one large enough;
 *   - all calls on one GPU share that GPU's array, whatever their handle: calls that overlap in time on one GPU race
 *     (issue them on one stream, or order them with events).
 */
int pconv_conv3x3_noalloc(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H, int W,
                          int stride, int pad, unsigned flags, void* stream);
size_t pconv_noalloc_scratch_bytes(void);

/*
 * pconv_conv3x3 with the kernel choice in the caller's hands, for tuning sweeps and for tests that must reach every
 * kernel.  A NULL `tuning`, or a field left 0, means "choose automatically" (what pconv_conv3x3 does).
 *   kernel            PCONV_KERNEL_TILED (one input column per lane, activations staged in LDS; stride 2 through
 *                     the parity form of the layer, see pconv_packed_parity_form), PCONV_KERNEL_QUAD (four input
 *                     columns per lane, for layers with many output tiles: unit stride, W a multiple of 4 and at
 *                     most 256; of the fields below it reads filters_per_wave (1 or 2), channel_order (balanced
 *                     orders exist for 16-channel chunks), channel_splits (0 = 1, or 2 or 4 where that evens out the
 *                     rounds of workgroups over the CUs) and slot_walk) or PCONV_KERNEL_GENERIC (any
 *                     stride and pad, straight from global memory).  Automatic: QUAD where it applies and has at
 *                     least 200 workgroups of its own, else TILED, else GENERIC
 *   rows              tiled: output rows held per lane (7)
 *   filters_per_wave  tiled: filters accumulated at once by one wave (1 or 2)
 *   waves             tiled: waves per workgroup, 1..16
 *   channels_per_wave tiled: channels each wave stages per chunk (1, 2 or 4); waves * channels_per_wave, the
 *                     channels resident in LDS at a time, must be a multiple of 16
 *   channel_order     tiled: PCONV_ORDER_PLAIN stages the input channels in their own order; PCONV_ORDER_BALANCED
 *                     uses the per-workgroup order computed at pack time that gives every wave the same number of
 *                     kept kernels per chunk (exists for waves x filters_per_wave = 16x2, 16x1, 8x1 with 32
 *                     channels per chunk); PCONV_ORDER_AUTO takes the balanced order where it exists.
 *                     Stride 2 with even H and W and waves = 16, channels_per_wave = 2 reads the parity planes
 *                     straight from x, channels in their own order (PLAIN or AUTO); PCONV_ORDER_BALANCED, any
 *                     other tiling, or an odd H or W splits x into planes in a pass of its own first
 *   channel_splits    tiled: workgroups that share one output tile, each taking a contiguous range of the channel
 *                     chunks (1 = no split, no workspace; at most the number of chunks; 0 = as many as give one
 *                     round of workgroups over the GPU's compute units)
 *   buffers           tiled: 1 = one chunk buffer in LDS and two barriers per chunk; 2 = two buffers of 16
 *                     channels (waves * channels_per_wave must be 16) and one barrier per chunk, the LDS writes of
 *                     one chunk running beside the multiply-adds of the chunk before
 *   slot_walk         quad (with two filters per wave: fp16 storage only; pad 1, y aligned to 16 bytes, no channel
 *                     split): 2 = one workgroup per CU and filter group walks over the output tiles, loading the next
 *                     tile's first chunk while it multiplies and stores the current tile (a layer whose channels fit
 *                     one chunk of 16, a network's first layer, also keeps its entries in LDS); 1 = one workgroup per
 *                     tile; 0 = walk if there are at least 1.5 tiles per workgroup (one chunk), or two and an
 *                     estimate of both forms' run time favours it (several chunks)
 *   mfma_shape        PCONV_KERNEL_MFMA (fp16 storage only; any stride and pad): the layer as a dense contraction
 *                     over its masked weights on the matrix cores, the automatic choice for fp16 storage.  Workgroup
 *                     tile: 0 = chosen by the library, 1 = 128 filters x 448 output pixels, 2 = 64 x 448,
 *                     3 = 128 x 224, 4 = 64 x 224.  `rows` (0 = as many as fit) caps the output rows per tile;
 *                     slot_walk = 1 gives every tile a workgroup of its own instead of persistent workgroups that
 *                     walk over the tiles; channel_splits (0 = chosen by the library: 1, 2, 4 or 8;
 *                     or 1, 2, 4, 8, 16, at most the number of 16-channel blocks) lets that many workgroups share a
 *                     tile, each with a part of the channel blocks: their partial sums meet in the handle's workspace
 *                     and are added in a fixed order (reproducible).  The library splits where a layer has fewer
 *                     tiles than compute units and many channel blocks; like the vector kernels' split this uses
 *                     the workspace (allocated on first use; pconv_conv3x3_noalloc takes it from its fixed array
 *                     and runs the layer unsplit if a split of the library's own choosing does not fit there).
 *                     Non-finite activations reach every output whose 3x3 window holds them, also through weights
 *                     that are pruned (0 * inf), which the vector kernels skip.
 *   split_reduce      PCONV_KERNEL_MFMA with channel_splits > 1: who adds the parts.  1 = the workgroup that arrives
 *                     last at a tile reads the other parts back and stores the tile (one launch); 2 = every part only
 *                     writes its partial sums and a second kernel adds them and stores (a launch more, but the parts
 *                     are read by the whole chip: pays from about four parts on); 0 = chosen by the library's
 *                     estimate.  Both add the parts in the same order: the results are equal bit for bit.
 * A combination the library has no kernel for returns PCONV_EUNSUPPORTED.
 */
enum { PCONV_KERNEL_AUTO = 0, PCONV_KERNEL_TILED = 1, PCONV_KERNEL_GENERIC = 2, PCONV_KERNEL_QUAD = 3,
       PCONV_KERNEL_MFMA = 4 };
enum { PCONV_ORDER_AUTO = 0, PCONV_ORDER_PLAIN = 1, PCONV_ORDER_BALANCED = 2 };
typedef struct pconv_tuning {
    int kernel;
    int rows;
    int filters_per_wave;
    int waves;
    int channels_per_wave;
    int channel_order;
    int channel_splits;
    int buffers;
    int slot_walk;
    int mfma_shape;
    int split_reduce;
} pconv_tuning;
int pconv_conv3x3_tuned(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H, int W,
                        int stride, int pad, unsigned flags, void* stream, const pconv_tuning* tuning);

/*
 * Which kernel pconv_conv3x3 takes for a shape, for device buffers aligned as allocations are (introspection; nothing
 * is launched or allocated): *kernel receives PCONV_KERNEL_TILED, _QUAD, _GENERIC or _MFMA, *mfma_shape the tile
 * shape of the matrix-core kernel (0 otherwise).  Either output pointer may be NULL.
 */
int pconv_conv3x3_choice(const pconv_packed* wp, int N, int H, int W, int stride, int pad, int* kernel, int* mfma_shape);

/*
 * Dense 3x3 convolution of the same shape, for comparison: all nine taps of all F*C kernels (give it the masked
 * dense tensor to compute the same function as pconv_conv3x3).  Same conventions and argument meaning.
 *   w_oihw  device, dtype[F*C*9]
 * fp16 storage runs on the matrix cores (the kernel of PCONV_KERNEL_MFMA on nine taps): each call first copies the
 * weights into that kernel's order, in a buffer the library keeps per device and grows on demand (hipMalloc on
 * growth), so calls that overlap in time on one device race.  fp32 storage, and fp16 with PCONV_FLAG_DENSE_DIRECT,
 * run a plain direct kernel on the vector ALUs (one thread per output, no tiling): a cross-check, not a fast kernel.
 */
int pconv_dense_conv3x3(const void* x, void* y, const void* w_oihw, const float* bias, int dtype, int N, int C, int F,
                        int H, int W, int stride, int pad, unsigned flags, void* stream);

/* 2x2 max-pool with stride 2 (between the VGG-16 stages): y[n][c][oy][ox] over floor(H/2) x floor(W/2) outputs.
 *   x device dtype[N*C*H*W]; y device dtype[N*C*(H/2)*(W/2)]. */
int pconv_maxpool2x2(const void* x, void* y, int dtype, int N, int C, int H, int W, void* stream);

/* Text for an error code (static storage). */
const char* pconv_strerror(int code);

/* Text of the last HIP error seen by the calling thread inside this library (static or thread-local storage). */
const char* pconv_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PCONV_H */
