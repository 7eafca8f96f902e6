// Shared between the host packer and the device code of libpconv.  Not part of the public ABI.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "pconv.h"

namespace pconv {

// The packed entries of a filter are bucketed by input channel in buckets of this many channels.  The tiled kernel
// stages a chunk of 1, 2 or 4 consecutive buckets of activations in LDS at a time.
constexpr int kBucket = 16;

// Bytes between the code sections of two patterns in the tiled kernel's generated inner loop.
constexpr int kLeafStride = 256;

// One kept kernel in the device layout (32 bytes so that one scalar load of eight dwords fetches it).
struct DevEntry {
    float w[4];       // the four kept weights, taps ascending, widened to fp32 (exact for fp16 storage)
    uint32_t hdr;     // what the tiled kernel's inner loop reads: bits 0..7 = c mod 256 (chunks are 16 or 32 channels
                      // and start at multiples of their size, so the low bits are the index inside the chunk),
                      // bits 8.. = code; code * kLeafStride is the byte offset of the pattern's code section
    uint32_t c;       // input channel
    uint32_t mask9;   // the pattern mask itself (bit t = 3*ky + kx)
    uint32_t code;    // rank of the mask among the 255 masks with one to four of nine bits, ascending (0..254)
};
static_assert(sizeof(DevEntry) == 32, "DevEntry must be 32 bytes");

// A device layout for one tiling of the tiled kernel (FW waves per workgroup, NF filters per wave, chunks of CC
// channels).  The filters of a workgroup (FW*NF consecutive positions of filter_order) share one order in which the
// input channels are staged; that order is chosen, per workgroup, so that every wave finds (nearly) the same number
// of kept kernels in every chunk: the waves of a workgroup meet at a barrier per chunk, so the slowest one sets the
// pace.  This is the kernel re-ordering for load balance of section 6.2 of the paper, applied to channels.
// Channels that no filter of the workgroup keeps are not staged at all.
struct BalancedLayout {
    int fw = 0, nf = 0, cc = 0;
    int n_groups = 0, n_chunks = 0;
    std::vector<DevEntry> ent;       // [n_kept]; DevEntry::c is the POSITION of the channel in the staging order
    std::vector<uint32_t> eptr;      // [F*n_chunks + 1]: entries of (filter position i, chunk k)
    std::vector<uint32_t> perm;      // [n_groups][n_chunks*cc]: channel staged at each position, 0xFFFFFFFF = none
    DevEntry* d_ent = nullptr;
    uint32_t* d_eptr = nullptr;
    uint32_t* d_perm = nullptr;
};

constexpr uint32_t kNoChannel = 0xFFFFFFFFu;

// The layer's weights as the matrix-core kernel (fp16 storage) stages them: dense over the taps that occur in the
// layer, explicit zeros where a kernel is removed or a tap lies outside its pattern.  For workgroup tiles of `mt`
// filters: w[m-tile][c-block of 16][tap slot][half of the c-block (8 channels)][filter in tile][8 channels], fp16,
// so that the weights one workgroup needs for one c-block are one contiguous piece that is copied to LDS as it is,
// and a lane's operand of v_mfma_f32_32x32x16_f16 (8 consecutive channels of one filter and tap) is 16 contiguous
// bytes.  Filters beyond F and channels beyond C are zero.
struct MfmaWeights {
    int mt = 0;
    int n_mtiles = 0, n_cblocks = 0, n_taps = 0;
    uint8_t taps[9] = {};             // tap index t = 3*ky + kx of every tap slot, ascending
    std::vector<uint16_t> w;          // host copy (fp16 bit patterns)
    void* d_w = nullptr;
    size_t bytes() const { return w.size() * sizeof(uint16_t); }
    // Channel lists (empty: every filter tile takes the channels in their own order, n_cblocks blocks each).  Where
    // the filters of a tile keep only part of the input channels -- connectivity pruning that removes the same
    // channels for similar filters, and filters ordered so that similar ones share a tile -- the tile's blocks are
    // made of the channels it keeps, ascending, 16 per block, the last padded with kNoChannel (zero weights; the
    // kernel loads nothing for it): tile t has tinfo[2t] blocks, the first of them block tinfo[2t+1] of `clist`
    // and of the weights, which are stored for the listed blocks only.  This is the compact, re-ordered kernel
    // storage of section 6.2 of the paper at the granularity the matrix cores work at.
    std::vector<uint32_t> clist;      // [total blocks][16] channel of every position
    std::vector<uint32_t> tinfo;      // [n_mtiles][2]
    int min_blocks = 0, total_blocks = 0;
    uint32_t* d_clist = nullptr;
    uint32_t* d_tinfo = nullptr;
    // A layer of 1x1 kernels (one tap) can be kept a second time with its channels in `groups` equal ranges that take
    // the place of taps: block b, tap slot t holds channels t*C/groups + 16b .. +15, so a block of the contraction is
    // 16*groups channels deep and a layer has C/(16*groups) of them (n_cblocks and n_taps say so).  1: not so.
    int groups = 1;
};

}  // namespace pconv

struct pconv_packed {
    int F = 0, C = 0, K = 0, dtype = 0;
    size_t n_kept = 0;
    bool is_1x1 = false;                  // made by pconv_pack_1x1: every entry is one weight of a 1x1 layer (centre tap)
    std::vector<uint16_t> lib;

    // canonical form (what pconv_packed_export returns)
    std::vector<uint32_t> filter_order;   // [F]
    std::vector<uint32_t> grp_ptr;        // [F*K+1]
    std::vector<uint16_t> cin;            // [n_kept]
    std::vector<unsigned char> w4;        // [n_kept*4] in the storage dtype, raw bytes

    // device layout, host copy: entries ordered by (position i in filter_order, channel bucket, pattern, channel)
    int n_buckets = 0;
    std::vector<pconv::DevEntry> ent;     // [n_kept]
    std::vector<uint32_t> eptr;           // [F*n_buckets + 1]: entries of (i, bucket) are eptr[i*n_buckets+bucket] ..
    std::vector<uint32_t> ent_of_canonical;   // [n_kept]: index in `ent` of each canonical entry
    // per canonical entry {filter, channel | mask << 16}: what the weight-gradient pass needs to find an entry's sums
    std::vector<uint32_t> canon;              // [n_kept*2]
    uint32_t* d_canon = nullptr;

    // balanced layouts for the tilings that the automatic choice uses (see pconv::BalancedLayout)
    std::vector<pconv::BalancedLayout> balanced;

    // fp16 storage only: the weights in matrix-core order, one copy per workgroup tile height (see MfmaWeights)
    std::vector<pconv::MfmaWeights> mfma;

    // Workspace of the tiled kernel when it splits the input channels of one output tile over several workgroups:
    // their partial sums and one arrival counter per tile.  Grown on demand by the convolution call, so calls that
    // share a handle must not overlap in time.
    mutable float* d_ws = nullptr;
    mutable size_t ws_floats = 0;
    mutable unsigned* d_counters = nullptr;
    mutable size_t n_counters = 0;
    // Stride-2 layers run as stride-1 layers over the four row/column parity planes of the input.  Per padding
    // (0, 1): the layer re-packed for that form (4*C input channels, kernels of one to four taps), made by the
    // first stride-2 call that needs it; and the buffer that holds the input split into planes.
    mutable pconv_packed* by_parity[2] = {nullptr, nullptr};
    mutable void* d_planes = nullptr;
    mutable size_t planes_bytes = 0;
    // device copies (null when packed host-only)
    int device = -1;
    pconv::DevEntry* d_ent = nullptr;
    uint32_t* d_eptr = nullptr;
    uint32_t* d_forder = nullptr;
};

namespace pconv {
// implemented in pconv_host.cpp
// The same layer for stride 2 and padding `pad`, as a stride-1 layer over parity planes: input channel 4*c + 2*a + b
// is the plane x[c][2i+a][2j+b]; tap (ky,kx) of kernel (f,c) becomes tap (ky',kx') of kernel (f, 4*c + 2*a + b) with
// a = (ky-pad) mod 2, ky' = floor((ky-pad)/2) + pad, likewise for columns.  Weights keep their storage type.
int derive_for_stride2(const pconv_packed* p, int pad, bool upload, pconv_packed** out);
// implemented in pconv_mfma.hip: the matrix-core kernel for fp16 storage
struct MfmaConv {
    const void* x;
    void* y;
    const float* bias;          // device, or null
    const void* d_w;            // MfmaWeights::d_w
    const uint32_t* d_clist;    // MfmaWeights::d_clist, d_tinfo: null where the tiles take the channels in their own order
    const uint32_t* d_tinfo;
    int min_blocks, total_blocks;   // with channel lists: the fewest blocks any tile has, and all of them
    size_t w_bytes;             // bytes of the weights at d_w
    int mt, n_taps;
    uint8_t taps[9];
    int groups;                 // MfmaWeights::groups
    int kext;                   // rows and columns of the kernel's extent: 3, or 1 for a layer of 1x1 kernels (its one tap
                                // is then tap 0 at padding 0: no halo rows or columns are staged); 0 means 3
    int N, C, F, H, W, Ho, Wo, stride, pad, relu;
    int nhwc;                   // x is [N][H][W][C] and y [N][Ho][Wo][F] (C and F multiples of 8, no channel lists)
    int shape;                  // 1..kMfmaShapes: the tile shape (mt must be its height)
    int rows;                   // 0: as many output rows per tile as fit; else that many
    int walk;                   // 1: one workgroup per tile; otherwise persistent workgroups that walk over the tiles
    int splits;                 // workgroups per tile, each with a part of the channel blocks (1: no split)
    int second_pass;            // splits > 1: the parts are added and stored by a second kernel, not by the last arriver
    float* ws;                  // splits > 1: workspace of mfma_workspace() floats
    unsigned* counters;         // splits > 1: mfma_workspace() counters, zero
};
constexpr int kMfmaShapes = 4;
// tile heights (filters per workgroup) that the kernel's tile shapes use; weights are kept for each
constexpr int kMfmaTileHeights[2] = {128, 64};
constexpr int kOneByOneGroups = 4;       // channel ranges per block of the second copy of a 1x1 layer's weights
int compute_units();        // of the current device
int mfma_shape_height(int shape);
// estimated run time in microseconds of shape `shape` with `splits` workgroups per tile, negative if it cannot run
double mfma_estimate_us(const MfmaConv& a, int shape, int splits);
// workspace that a launch with a.shape and a.splits > 1 needs
int mfma_workspace(const MfmaConv& a, size_t* floats, size_t* counters);
int launch_mfma_conv(const MfmaConv& a, void* stream);
// dense fp16 weights OIHW on the device -> MfmaWeights order for tile height mt, all nine taps (the dense baseline)
int launch_mfma_arrange(const void* w_oihw, void* out, int F, int C, int mt, void* stream);
size_t mfma_weight_bytes(int F, int C, int mt, int n_taps);
// implemented in pconv_device.hip
int upload_packed(pconv_packed* p);
void release_device(pconv_packed* p);
void set_hip_error(const char* what, int hip_code);
}  // namespace pconv
