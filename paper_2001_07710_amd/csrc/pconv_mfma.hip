// Matrix-core kernel of libpconv for fp16 storage on gfx950 (MI355X): the pruned layer as an implicit GEMM on
// v_mfma_f32_32x32x16_f16, fp32 accumulation.
//
// Why a dense contraction for a sparse layer.  Pattern and connectivity sparsity leave 4/9 * keep of the weights
// (12 % at the paper's 8x compression), unstructured at the granularity of a matrix-core operand: for a tile of 32
// filters and 16 channels of one tap, the chance that all 512 weights are pruned is nil, and no re-ordering of
// filters or channels changes that for connectivity chosen by kernel norm.  So the matrix cores can only run the
// layer as the dense convolution with explicit zeros that it equals (section 3 of the paper: pruning is a mask on the
// weights) -- and on this chip that is still the faster way for fp16 storage: 2.5 PFLOP/s of fp16 MFMA against
// 157 TFLOP/s of fp32 vector multiply-adds is a factor of 16, the layer has 8 times fewer multiply-adds.  What the
// sparsity still buys here: taps that no kept kernel of the layer uses are skipped altogether.
//
// Roles.  D[filter][pixel] += A[filter][channel] * B[channel][pixel] per tap: A = weights, B = activations shifted by
// the tap.  With that assignment a lane of the result holds one pixel and its registers hold filters, so NCHW rows
// are contiguous across lanes.
//
// Tile.  A workgroup of WM x WN waves owns MT = WM*AF*32 filters and R consecutive output rows of the batch (rows
// numbered n*Ho + oy, so a tile may run from one image into the next) = up to NT = WN*BF*32 output pixels; a wave
// owns AF x BF operand tiles of 32 x 32.  Channels are taken in blocks of 16 (one MFMA K step); per block the
// workgroup stages, in LDS, the weights of its filters for every tap and the input rows that its pixels read.
//
// LDS layouts (two stages each, one barrier per channel block; a layer with a single block of weights keeps it
// in one stage for good, and one stage of activations written between two barriers is used where that lets a second
// workgroup share the compute unit).
//   weights      [tap slot][half: channels 0-7 | 8-15][filter in tile][8 channels]   as they lie in global memory,
//                                                                                    copied by buffer_load ... lds
//   activations  [half][input row slot][position = column + pad][8 channels]         channel-minor, 16 B per position
//                (channel-minor tensors: [input row slot][position][half][8 channels], 32 B per position, as their
//                 loads deliver them)
// A lane's operand (8 consecutive channels of one filter, or of one pixel) is one 128-bit LDS read; lanes that are
// neighbours in the filter or pixel index read neighbouring 16-byte pieces, so the reads are free of bank
// conflicts, and a tap is nothing but a constant added to the pixel's byte offset: stride 2, either padding and any
// image width come for free.  The activations arrive from global memory row by row (NCHW: pixel-minor), 1, 2, 4 or 8
// pixels of one channel per load; a lane gathers the same pixels of 8 channels and interleaves them in registers
// (v_perm_b32) before the 128-bit LDS writes.  Positions left and right of the image are zeroed once per workgroup;
// rows above and below it, images beyond the batch and channels beyond C are loads at an offset outside the buffer
// descriptor, which return zero.
//
// Workgroups are persistent: each walks a sequence of (tile, channel block) pairs and fetches the next pair while it
// multiplies the current one, also across tiles.
//
// Epilogue.  The accumulators start at the bias; ReLU and the rounding to fp16 in registers, two filters packed per
// word; the tile goes through a wave-private window in LDS once more, [filter pair][pixel], and leaves in pieces of
// 8, 4, 2 or 1 pixels of one filter per lane (whatever divides the row length), coalesced, as streaming stores.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>

#include "pconv_internal.h"

namespace pconv {

#define PCONV_HIP(call)                                  \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) {                          \
            pconv::set_hip_error(#call, (int)e_);        \
            return PCONV_EHIP;                           \
        }                                                \
    } while (0)

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned uint4v __attribute__((ext_vector_type(4)));
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

constexpr uint32_t kInvalid = 0x80000000u;

// Division by a divisor fixed for the launch (Granlund and Montgomery's round-up method, exact for 32-bit dividends).
struct FastDiv {
    unsigned m, s1, s2;
};
FastDiv make_fastdiv(unsigned d) {
    unsigned l = 0;
    while ((1ull << l) < d) ++l;
    FastDiv f;
    f.m = (unsigned)((((1ull << l) - d) << 32) / d + 1);
    f.s1 = l < 1 ? l : 1;
    f.s2 = l > 0 ? l - 1 : 0;
    return f;
}
__device__ __forceinline__ unsigned fastdiv(unsigned x, const FastDiv& f) {
    const unsigned t = __umulhi(x, f.m);
    return (t + ((x - t) >> f.s1)) >> f.s2;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

struct MfmaParams {
    const unsigned char* x;
    unsigned char* y;
    const float* bias;
    const unsigned char* wq;
    const unsigned* clist;  // null: every filter tile takes the channels in their own order, CB blocks.  Else the channels
    const unsigned* tinfo;  // of every block of every tile (16 each, kNoChannel = none), and per tile {blocks, first block}
    int N, C, F, H, W, Ho, Wo, stride, pad, relu;
    int CB;                 // channel blocks of 16
    int nt;                 // tap slots
    int tap_off[9];         // byte offset of a tap inside an activation plane: (ky*PW + kx) * 16 (channel-minor: * 32)
    int R;                  // output rows (of the batch, n*Ho + oy) per tile
    int PW;                 // positions per input row slot: W + 2*pad, or more (plan())
    int max_slots;          // input row slots reserved per buffer
    int kext;               // the kernel's extent in rows (3; 1 for a layer of 1x1 kernels)
    int cnt_full;           // input row slots of a whole image: (Ho-1)*stride + kext
    int tiles_n, tiles_m;
    int G;                  // pieces per input row: W / LW
    int a_bytes;            // weights of one channel block: nt * 2 * MT * 16
    int plane_bytes;        // one half (8 channels) of the activations of one block: max_slots * PW * 16
    int bias_off;           // byte offset in LDS of the bias values (three tiles), behind the staging buffers
    int sw;                 // pixels per store piece: 8, 4, 2 or 1
    unsigned long long y_bytes, x_bytes;
    unsigned wq_bytes;
    unsigned chan_bytes;    // H*W*2
    unsigned img_bytes;     // C*H*W*2
    int nhwc;                    // activations and outputs channel-minor ([N][H][W][C], [N][Ho][Wo][F])
    int P;                       // nhwc: 1 KB pieces (64 positions) per half of a staged block: ceil(max_slots * PW / 64)
    FastDiv div_PW;
    int groups;                  // 1; or (1x1 layers) channel ranges in the place of taps: C is the channels of ONE range,
                                 // range t of a block is staged in row slots t*max_slots .. and read as tap slot t
    unsigned group_bytes;        // bytes from a range's channel to the same channel of the next range (channel-major: whole
                                 // planes; channel-minor: inside a pixel's channel vector)
    int Cpix;                    // channel-minor: channels per pixel in memory (C, or C * groups with channel ranges)
    int KS;                      // workgroups that share one tile, each taking a contiguous range of the channel blocks
    int second_pass;             // KS > 1: every part only writes its partial sums; mfma_split_reduce_kernel adds and stores
    int win_alias;               // the epilogue's windows lie in the staging buffer that is free meanwhile: 1 = its
                                 // weights, 2 = its activations; 0 = in a place of their own behind the bias
    int a_stages;                // 2; or 1: the layer has a single block of weights, staged once per workgroup
    int b_stages;                // 2; or 1: one buffer for the activations, written between two barriers (where that
                                 // makes the LDS small enough for a second workgroup on the compute unit)
    int stagger;                 // every second workgroup starts this many steps of 2048 clocks late (0: none)
    float* ws;              // KS > 1: partial sums [tile][split][wave][operand tile][4 rows][64 lanes][4], as held
    unsigned* counters;     // KS > 1: one arrival counter per tile, zero between launches
    int flag_off;           // byte offset in LDS of the word that tells a workgroup's waves whether it arrived last
    FastDiv div_KS;
    FastDiv div_Wo, div_Ho, div_G, div_cnt_full, div_tiles_m, div_sw_groups;
    int sw_groups;          // store pieces per output row: Wo / sw
};

template <int LW>
struct Piece;   // LW pixels of one channel, as loaded
template <>
struct Piece<8> {
    uint4v v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
    }
    __device__ __forceinline__ unsigned dword(int i) const { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
};
template <>
struct Piece<4> {
    uint2v v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, 0);
    }
    __device__ __forceinline__ unsigned dword(int i) const { return i ? v.y : v.x; }
};
template <>
struct Piece<2> {
    unsigned v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        v = __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0);
    }
    __device__ __forceinline__ unsigned dword(int) const { return v; }
};
template <>
struct Piece<1> {
    unsigned v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        v = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)voff, (int)soff, 0);
    }
    __device__ __forceinline__ unsigned dword(int) const { return v; }
};

// pixel `px` (0: low halves, 1: high halves) of two channels' dwords -> one dword {channel a, channel b}
__device__ __forceinline__ unsigned interleave(unsigned a, unsigned b, int px) {
    return px ? __builtin_amdgcn_perm(b, a, 0x07060302u) : __builtin_amdgcn_perm(b, a, 0x05040100u);
}

// Geometry of one tile (all wave-uniform): the m-tile, and the R consecutive output rows of the batch it covers.
struct TileGeo {
    int tile, split;   // the tile and, if its channel blocks are split over several workgroups, which part
    int cb0, cb1;      // the channel blocks of this part (positions in the tile's list of blocks)
    int wb;            // the tile's first block in the weights (and in the channel list)
    int tm;            // which MT filters
    int Rv;            // output rows in the tile (the last tile of the batch may have fewer than R)
    int n0, oy0;       // image and row of its first output row
    int cnt0;          // input row slots of the part in image n0
    int used_slots;    // input row slots in all
};

// KI: staging pieces of the activations per lane and channel block.  FULL: all nine taps occur; the channel block is
// then one straight run of code in which the loads of the next block are issued a few at a time between the MFMAs.
//
// Workgroups are persistent: workgroup w takes tiles w, w + G, w + 2G, ... and runs the (tile, channel block) pairs of
// all of them as one sequence, so the first block of the next tile is loaded while the last block of the current one
// is multiplied, and the stores of a tile drain while the next tile is computed.
// NHWC: activations and outputs are channel-minor in memory.  That is the order the staged activations have in LDS
// anyway, so they go from memory straight into LDS like the weights (buffer_load ... lds, 16 bytes = 8 channels of one
// position per lane, 64 consecutive positions per wave-wide load; positions outside the image are loads outside the
// descriptor and arrive as zeros, which is the padding): no staging registers, no byte permutes, no LDS writes.  The
// epilogue turns 32 pixels at a time through a wave-private LDS window so that whole runs of a pixel's filters are
// stored.
template <int AF, int BF, int WM, int WN, int LW, int KI, bool FULL, bool NHWC>
__global__ __launch_bounds__(WM* WN * 64, (AF == 1 && WM == 2 && WN == 2) ? 2 : 1) void mfma_conv_kernel(const MfmaParams p) {
    constexpr int kItems = NHWC ? 0 : KI;
    constexpr int kAL = NHWC ? 12 : 0;      // NHWC: wave-wide activation loads per wave and block, at most
    constexpr bool CAN_ALIAS = AF == 1 && WM == 2 && WN == 2;
    constexpr int NW = WM * WN, NTH = NW * 64, MT = WM * AF * 32, HALF = NTH / 2;
    constexpr int WPIECES = (9 * 2 * MT + NTH - 1) / NTH;      // 16-byte pieces of weights per lane and block, at most
    constexpr int WP = BF * 32 + 16;                           // words between two filter pairs of a wave's output window
                                                               // (twice that is 32 mod 64: the two halves of a wave
                                                               // write different LDS banks)
    extern __shared__ __align__(16) unsigned char lds[];

    // ---- which tiles: consecutive workgroup ids go round the XCDs; workgroups of one XCD get consecutive tiles, so
    // the m-tiles of one n-tile (which read the same activations) and n-tiles that are neighbours in memory share
    // an L2.  gridDim.x is a multiple of 8.
    const unsigned nwg = gridDim.x;
    unsigned w0 = (blockIdx.x & 7u) * (nwg >> 3) + (blockIdx.x >> 3);
    // Staggered start (p.stagger > 0, set by the host when it costs no extra round): every second workgroup of an
    // XCD starts half a tile's time late, and takes its tiles from the upper half of the ids, so the late ones are
    // those with one tile less.  Left alone, all workgroups reach their epilogue at the same moment, the stores of
    // the whole chip arrive in one burst, and the loads of the next tile queue behind them.
    const bool late = p.stagger > 0 && ((blockIdx.x >> 3) & 1u);
    if (p.stagger > 0) {
        const unsigned half_per = nwg >> 4;
        w0 = (late ? (nwg >> 1) : 0u) + (blockIdx.x & 7u) * half_per + (blockIdx.x >> 4);
    }
    // (a work item is a tile, or one of the KS parts of a tile's channel blocks; the parts of a tile are neighbours)
    const unsigned ntiles = (unsigned)p.tiles_n * (unsigned)p.tiles_m * (unsigned)p.KS;
    if (w0 >= ntiles) return;
    if (late)
        for (int i = 0; i < p.stagger; ++i) __builtin_amdgcn_s_sleep(32);      // 2048 clocks each

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (tells the compiler that it is wave-uniform)
    const int wm = wave / WN, wn = wave - wm * WN;
    const int s = p.stride, Ho = p.Ho, Wo = p.Wo, PW = p.PW;

    auto geometry = [&](unsigned item) {
        TileGeo g;
        const unsigned T = fastdiv(item, p.div_KS);
        g.tile = (int)T;
        g.split = (int)(item - T * (unsigned)p.KS);
        const unsigned tn = fastdiv(T, p.div_tiles_m);
        g.tm = (int)(T - tn * (unsigned)p.tiles_m);
        int blocks = p.CB;
        g.wb = g.tm * p.CB;
        if (p.clist) {
            blocks = (int)__builtin_amdgcn_readfirstlane(p.tinfo[2 * g.tm]);
            g.wb = (int)__builtin_amdgcn_readfirstlane(p.tinfo[2 * g.tm + 1]);
        }
        g.cb0 = g.split * blocks / p.KS;
        g.cb1 = (g.split + 1) * blocks / p.KS;
        const int R0 = (int)tn * p.R;
        g.Rv = min(p.R, p.N * Ho - R0);
        g.n0 = (int)fastdiv((unsigned)R0, p.div_Ho);
        g.oy0 = R0 - g.n0 * Ho;
        const int rows0 = min(g.Rv, Ho - g.oy0);                   // rows in the first image
        g.cnt0 = (rows0 - 1) * s + p.kext;
        const int last_g = (int)fastdiv((unsigned)(g.oy0 + g.Rv - 1), p.div_Ho);
        const int rows_last = last_g == 0 ? rows0 : g.oy0 + g.Rv - last_g * Ho;
        g.used_slots = last_g == 0 ? g.cnt0 : g.cnt0 + (last_g - 1) * p.cnt_full + (rows_last - 1) * s + p.kext;
        return g;
    };

    unsigned char* const ldsA = lds;
    const int a_stages = CAN_ALIAS ? p.a_stages : 2;           // (plan() keeps the weights resident for that shape only)
    unsigned char* const ldsB = lds + a_stages * p.a_bytes;
    const int b_stages = CAN_ALIAS ? p.b_stages : 2;
    float* const ldsBias = reinterpret_cast<float*>(lds + p.bias_off);          // [3][MT]: by tile count modulo 3
    unsigned* const win_fixed = reinterpret_cast<unsigned*>(lds + p.bias_off + 3 * MT * 4) +
                                wave * (NHWC ? 32 * (AF * 64 + 8) / 4 : 4 * WP);

    // ---- zero columns left and right of the image, in one staging buffer: once per workgroup (no tile's staging
    // ever writes them), and again behind an epilogue whose windows lay in that buffer
    auto zero_halo = [&](int stage) {
        if (NHWC || !p.pad) return;
        const uint4v zero = {0u, 0u, 0u, 0u};
        for (int i = tid; i < p.max_slots * p.groups * 4; i += NTH) {
            const int sl = i >> 2, which = i & 3;               // half (2) x side (2)
            const int pos = (which & 1) ? p.pad + p.W : 0;
            *reinterpret_cast<uint4v*>(ldsB + (stage * 2 + (which >> 1)) * p.plane_bytes + (sl * PW + pos) * 16) = zero;
        }
    };
    zero_halo(0);
    if (b_stages == 2) zero_halo(1);
    // The tile's biases: 4 bytes per lane straight into LDS (buffer_load ... lds), in flight while the block that
    // issues them is multiplied; outside the tensor (filters behind the last, or no bias at all) the load gives zero.
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const __amdgpu_buffer_rsrc_t br = make_rsrc(p.bias, p.bias ? (unsigned)p.F * 4u : 0u);
    auto stage_bias = [&](int tm, int slot) {
        if (wave * 64 < MT)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(br, (lds_ptr)(ldsBias + slot * MT + wave * 64), 4,
                                                     (tm * MT + wave * 64 + lane) * 4, 0, 0, 0);
    };

    // ---- staging state: descriptors of this lane for the tile whose blocks are being loaded
    const int kbs = wave >= NW / 2 ? 1 : 0;                     // which half of the block's channels this wave stages
    const int ltid = tid - kbs * HALF;
    uint32_t goff[kItems > 0 ? kItems : 1];
    int loff[kItems > 0 ? kItems : 1];
    uint32_t agoff[kAL > 0 ? kAL : 1];      // NHWC: this lane's byte offset in x for each of the wave's activation loads
    int stage_wb = 0;                                           // first block of the tile being loaded, in the weights
    bool stage_on = true;                                       // false: nothing left to load (offsets outside)
    bool weights_on = true;                                     // false: the only block of weights is in LDS for good
    // (the descriptor of x is put together where it is used, from three scalars that are marked wave-uniform: as a
    // variable that changes from tile to tile the compiler would keep it in vector registers and wrap every load in
    // a loop over its distinct values)
    unsigned xb_lo = 0, xb_hi = 0, x_records = 0;
    const __amdgpu_buffer_rsrc_t wr = make_rsrc(p.wq, p.wq_bytes);
    auto stage_descriptors = [&](const TileGeo& g) {
        stage_wb = g.wb;
        if constexpr (NHWC) {
            // load `id` of a block = positions 32 id .. 32 id + 31 of the [row slot][position] array, both halves:
            // a pair of neighbouring lanes takes the 32 consecutive bytes of one pixel's sixteen channels, so LDS
            // holds [position][half][8 channels] and the load touches 32 memory lines, not 64 (with one half per
            // load, 16 bytes per line and lane, the address unit's line rate bound the 64-channel layers); wave w
            // issues loads w, w + NW, ...
#pragma unroll
            for (int i = 0; i < kAL; ++i) {
                const int id = wave + i * NW;
                const int half = lane & 1;
                const unsigned q = (unsigned)(id * 32 + (lane >> 1));
                const unsigned sl = fastdiv(q, p.div_PW), pos = q - sl * (unsigned)PW;
                const int col = (int)pos - p.pad;
                agoff[i] = kInvalid;
                if (id < 2 * p.P && (int)sl < g.used_slots && col >= 0 && col < p.W) {
                    int seg, iy;
                    if ((int)sl < g.cnt0) {
                        seg = 0;
                        iy = g.oy0 * s - p.pad + (int)sl;
                    } else {
                        const unsigned t = sl - (unsigned)g.cnt0, qq = fastdiv(t, p.div_cnt_full);
                        seg = 1 + (int)qq;
                        iy = (int)(t - qq * (unsigned)p.cnt_full) - p.pad;
                    }
                    if (g.n0 + seg < p.N && iy >= 0 && iy < p.H)
                        agoff[i] = (uint32_t)seg * p.img_bytes + (uint32_t)((iy * p.W + col) * p.Cpix + half * 8) * 2u;
                }
            }
        }
        const int slots_all = g.used_slots * p.groups;         // (with channel ranges: the row slots of every range)
        const float inv_slots = 1.0f / (float)slots_all;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            // Neighbouring lanes take neighbouring ROWS of the same column group, not neighbouring groups of one row:
            // a lane writes its LW positions to LDS one after the other, so the 16 lanes that one 128-bit LDS write
            // serves together are LW*16 bytes apart along a row -- with 8 pixels per lane only two different bank
            // groups, an 8-way conflict -- but a row pitch of W + 2 positions apart across rows, which spreads them
            // (measured before the change: 37 to 48 % of the LDS's busy time were bank conflicts).
            // (the quotient by way of the reciprocal: exact for these sizes, the remainder of (it + 1/2) / slots is
            // at least 1/(2 slots) away from a whole number, far more than the rounding errors; an integer division
            // by a number that is not known when compiling is some forty instructions)
            const unsigned it = (unsigned)(ltid + i * HALF);
            const unsigned gg = (unsigned)(((float)it + 0.5f) * inv_slots);
            unsigned sl = it - gg * (unsigned)slots_all, range = 0;
            while (sl >= (unsigned)g.used_slots) {              // (at most groups - 1 times)
                sl -= (unsigned)g.used_slots;
                ++range;
            }
            goff[i] = kInvalid;
            loff[i] = -1;
            if (gg < (unsigned)p.G) {
                int seg, iy;
                if ((int)sl < g.cnt0) {
                    seg = 0;
                    iy = g.oy0 * s - p.pad + (int)sl;
                } else {
                    const unsigned t = sl - (unsigned)g.cnt0, q = fastdiv(t, p.div_cnt_full);
                    seg = 1 + (int)q;
                    iy = (int)(t - q * (unsigned)p.cnt_full) - p.pad;
                }
                if (g.n0 + seg < p.N && iy >= 0 && iy < p.H)
                    goff[i] = (uint32_t)seg * p.img_bytes + (uint32_t)(iy * p.W + (int)gg * LW) * 2u + range * p.group_bytes;
                loff[i] = kbs * p.plane_bytes + (((int)range * p.max_slots + (int)sl) * PW + p.pad + (int)gg * LW) * 16;
            }
        }
        // (at most 2^31 - 1 bytes, so that the offset that stands for "nothing to load" is outside whatever the
        // tensor's size; the host has checked that the images one tile touches end below that)
        const unsigned long long x_off = (unsigned long long)g.n0 * p.img_bytes;
        const unsigned long long x_left = p.x_bytes - x_off;
        const unsigned long long xb = reinterpret_cast<unsigned long long>(p.x) + x_off;
        xb_lo = __builtin_amdgcn_readfirstlane((unsigned)xb);
        xb_hi = __builtin_amdgcn_readfirstlane((unsigned)(xb >> 32));
        x_records = __builtin_amdgcn_readfirstlane(x_left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (unsigned)x_left);
    };

    Piece<LW> stg[kItems > 0 ? kItems : 1][8];
    const int w_pieces = p.a_bytes >> 4;                       // (a multiple of 128: whole waves)

    // One of the loads of channel block cb, which will be multiplied out of LDS buffer `buf`.  j < 8*kItems: channel
    // j%8 of piece j/8 of the activations, into registers.  Then the weights, 1 KB per wave and load, straight into
    // LDS (buffer_load ... lds: lane l's 16 bytes land at the wave's base + 16*l, no registers in between); the
    // buffer is free from the barrier that ended the block before the current one.
    constexpr int NLOADS = (NHWC ? kAL : 8 * kItems) + WPIECES;
    constexpr int NACT = NHWC ? kAL : 8 * kItems;
    // The eight channels of block `cb` that this wave stages: consecutive ones, or (channel lists) whichever the
    // tile's list names at that place -- kNoChannel, beyond any C, where the list's last block is not full.
    int chans[8];
    auto block_channels = [&](int cb) {
#pragma unroll
        for (int ch = 0; ch < 8; ++ch) {
            chans[ch] = cb * 16 + kbs * 8 + ch;
            if (p.clist) chans[ch] = (int)__builtin_amdgcn_readfirstlane(p.clist[(stage_wb + cb) * 16 + kbs * 8 + ch]);
        }
    };
    auto issue_one = [&](int cb, int buf, int j) {
        if (j < NACT) {
          if constexpr (NHWC) {
            const int id = wave + j * NW;
            if (id < 2 * p.P) {
                const __amdgpu_buffer_rsrc_t xr =
                    make_rsrc(reinterpret_cast<const void*>(((unsigned long long)xb_hi << 32) | xb_lo), x_records);
                // (with channel ranges in the place of taps: the same positions of every range, each range into its
                // own part of the stage, 2 P pieces long)
                for (int t = 0; t < p.groups; ++t)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        xr, (lds_ptr)(ldsB + buf * 2 * p.plane_bytes + t * (2 * p.P * 1024) + id * 1024), 16,
                        (int)(stage_on ? agoff[j] : kInvalid), cb * 32 + t * (int)p.group_bytes, 0, 0);
            }
          } else {
            const int i = j >> 3, ch = j & 7;
            const unsigned chan = (unsigned)chans[ch];
            const __amdgpu_buffer_rsrc_t xr =
                make_rsrc(reinterpret_cast<const void*>(((unsigned long long)xb_hi << 32) | xb_lo), x_records);
            stg[i][ch].load(xr, (chan < (unsigned)p.C && stage_on) ? goff[i] : kInvalid,
                            chan < (unsigned)p.C ? chan * p.chan_bytes : 0u);
          }
        } else {
            const int first = ((j - NACT) * NW + wave) * 64;              // the wave's first piece (uniform)
            if (first < w_pieces && stage_on && weights_on) {
                const uint32_t wsoff = (uint32_t)((stage_wb + cb) * p.a_bytes);
                const int abuf = a_stages == 2 ? buf : 0;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, (lds_ptr)(ldsA + abuf * p.a_bytes + first * 16), 16,
                                                         (first + lane) * 16, (int)wsoff, 0, 0);
            }
        }
    };
    // The staged activations of the next block: interleave the channels and write them to LDS; then wait for the
    // weights that are on their way into LDS, so that the barrier behind this publishes both.
    auto write_lds = [&](int buf) {
        // (a single buffer: every wave must be done reading the current block before the next one is written over it)
        if (b_stages == 1) __syncthreads();
        unsigned char* const b = ldsB + (b_stages == 2 ? buf : 0) * 2 * p.plane_bytes;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            if (loff[i] >= 0) {
#pragma unroll
                for (int px = 0; px < LW; ++px) {
                    uint4v v;
                    v.x = interleave(stg[i][0].dword(px >> 1), stg[i][1].dword(px >> 1), px & 1);
                    v.y = interleave(stg[i][2].dword(px >> 1), stg[i][3].dword(px >> 1), px & 1);
                    v.z = interleave(stg[i][4].dword(px >> 1), stg[i][5].dword(px >> 1), px & 1);
                    v.w = interleave(stg[i][6].dword(px >> 1), stg[i][7].dword(px >> 1), px & 1);
                    *reinterpret_cast<uint4v*>(b + loff[i] + px * 16) = v;
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
    };

    // ---- compute state: operand offsets of this lane for the tile being multiplied
    const int li = lane & 31, lk = lane >> 5;                   // row/column of the operand tile, half of its K
    const int aoff = (lk * MT + wm * AF * 32 + li) * 16;
    int boff[BF];
    int boff_rows = -1;             // >= 0: boff is that of a tile of so many rows inside one image (the same for all)
    auto compute_descriptors = [&](const TileGeo& g) {
        const int rows_key = g.oy0 + g.Rv <= Ho ? g.Rv : -1;
        if (rows_key >= 0 && rows_key == boff_rows) return;
        boff_rows = rows_key;
#pragma unroll
        for (int bf = 0; bf < BF; ++bf) {
            const unsigned q = (unsigned)((wn * BF + bf) * 32 + li);
            const unsigned r = fastdiv(q, p.div_Wo), ox = q - r * (unsigned)Wo;
            int off = 0;
            if ((int)r < g.Rv) {
                const unsigned rr = (unsigned)g.oy0 + r, sg = fastdiv(rr, p.div_Ho), oy = rr - sg * (unsigned)Ho;
                const int slot = sg == 0 ? (int)r * s : g.cnt0 + ((int)sg - 1) * p.cnt_full + (int)oy * s;
                off = (slot * PW + (int)ox * s) * 16;
            }
            boff[bf] = NHWC ? off * 2 + lk * 16 : off + lk * p.plane_bytes;
        }
    };

    // The accumulators of a tile start at the bias of their filter (accumulator row r of a 32 x 32 block is filter
    // (r/4)*8 + (lane/32)*4 + r%4), or at zero in the workgroups that take a later part of a split tile's channels.
    float16v acc[AF][BF];
    auto start_acc = [&](const TileGeo& g, int bias_slot) {
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));                         // (computed here, not ahead of everything)
        const float4v* const b4 =
            reinterpret_cast<const float4v*>(ldsBias + bias_slot * MT + wm * AF * 32 + (lane_e >> 5) * 4);
#pragma unroll
        for (int af = 0; af < AF; ++af)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                float4v b = b4[af * 8 + rq * 2];
                if (g.split != 0) b = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int bf = 0; bf < BF; ++bf)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[af][bf][rq * 4 + i] = b[i];
            }
    };

    // fp16, ReLU; eight filters of the wave's pixels at a time through the wave's own window in LDS.  A lane holds
    // four of the eight filters for its pixel: it rounds them to fp16 two at a time (one packed conversion) and
    // writes the two words to [filter pair][pixel]; a lane then reads back 8 consecutive pixels of one pair, takes the
    // two filters apart (byte permutes) and stores each in 8/sw pieces of sw pixels, sw being the widest piece that
    // never crosses an output row.  No workgroup barrier: a wave reads back only what it wrote itself, and LDS
    // operations of one wave complete in order -- which also lets the next eight filters be written into the window
    // right behind the reads of the current ones, before their data has come back.  Everything that depends on the
    // pixel alone (row, image, column: two divisions by constants) is worked out once per tile and lane; a store
    // adds one wave-uniform filter offset.  (Per value this is one maximum, half a conversion and half an LDS write;
    // the first version, which added the bias here, wrote 16-bit words and worked every address out per store,
    // took as long as two to three channel blocks.)
    auto epilogue = [&](const TileGeo& g, int free_buf) {
        // The windows: a place of their own, or (p.win_alias) the weights' half of the staging buffer that nothing
        // uses between the barrier that ended the tile's last block and the first loads of the block after next --
        // the caller puts a barrier behind the epilogue then, so that no wave starts those loads while another
        // still reads its window.  That saves the LDS that decides whether a second workgroup fits the compute unit.
        unsigned* win = win_fixed;
        if constexpr (CAN_ALIAS) {                 // (only the shape that can share a compute unit: plan() agrees)
            if (p.win_alias == 1) win = reinterpret_cast<unsigned*>(ldsA + free_buf * p.a_bytes) + wave * (4 * WP);
            if (p.win_alias == 2) win = reinterpret_cast<unsigned*>(ldsB + free_buf * 2 * p.plane_bytes) + wave * (4 * WP);
        }
        // (the lane index as the compiler cannot see through it: everything below depends on it and is computed
        // here, not ahead of the channel blocks, where it would sit in registers that the multiply loop needs)
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int li = lane_e & 31, lk = lane_e >> 5;
        const unsigned plane = (unsigned)(Ho * Wo);
        const int valid = g.Rv * Wo - wn * BF * 32;              // pixels of the wave's range that exist
        const int sw = p.sw;
        // ReLU on the rounded halves, both at once: the maximum with +0, or, where there is no ReLU, with a quiet
        // NaN -- the maximum of a number and a NaN is the number (IEEE 754 maxNum), so that leaves every value as
        // it is, NaN included, without a second copy of this code and without a select per value
        const half2v floor2 = __builtin_bit_cast(half2v, p.relu ? 0u : 0x7E007E00u);
        // The lane's pieces: byte offset of pixel q0 and on, for the first filter of the lane's pair (2*lk), from the
        // tile's first image; kInvalid (beyond the descriptor's range, the store is dropped) where there is none.
        // (The host has checked that the images one tile touches end below 2^31 bytes.)
        uint32_t dst0[8];
        const int f_lane = g.tm * MT + 2 * lk;
        auto piece = [&](int j) -> uint32_t {
            const int q_wave = li * 8 + j * sw;                   // pixel in the wave's range
            if (li * 8 >= BF * 32 || q_wave >= valid) return kInvalid;
            const unsigned q0 = (unsigned)(wn * BF * 32 + q_wave);
            const unsigned row = fastdiv(q0, p.div_Wo), ox = q0 - row * (unsigned)Wo;
            const unsigned rr = (unsigned)g.oy0 + row, sg = fastdiv(rr, p.div_Ho), oy = rr - sg * (unsigned)Ho;
            return ((sg * (unsigned)p.F + (unsigned)f_lane) * plane + oy * (unsigned)Wo + ox) * 2u;
        };
#pragma unroll
        for (int j = 0; j < 8; ++j) dst0[j] = kInvalid;
        dst0[0] = piece(0);
        if (sw < 8) {
            dst0[1] = piece(1);
            if (sw < 4) {
                dst0[2] = piece(2);
                dst0[3] = piece(3);
                if (sw < 2) {
#pragma unroll
                    for (int j = 4; j < 8; ++j) dst0[j] = piece(j);
                }
            }
        }
        const unsigned long long y_off = (unsigned long long)g.n0 * p.F * plane * 2;
        const unsigned long long y_left = p.y_bytes - y_off, yb = reinterpret_cast<unsigned long long>(p.y) + y_off;
        const unsigned yb_lo = __builtin_amdgcn_readfirstlane((unsigned)yb);
        const unsigned yb_hi = __builtin_amdgcn_readfirstlane((unsigned)(yb >> 32));
        const unsigned y_records = __builtin_amdgcn_readfirstlane(y_left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (unsigned)y_left);
        const __amdgpu_buffer_rsrc_t yr =
            make_rsrc(reinterpret_cast<const void*>(((unsigned long long)yb_hi << 32) | yb_lo), y_records);
        constexpr int kStream = 2;     // cache-policy bit "nt": the outputs are not read again by this kernel and leave
                                       // the L2 sooner (measured 5 to 8 % of the layer time where outputs are large)
        unsigned* const wbase = win + lk * 2 * WP + li;            // the lane's own pixel, its first filter pair
        const unsigned* const rbase = win + lk * WP + li * 8;      // 8 pixels of the pair the lane stores first
        constexpr int P = AF * 4;
        auto write_pass = [&](int pass) {
            const int af = pass >> 2, rq = pass & 3;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int bf = 0; bf < BF; ++bf) {
                    const float2v v = {acc[af][bf][rq * 4 + 2 * h], acc[af][bf][rq * 4 + 2 * h + 1]};
                    const half2v hv = __builtin_elementwise_max(__builtin_convertvector(v, half2v), floor2);
                    wbase[h * WP + bf * 32] = __builtin_bit_cast(unsigned, hv);
                }
        };
        write_pass(0);
#pragma unroll
        for (int pass = 0; pass < P; ++pass) {
            __builtin_amdgcn_wave_barrier();
            uint4v r[2][2];                                         // [round: pairs 0,1 / 2,3][pixels 0-3 / 4-7]
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int hx = 0; hx < 2; ++hx) r[k][hx] = *reinterpret_cast<const uint4v*>(rbase + 2 * k * WP + hx * 4);
            __builtin_amdgcn_wave_barrier();
            if (pass + 1 < P) write_pass(pass + 1);
            __builtin_amdgcn_wave_barrier();
            // the four filters this lane stores in this pass: 4*k + which (+ 2*lk), 8 pixels each
            const int fbase = (wm * AF + (pass >> 2)) * 32 + (pass & 3) * 8;      // (wave-uniform)
            unsigned o[4][4];
            int foff[4];
            bool f_ok[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int k = t >> 1;
                const unsigned sel = (t & 1) ? 0x07060302u : 0x05040100u;   // the pair's second filter / its first
                o[t][0] = __builtin_amdgcn_perm(r[k][0].y, r[k][0].x, sel);
                o[t][1] = __builtin_amdgcn_perm(r[k][0].w, r[k][0].z, sel);
                o[t][2] = __builtin_amdgcn_perm(r[k][1].y, r[k][1].x, sel);
                o[t][3] = __builtin_amdgcn_perm(r[k][1].w, r[k][1].z, sel);
                const int fi = fbase + 4 * k + (t & 1);
                f_ok[t] = f_lane + fi < p.F;
                foff[t] = fi * (int)plane * 2;                        // (wave-uniform: the scalar offset)
            }
            auto at = [&](int t, int j) { return (int)(f_ok[t] ? dst0[j] : kInvalid); };
            // (the piece width is chosen once per pass: with the choice around every single store, each sat behind
            // half a dozen branches, and those, not the stores, were most of the epilogue's time)
            if (sw == 8) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    __builtin_amdgcn_raw_buffer_store_b128(uint4v{o[t][0], o[t][1], o[t][2], o[t][3]}, yr, at(t, 0), foff[t],
                                                           kStream);
            } else if (sw == 4) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    __builtin_amdgcn_raw_buffer_store_b64(uint2v{o[t][0], o[t][1]}, yr, at(t, 0), foff[t], kStream);
                    __builtin_amdgcn_raw_buffer_store_b64(uint2v{o[t][2], o[t][3]}, yr, at(t, 1), foff[t], kStream);
                }
            } else if (sw == 2) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        __builtin_amdgcn_raw_buffer_store_b32(o[t][j], yr, at(t, j), foff[t], kStream);
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(o[t][j >> 1] >> ((j & 1) * 16)), yr, at(t, j),
                                                              foff[t], kStream);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    // NHWC outputs.  A lane holds, for its pixel, filters (r/4)*8 + (lane/32)*4 + r%4 of each 32-filter block.  Written
    // out as they lie that is 8 bytes per lane and pixel, scattered over the pixels' lines (measured: the first layer
    // at batch 64 took 559 us, five times the channel-major form).  So 32 pixels at a time go through a wave-private
    // window in LDS, [pixel][the wave's AF*32 filters] (8 bytes of padding per pixel against bank conflicts): the lanes
    // write their groups of four filters, then AF*4 neighbouring lanes read back the AF*64 bytes of one pixel, 16 bytes
    // each, and a wave-wide store writes whole runs of AF*64 bytes.  LDS operations of one wave complete in order, so
    // no barrier is needed between the two phases.
    auto epilogue_nhwc = [&](const TileGeo& g) {
        constexpr int PITCH = AF * 64 + 8;                       // bytes per pixel in the window
        constexpr int LPP = AF * 4, PPR = 64 / LPP;              // lanes per pixel when reading back; pixels per read
        unsigned char* const win = reinterpret_cast<unsigned char*>(win_fixed);
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int li = lane_e & 31, lk = lane_e >> 5;
        const int valid = g.Rv * Wo - wn * BF * 32;              // pixels of the wave's range that exist
        const half2v floor2 = __builtin_bit_cast(half2v, p.relu ? 0u : 0x7E007E00u);
        const unsigned long long y_off = (unsigned long long)g.n0 * p.F * (unsigned)(Ho * Wo) * 2;
        const unsigned long long y_left = p.y_bytes - y_off, yb = reinterpret_cast<unsigned long long>(p.y) + y_off;
        const unsigned yb_lo = __builtin_amdgcn_readfirstlane((unsigned)yb);
        const unsigned yb_hi = __builtin_amdgcn_readfirstlane((unsigned)(yb >> 32));
        const unsigned y_records = __builtin_amdgcn_readfirstlane(y_left > 0x7FFFFFFFull ? 0x7FFFFFFFu : (unsigned)y_left);
        const __amdgpu_buffer_rsrc_t yr =
            make_rsrc(reinterpret_cast<const void*>(((unsigned long long)yb_hi << 32) | yb_lo), y_records);
        constexpr int kStream = 2;
        auto pack2 = [&](float a, float b) {
            const float2v v = {a, b};
            return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_convertvector(v, half2v), floor2));
        };
        const int part = lane_e % LPP, rpix = lane_e / LPP;      // reading back: which 16 bytes of which pixel of a read
        const int fwave = g.tm * MT + wm * AF * 32;              // the wave's first filter (uniform)
        const bool f_ok = fwave + part * 8 < p.F;                // (F is a multiple of 8)
#pragma unroll
        for (int bf = 0; bf < BF; ++bf) {
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int af = 0; af < AF; ++af)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint2v v = {pack2(acc[af][bf][q * 4 + 0], acc[af][bf][q * 4 + 1]),
                                      pack2(acc[af][bf][q * 4 + 2], acc[af][bf][q * 4 + 3])};
                    *reinterpret_cast<uint2v*>(win + li * PITCH + (af * 32 + q * 8 + lk * 4) * 2) = v;
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int r = 0; r < 32 / PPR; ++r) {
                const int px = r * PPR + rpix;                   // pixel of the 32
                const uint4v v = *reinterpret_cast<const uint4v*>(win + px * PITCH + part * 16);
                const int q_wave = bf * 32 + px;
                uint32_t dst = kInvalid;
                if (q_wave < valid && f_ok) {
                    const unsigned q0 = (unsigned)(wn * BF * 32 + q_wave);
                    const unsigned row = fastdiv(q0, p.div_Wo), ox = q0 - row * (unsigned)Wo;
                    const unsigned rr = (unsigned)g.oy0 + row, sg = fastdiv(rr, p.div_Ho), oy = rr - sg * (unsigned)Ho;
                    dst = (((sg * (unsigned)Ho + oy) * (unsigned)Wo + ox) * (unsigned)p.F) * 2u + (unsigned)part * 16u;
                }
                __builtin_amdgcn_raw_buffer_store_b128(v, yr, (int)dst, fwave * 2, kStream);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    // Channel blocks of a tile split over KS workgroups: every one writes its partial sums to the workspace (laid out
    // like the registers: 16 bytes per lane and group of four accumulator rows, 1 KB per wave-wide store); the one
    // that arrives last at the tile's counter adds the parts in the order of the splits, its own from registers, so
    // the result does not depend on who arrives last, and goes on to the epilogue.  Memory ordering as in the vector
    // kernels' channel split: device-scope (sc1) buffer stores, wait for them, workgroup barrier, one relaxed
    // device-scope atomic, device-scope loads by the last arriver.  Returns whether this workgroup stores the tile.
    auto combine_splits = [&](const TileGeo& g) -> bool {
        constexpr int kDeviceScope = 16;   // cache-policy bit "sc1" of gfx942/gfx950 buffer instructions
        constexpr unsigned PART = (unsigned)NW * AF * BF * 4 * 64 * 4 * 4;      // bytes of one part: MT x NT floats
        const size_t tile_base = (size_t)g.tile * p.KS * PART;
        const __amdgpu_buffer_rsrc_t wsr = make_rsrc(reinterpret_cast<const char*>(p.ws) + tile_base, (unsigned)p.KS * PART);
        auto off = [&](int part, int af, int bf, int rq) {
            return (int)((unsigned)part * PART + ((((unsigned)wave * AF + af) * BF + bf) * 4 + rq) * 1024u + lane * 16u);
        };
#pragma unroll
        for (int af = 0; af < AF; ++af)
#pragma unroll
            for (int bf = 0; bf < BF; ++bf)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    uint4v v;
                    v.x = __builtin_bit_cast(unsigned, (float)acc[af][bf][rq * 4 + 0]);
                    v.y = __builtin_bit_cast(unsigned, (float)acc[af][bf][rq * 4 + 1]);
                    v.z = __builtin_bit_cast(unsigned, (float)acc[af][bf][rq * 4 + 2]);
                    v.w = __builtin_bit_cast(unsigned, (float)acc[af][bf][rq * 4 + 3]);
                    __builtin_amdgcn_raw_buffer_store_b128(v, wsr, off(g.split, af, bf, rq), 0, kDeviceScope);
                }
        // (added and stored by a second kernel: nothing to wait for or to count here -- the end of this kernel is what
        // makes the parts visible)
        if (p.second_pass) return false;
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): the partial sums have left
        __syncthreads();
        unsigned* const flag = reinterpret_cast<unsigned*>(lds + p.flag_off);
        if (tid == 0) {
            const unsigned arrived = __hip_atomic_fetch_add(p.counters + g.tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const bool last = arrived == (unsigned)p.KS - 1u;
            if (last) __hip_atomic_store(p.counters + g.tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = last ? 1u : 0u;
        }
        __syncthreads();
        const bool last = __builtin_amdgcn_readfirstlane(*flag) != 0u;
        __syncthreads();                         // (the flag is read before the next tile's arrival rewrites it)
        if (!last) return false;
        // All parts come from the workspace, this workgroup's own too, in the order of the splits.  Per group of 32
        // filters, the loads of half a part are issued before the first is used: two round trips to memory per part
        // and group, not one per 16 bytes (which is what a loop over the parts around each single load came to, and
        // made the last arriver of 8 parts take 200 us).
#pragma unroll
        for (int af = 0; af < AF; ++af)
#pragma unroll
            for (int b0 = 0; b0 < BF; b0 += 4)                   // (half a group at a time: 64 registers in flight)
                for (int part = 0; part < p.KS; ++part) {
                    uint4v v[4][4];
#pragma unroll
                    for (int bf = b0; bf < BF && bf < b0 + 4; ++bf)
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq)
                            v[bf - b0][rq] =
                                __builtin_amdgcn_raw_buffer_load_b128(wsr, off(part, af, bf, rq), 0, kDeviceScope);
#pragma unroll
                    for (int bf = b0; bf < BF && bf < b0 + 4; ++bf)
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq) {
                            const uint4v u = v[bf - b0][rq];
                            const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float q = __builtin_bit_cast(float, w[i]);
                                acc[af][bf][rq * 4 + i] = part == 0 ? q : acc[af][bf][rq * 4 + i] + q;
                            }
                        }
                }
        return true;
    };

    // ---- the sequence of (tile, channel block) pairs
    unsigned T = w0;
    TileGeo gc = geometry(T);
    stage_descriptors(gc);
    stage_bias(gc.tm, 0);
    block_channels(gc.cb0);
#pragma unroll
    for (int j = 0; j < NLOADS; ++j) issue_one(gc.cb0, 0, j);
    if (a_stages == 1) weights_on = false;
    write_lds(0);
    __syncthreads();
    compute_descriptors(gc);
    start_acc(gc, 0);
    constexpr int SPAN_TAPS = 7;            // taps over which the next block's loads are spread (1..8 measure alike)
    int buf = 0, bias_slot = 0;
    for (;;) {
        const unsigned Tn = T + nwg;
        TileGeo gn = gc;
        for (int cb = gc.cb0; cb < gc.cb1; ++cb) {
            // what is loaded during this block: the tile's next block, or the first block of the workgroup's next
            // tile, or (behind the last tile) nothing
            int ncb = cb + 1;
            if (ncb == gc.cb1) {
                if (Tn < ntiles) {
                    gn = geometry(Tn);
                    stage_descriptors(gn);
                    stage_bias(gn.tm, bias_slot == 2 ? 0 : bias_slot + 1);
                    ncb = gn.cb0;
                } else {
                    stage_on = false;
                    ncb = gc.cb0;
                }
            }
            block_channels(ncb);
            const unsigned char* const a = ldsA + (a_stages == 2 ? buf : 0) * p.a_bytes + aoff;
            const unsigned char* const b = ldsB + (b_stages == 2 ? buf : 0) * 2 * p.plane_bytes;
            auto load_a = [&](int ts, int af) {
                return *reinterpret_cast<const half8*>(a + (ts * 2 * MT + af * 32) * 16);
            };
            auto load_b = [&](int ts, int bf) {
                return *reinterpret_cast<const half8*>(b + boff[bf] + p.tap_off[ts]);
            };
            if constexpr (FULL) {
                // One straight run of code for the nine taps.  The operands of a tap sit in one set of registers for
                // the activations and two for the weights; as soon as the MFMAs that read an activation operand
                // have been issued, the same registers are asked to fetch that operand of the next tap, which leaves
                // the LDS a whole tap's time to answer.  The loads of the next channel block are issued one at a
                // time between those groups, evenly over the first SPAN_TAPS taps.  The order is pinned group by
                // group: left alone, the scheduler hoists reads and address arithmetic far ahead, and the registers
                // that costs are paid for with spills to memory in this loop.
                half8 fa[2][AF], fb[BF];
#pragma unroll
                for (int af = 0; af < AF; ++af) fa[0][af] = load_a(0, af);
#pragma unroll
                for (int bf = 0; bf < BF; ++bf) fb[bf] = load_b(0, bf);
                constexpr int NGROUPS = SPAN_TAPS * BF;          // (tap, activation operand) groups that carry loads
#pragma unroll
                for (int ts = 0; ts < 9; ++ts) {
#pragma unroll
                    for (int bf = 0; bf < BF; ++bf) {
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int af = 0; af < AF; ++af)
                            acc[af][bf] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ts & 1][af], fb[bf], acc[af][bf], 0, 0, 0);
                        if (ts < 8) {
                            fb[bf] = load_b(ts + 1, bf);
                            if (bf < AF) fa[(ts + 1) & 1][bf] = load_a(ts + 1, bf);
                        }
#pragma unroll
                        for (int j = 0; j < NLOADS; ++j)
                            if ((j * NGROUPS) / NLOADS == ts * BF + bf) issue_one(ncb, buf ^ 1, j);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            } else {
                half8 fa[2][AF], fb[2][BF];
                auto fetch = [&](int ts, int set) {
#pragma unroll
                    for (int af = 0; af < AF; ++af) fa[set][af] = load_a(ts, af);
#pragma unroll
                    for (int bf = 0; bf < BF; ++bf) fb[set][bf] = load_b(ts, bf);
                };
                fetch(0, 0);
#pragma unroll
                for (int j = 0; j < NLOADS; ++j) issue_one(ncb, buf ^ 1, j);
#pragma unroll
                for (int ts = 0; ts < 9; ++ts) {
                    if (ts < p.nt) {
                        if (ts + 1 < p.nt) fetch(ts + 1, (ts + 1) & 1);
#pragma unroll
                        for (int bf = 0; bf < BF; ++bf)
#pragma unroll
                            for (int af = 0; af < AF; ++af)
                                acc[af][bf] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ts & 1][af], fb[ts & 1][bf],
                                                                                    acc[af][bf], 0, 0, 0);
                    }
                }
            }
            write_lds(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
        if (p.KS == 1 || combine_splits(gc)) {
            if constexpr (NHWC)
                epilogue_nhwc(gc);
            else
                epilogue(gc, buf ^ 1);
        }
        if constexpr (CAN_ALIAS) {
            if (p.win_alias) __syncthreads();
            if (p.win_alias == 2) zero_halo(buf ^ 1);    // (the windows lay over that buffer's zero columns)
        }
        if (Tn >= ntiles) break;
        T = Tn;
        gc = gn;
        bias_slot = bias_slot == 2 ? 0 : bias_slot + 1;
        compute_descriptors(gc);
        start_acc(gc, bias_slot);
    }
}

// Second pass of a split layer (MfmaParams::second_pass): the KS parts of every tile, which lie in the workspace as the
// accumulators held them ([tile][part][wave][filter block][pixel block][four rows][lane][4]), added in the order of
// the parts (the first of which started from the bias); ReLU, fp16, store.  One thread per 16 bytes of a part: lane `lane` of wave
// `wave` holds, for pixel (lane % 32) of its pixel block, the four filters 8*rq + 4*(lane/32) + 0..3 of its filter block.
// Every workgroup of the first pass took part, so the sum needs neither counters nor an order of arrival, and however
// many parts there are they are read at the rate of a copy (the last arriver of the other form reads them alone).
struct ReduceParams {
    const float* ws;
    unsigned char* y;
    int N, F, Ho, Wo, relu, nhwc;
    int KS, R, tiles_m;
    int AF, BF, WM, WN;
    long long threads;      // tiles * NW * AF * BF * 4 * 64
};
__global__ __launch_bounds__(256) void mfma_split_reduce_kernel(const ReduceParams p) {
    typedef float float4v __attribute__((ext_vector_type(4)));
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= p.threads) return;
    const int lane = (int)(t & 63);
    long long r = t >> 6;
    const int rq = (int)(r & 3); r >>= 2;
    const int bf = (int)(r % p.BF); r /= p.BF;
    const int af = (int)(r % p.AF); r /= p.AF;
    const int NW = p.WM * p.WN;
    const int wave = (int)(r % NW);
    const long long tile = r / NW;
    const int wm = wave / p.WN, wn = wave - wm * p.WN;
    const int MT = p.WM * p.AF * 32;
    const long long part4 = (long long)NW * p.AF * p.BF * 4 * 64;                 // float4s per part
    const long long at = t - tile * part4;                                          // this thread's float4 within a part
    const float4v* const w4 = reinterpret_cast<const float4v*>(p.ws) + tile * p.KS * part4 + at;
    const int tm = (int)(tile % p.tiles_m);
    const long long tn = tile / p.tiles_m;
    const int f0 = tm * MT + (wm * p.AF + af) * 32 + rq * 8 + (lane >> 5) * 4;
    // (the first part started from the bias; the same additions in the same order as the last arriver of the other form)
    float4v sum = w4[0];
    for (int k = 1; k < p.KS; ++k) sum += w4[(long long)k * part4];
    // the pixel: number q of the tile's R rows of the batch
    const int q = (wn * p.BF + bf) * 32 + (lane & 31);
    const int row = q / p.Wo, ox = q - row * p.Wo;
    const long long rr = tn * p.R + row;
    if (row >= p.R || rr >= (long long)p.N * p.Ho) return;
    const long long n = rr / p.Ho;
    const int oy = (int)(rr - n * p.Ho);
    _Float16* const y = reinterpret_cast<_Float16*>(p.y);
    for (int i = 0; i < 4; ++i) {
        if (f0 + i >= p.F) break;
        float v = sum[i];
        if (p.relu) v = v > 0.f ? v : 0.f;
        const long long idx = p.nhwc ? (((n * p.Ho + oy) * p.Wo + ox) * p.F + f0 + i)
                                     : (((n * p.F + f0 + i) * p.Ho + oy) * p.Wo + ox);
        y[idx] = (_Float16)v;
    }
}

// dense OIHW fp16 weights on the device -> MfmaWeights order, all nine taps
__global__ __launch_bounds__(256) void mfma_arrange_kernel(const unsigned short* __restrict__ w, unsigned short* __restrict__ out,
                                                           int F, int C, int mt, int CB, long long total) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        long long r = i;
        const int c8 = (int)(r % 8); r /= 8;
        const int fl = (int)(r % mt); r /= mt;
        const int kb = (int)(r % 2); r /= 2;
        const int ts = (int)(r % 9); r /= 9;
        const int cb = (int)(r % CB); r /= CB;
        const int f = (int)r * mt + fl, c = cb * 16 + kb * 8 + c8;
        out[i] = (f < F && c < C) ? w[((size_t)f * C + c) * 9 + ts] : (unsigned short)0;
    }
}

struct Shape {
    int af, bf, wm, wn;
};
// measured time of one channel block of one tile with the device full, microseconds, per tile shape
const double kBlockUs[kMfmaShapes] = {3.2, 1.7, 1.7, 1.8};
// tile shapes: (128 filters x 448 pixels), (64 x 448), (128 x 224), (64 x 224).  (64 x 896, four waves side by
// side, was tried for layers of 64 filters at 224 x 224 and measured no faster than 64 x 448 there; 128 x 512 on
// eight waves of 64 x 128 each -- two waves per SIMD with the first shape's operand economy -- fits 256 registers
// only with spills, wastes the pixels that 512 has over a multiple of the row, and measured 4 to 45 % slower than the
// first shape on the 112-, 56- and 28-column layers of VGG-16 at batch 64.)
const Shape kShapes[kMfmaShapes] = {{2, 7, 2, 2}, {1, 7, 2, 2}, {1, 7, 4, 1}, {1, 7, 2, 1}};

// Workgroups of the persistent grid: as many as the device holds at once (compute units x workgroups that fit one),
// no more than there are tiles, a multiple of 8 (one share per XCD).
int persistent_grid(const void* kern, int threads, size_t lds, long long ntiles, int walk) {
    if (walk == 1) return (int)std::min<long long>((ntiles + 7) / 8 * 8, 0x7FFFFFF8);   // one workgroup per tile
    int per_cu = 1;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, threads, lds) != hipSuccess || per_cu < 1) per_cu = 1;
    const long long resident = (long long)compute_units() * per_cu / 8 * 8;
    return (int)std::max<long long>(8, std::min<long long>((ntiles + 7) / 8 * 8, resident));
}

// Steps of 2048 clocks by which every second workgroup starts late (0: all start together).  Half a tile's time,
// and only where the late workgroups do not add a round of their own: the last round is at most half full, and they
// are the ones that sit it out.  (Measured on 128 x 256 channels at 56 x 56, batch 64, 3.5 rounds: 209 -> 198 us;
// with 7 or 14 full rounds the half tile more costs as much as the smoother stores gain.)
int stagger_steps(const MfmaParams& p, int grid, long long ntiles, int walk, double block_us) {
    if (walk == 1 || p.KS != 1 || (grid & 15) || ntiles <= grid) return 0;
    const long long rem = ntiles % grid;
    if (rem == 0 || rem > grid / 2) return 0;
    const double half_tile_us = 0.5 * p.CB * block_us;
    return (int)std::min(4096.0, half_tile_us * 2400.0 / 2048.0 + 0.5);
}

template <int AF, int BF, int WM, int WN>
int launch_shape(const MfmaParams& p, int lw, int ki, size_t lds, int walk, double block_us, hipStream_t st) {
    const bool full = p.nt == 9;
    const long long ntiles = (long long)p.tiles_n * p.tiles_m * p.KS;
#define PCONV_MFMA_CASE1(LWv, KIv, FULLv) PCONV_MFMA_CASE2(LWv, KIv, FULLv, false)
#define PCONV_MFMA_CASE2(LWv, KIv, FULLv, NHWCv)                                                                \
    if (lw == LWv && ki == KIv && full == FULLv && (p.nhwc != 0) == NHWCv) {                                    \
        auto kern = mfma_conv_kernel<AF, BF, WM, WN, LWv, KIv, FULLv, NHWCv>;                                   \
        if (lds > 64 * 1024)                                                                                    \
            PCONV_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        const int grid = persistent_grid((const void*)kern, WM * WN * 64, lds, ntiles, walk);                        \
        MfmaParams q = p;                                                                                       \
        q.stagger = stagger_steps(p, grid, ntiles, walk, block_us);                                             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(WM* WN * 64), lds, st, q);                                    \
        PCONV_HIP(hipGetLastError());                                                                           \
        return PCONV_OK;                                                                                        \
    }
#define PCONV_MFMA_CASE(LWv, KIv) PCONV_MFMA_CASE1(LWv, KIv, true) PCONV_MFMA_CASE1(LWv, KIv, false)
#ifdef PCONV_ONLY_ONE
    PCONV_MFMA_CASE1(8, 1, true)
#else
    PCONV_MFMA_CASE(8, 1) PCONV_MFMA_CASE(8, 2) PCONV_MFMA_CASE(4, 2) PCONV_MFMA_CASE(4, 3) PCONV_MFMA_CASE(2, 3)
    PCONV_MFMA_CASE(1, 3) PCONV_MFMA_CASE1(2, 4, false) PCONV_MFMA_CASE1(1, 7, false)
    PCONV_MFMA_CASE2(8, 1, true, true) PCONV_MFMA_CASE2(8, 1, false, true)
#endif
#undef PCONV_MFMA_CASE
#undef PCONV_MFMA_CASE1
#undef PCONV_MFMA_CASE2
    return PCONV_EUNSUPPORTED;
}

// Fills the launch parameters for one tile shape; false if the shape cannot take the layer.
bool plan(const MfmaConv& a, int shape, int rows, MfmaParams* out, int* lw_out, int* ki_out, size_t* lds_out,
          int* grid_out) {
    const Shape& sh = kShapes[shape];
    const int MT = sh.wm * sh.af * 32, NT = sh.wn * sh.bf * 32, NTH = sh.wm * sh.wn * 64;
    if (MT != a.mt) return false;
    MfmaParams p{};
    p.x = static_cast<const unsigned char*>(a.x);
    p.y = static_cast<unsigned char*>(a.y);
    p.bias = a.bias;
    p.wq = static_cast<const unsigned char*>(a.d_w);
    p.N = a.N; p.C = a.C; p.F = a.F; p.H = a.H; p.W = a.W; p.Ho = a.Ho; p.Wo = a.Wo;
    p.stride = a.stride; p.pad = a.pad; p.relu = a.relu;
    p.groups = a.groups > 1 ? a.groups : 1;
    if (p.groups > 1 && (a.d_clist || a.C % (16 * p.groups) || a.n_taps != p.groups)) return false;
    p.C = a.C / p.groups;
    p.CB = (p.C + 15) / 16;
    p.clist = a.d_clist;
    p.tinfo = a.d_tinfo;
    // (channel-minor activations are loaded eight channels at a time as they lie: no channel lists, whole groups)
    if (a.nhwc && (a.d_clist || a.C % 8 || a.F % 8)) return false;
    p.KS = a.splits < 1 ? 1 : a.splits;
    p.second_pass = (p.KS > 1 && a.second_pass) ? 1 : 0;
    // (every part of a split tile has at least one block: the sequence of (tile, block) pairs has no empty member)
    if (p.KS > (a.d_clist ? a.min_blocks : p.CB) || p.KS > 64) return false;
    p.div_KS = make_fastdiv((unsigned)p.KS);
    p.ws = a.ws;
    p.counters = a.counters;
    p.nt = a.n_taps;
    if (p.nt < 0 || p.nt > 9) return false;
    if (a.Wo > NT) return false;                                   // a tile is made of whole output rows
    int R = NT / a.Wo;
    if (rows > 0) R = std::min(R, rows);
    const long long total_rows = (long long)a.N * a.Ho;
    if (total_rows > 0x3FFFFFFF) return false;
    R = (int)std::min<long long>(R, total_rows);
    const uintptr_t xa = reinterpret_cast<uintptr_t>(a.x), ya = reinterpret_cast<uintptr_t>(a.y);
    int lw = (a.W % 8 == 0 && xa % 16 == 0) ? 8 : (a.W % 4 == 0 && xa % 8 == 0) ? 4 : (a.W % 2 == 0 && xa % 4 == 0) ? 2 : 1;
    // pieces of the activations per lane that the kernels are built for, by load width
    // (1x1 layers with channel ranges in the place of taps stage several ranges per block: more of the narrow pieces)
    auto max_items = [&](int w) { return w == 8 ? 2 : a.groups > 1 ? (w == 2 ? 4 : w == 1 ? 7 : 3) : 3; };
    p.PW = a.W + 2 * a.pad;
    // Maps of at most 16 columns: 32 consecutive pixels span three or more rows, and a lane's operand read jumps by
    // PW - Wo positions at every row end.  With that gap a multiple of 8 positions (128 bytes, all LDS banks once) the
    // pieces of a read fall on the banks like one straight run (512 -> 512 channels at 14 x 14, batch 64: 69.5 ->
    // 66 us).  Wider maps are left alone: there the row pitch this gives makes the staging writes collide instead
    // (256 -> 256 channels at 56 x 56: 180 -> 194 us).
    if (a.stride == 1 && a.W <= 16)
        while ((p.PW - a.Wo) % 8) ++p.PW;
    p.kext = a.kext == 1 ? 1 : 3;
    p.cnt_full = (a.Ho - 1) * a.stride + p.kext;
    // rows per tile: as many as fit the pixels of the tile, the staging pieces of a lane and the LDS
    // Input row slots: a tile of R output rows that touches k images needs (R - k)*stride + 3k of them, most for the
    // largest k: at most (R + Ho - 2)/Ho + 1 images, and no more than it has rows.
    size_t lds = 0;
    int segs = 1;
    for (;; --R) {
        if (R < 1) return false;
        segs = std::min(R, (R + a.Ho - 2) / a.Ho + 1);
        if (a.Ho % R == 0) segs = 1;                         // (tiles never cross from one image into the next)
        // (a kernel of extent 1 at stride 2 is the other way round: every further image SAVES a row slot, so the most
        // are needed by a tile that touches as few images as its rows allow)
        const int most_at = a.stride > p.kext ? std::max(1, (R + a.Ho - 1) / a.Ho) : segs;
        p.max_slots = (R - most_at) * a.stride + p.kext * most_at;
        p.a_bytes = p.nt * 2 * MT * 16;
        p.plane_bytes = p.groups * p.max_slots * p.PW * 16;
        // (channel-minor activations arrive in wave-wide pieces of 32 positions, both halves: a stage is 2 P pieces)
        p.P = (p.max_slots * p.PW + 63) / 64;
        if (a.nhwc) p.plane_bytes = p.groups * p.P * 1024;
        // (a layer of at most 16 channels and one tile of filters has a single block of weights: staged once)
        const bool shares_cu = sh.af == 1 && sh.wm == 2 && sh.wn == 2;    // (the shape two workgroups of which fit)
        p.a_stages = (shares_cu && p.CB == 1 && (a.F + MT - 1) / MT == 1 && p.KS == 1) ? 1 : 2;
        // (one buffer for the activations instead of two where that, and nothing less, lets a second workgroup in)
        p.b_stages = 2;
        const size_t extra = 3 * (size_t)MT * 4 + 16;
        // (not with channel-minor activations: their loads write the next block's buffer while this one is read)
        if (!a.nhwc && shares_cu && p.a_stages == 2 &&
            (size_t)p.a_stages * p.a_bytes + 4 * (size_t)p.plane_bytes + extra > 80 * 1024 &&
            (size_t)p.a_stages * p.a_bytes + 2 * (size_t)p.plane_bytes + extra <= 80 * 1024)
            p.b_stages = 1;
        const size_t staging = (size_t)p.a_stages * p.a_bytes + 2 * (size_t)p.b_stages * p.plane_bytes;
        p.bias_off = (int)staging;
        // behind the staging buffers: the bias of three tiles, and per wave a window of 4 filter pairs x its pixels
        // -- unless the shape is one whose registers leave room for a second workgroup on the compute unit and the
        // windows fit the weights' half of a staging buffer (or, where the weights stay, the activations' half): then
        // they live there
        // (channel-minor outputs: 32 pixels x the wave's filters, see epilogue_nhwc)
        const size_t windows = a.nhwc ? (size_t)(NTH / 64) * 32 * (sh.af * 64 + 8) : (size_t)(NTH / 64) * 4 * (sh.bf * 32 + 16) * 4;
        p.win_alias = 0;
        if (shares_cu && !a.nhwc) {
            if (p.a_stages == 2 && windows <= (size_t)p.a_bytes) p.win_alias = 1;
            if (p.a_stages == 1 && windows <= 2 * (size_t)p.plane_bytes) p.win_alias = 2;
        }
        lds = staging + 3 * (size_t)MT * 4 + (p.win_alias ? 0 : windows);
        p.flag_off = (int)lds;                   // one word for the channel split's "arrived last" flag
        lds += 16;
        if (lds > 160 * 1024) continue;
        if (a.nhwc) {
            if (2 * p.P > 12 * (NTH / 64)) continue;          // (pieces per wave that the kernel is built for)
            lw = 8;
            break;
        }
        // widest loads whose pieces fit the lanes; fewer rows only when even the narrowest fit nowhere
        int w = lw;
        const long long slots_all = (long long)p.max_slots * p.groups;
        while (w > 1 && slots_all * (a.W / w) > (long long)max_items(w) * (NTH / 2)) w /= 2;
        if (slots_all * (a.W / w) <= (long long)max_items(w) * (NTH / 2)) {
            lw = w;
            break;
        }
    }
    p.G = a.nhwc ? 1 : a.W / lw;                  // (channel-minor staging has no pieces of lw pixels)
    const int need_items = (int)(((long long)p.max_slots * p.groups * p.G + NTH / 2 - 1) / (NTH / 2));
    const int ki = a.nhwc ? 1 : lw == 8 ? std::max(need_items, 1) : lw == 4 ? std::max(need_items, 2) : need_items <= 3 ? 3 : lw == 2 ? 4 : 7;
    p.nhwc = a.nhwc ? 1 : 0;
    p.div_PW = make_fastdiv((unsigned)p.PW);
    p.R = R;
    p.tiles_n = (int)((total_rows + R - 1) / R);
    p.tiles_m = (a.F + MT - 1) / MT;
    p.sw = (a.Wo % 8 == 0 && ya % 16 == 0) ? 8 : (a.Wo % 4 == 0 && ya % 8 == 0) ? 4 : (a.Wo % 2 == 0 && ya % 4 == 0) ? 2 : 1;
    p.sw_groups = a.Wo / p.sw;
    for (int t = 0; t < p.nt; ++t) p.tap_off[t] = ((a.taps[t] / 3) * p.PW + a.taps[t] % 3) * (a.nhwc ? 32 : 16);
    // (channel ranges in the place of taps: range t lies max_slots row slots behind range t - 1)
    if (p.groups > 1)
        for (int t = 0; t < p.nt; ++t) p.tap_off[t] += a.nhwc ? t * (2 * p.P * 1024) : t * p.max_slots * p.PW * 16;
    p.x_bytes = (unsigned long long)a.N * a.C * a.H * a.W * 2ull;
    p.chan_bytes = (unsigned)((size_t)a.H * a.W * 2);
    p.group_bytes = p.groups > 1 ? (a.nhwc ? (unsigned)p.C * 2u : (unsigned)p.C * p.chan_bytes) : 0u;
    p.Cpix = a.C;
    const unsigned long long img = (unsigned long long)a.C * a.H * a.W * 2ull;
    if (img * (unsigned long long)(segs + 1) >= 0x7FFFFFFFull) return false;   // 32-bit offsets inside a tile's images
    p.img_bytes = (unsigned)img;
    p.y_bytes = (unsigned long long)a.N * a.F * a.Ho * a.Wo * 2ull;
    if ((unsigned long long)a.F * a.Ho * a.Wo * 2ull * (unsigned long long)(segs + 1) >= 0x7FFFFFFFull) return false;
    const size_t wq_bytes = a.d_clist ? a.w_bytes : mfma_weight_bytes(a.F, p.C, MT, p.nt);
    if (wq_bytes >= 0x7FFFFFFFull) return false;
    p.wq_bytes = (unsigned)wq_bytes;
    p.div_Wo = make_fastdiv((unsigned)a.Wo);
    p.div_Ho = make_fastdiv((unsigned)a.Ho);
    p.div_G = make_fastdiv((unsigned)p.G);
    p.div_cnt_full = make_fastdiv((unsigned)p.cnt_full);
    p.div_tiles_m = make_fastdiv((unsigned)p.tiles_m);
    p.div_sw_groups = make_fastdiv((unsigned)p.sw_groups);
    const long long ntiles = (long long)p.tiles_n * p.tiles_m * p.KS;
    if (ntiles > 0x7FFFFFF0) return false;
    // (the parts of one tile in the workspace are addressed with 32-bit offsets)
    if (p.KS > 1 && (unsigned long long)p.KS * MT * NT * 4ull >= 0x7FFFFFFFull) return false;
    const long long grid = 0;   // (decided at launch: persistent workgroups, see persistent_grid)
    *out = p;
    *lw_out = lw;
    *ki_out = ki;
    *lds_out = lds;
    *grid_out = (int)grid;
    return true;
}

}  // namespace

// Compute units of the current device (asked once per device, 256 if the runtime does not say).
int compute_units() {
    static std::mutex mu;
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (!cached[dev]) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

size_t mfma_weight_bytes(int F, int C, int mt, int n_taps) {
    return (size_t)((F + mt - 1) / mt) * ((C + 15) / 16) * n_taps * 2 * mt * 8 * sizeof(uint16_t);
}

int mfma_shape_height(int shape) {
    return shape >= 1 && shape <= kMfmaShapes ? kShapes[shape - 1].wm * kShapes[shape - 1].af * 32 : 0;
}

// Estimated run time, in microseconds, of the layer with tile shape `shape` (1..kMfmaShapes); negative if the shape
// cannot take it.  Rounds of resident workgroups times (a fixed part + channel blocks x time per block).  The block
// times are measured ones (MI355X, VGG-16 and ResNet-50 shapes); while a workgroup has its compute unit to itself a
// block cannot take less than the round trip of the loads that fetch the next one.
double mfma_estimate_us(const MfmaConv& a0, int shape, int splits) {
    if (shape < 1 || shape > kMfmaShapes) return -1.0;
    MfmaConv a = a0;
    a.mt = mfma_shape_height(shape);
    a.splits = splits;
    MfmaParams p;
    int lw = 0, ki = 0, grid = 0;
    size_t lds = 0;
    if (!plan(a, shape - 1, a.rows, &p, &lw, &ki, &lds, &grid)) return -1.0;
    const long long tiles = (long long)p.tiles_n * p.tiles_m * p.KS;
    // the shapes whose waves keep within half the registers leave room for a second workgroup on a compute unit, if
    // the LDS fits twice
    const int per_cu = (shape == 4 || p.win_alias) && 2 * lds <= 160 * 1024 ? 2 : 1;
    const long long resident = (long long)compute_units() * per_cu;
    const double rounds = (double)((tiles + resident - 1) / resident);
    // (while the device is not full a block lasts as long as the loads of the next one take to come back: measured
    // on ResNet-50's layers at batch 32, per shape, stride 1 / stride 2 -- a wider tile stages more rows per block)
    static const double kFloorUs[kMfmaShapes][2] = {{2.8, 2.8}, {2.0, 2.7}, {1.9, 2.2}, {1.75, 1.85}};
    // (a layer of one or two taps -- a 1x1 layer is a layer of centre taps -- multiplies for a fraction of the time its
    // next block's loads are under way, however full the device is: the round trip binds every block)
    const bool few_taps = p.nt <= 2;
    // (measured on the 1x1 layers of ResNet-50's bottlenecks at batch 32: 0.65 of the 3x3 layers' figure, whose blocks
    // stage three rows of halo besides)
    const double floor_us = (tiles <= resident || few_taps) ? kFloorUs[shape - 1][a.stride == 2 ? 1 : 0] * (few_taps ? 0.65 : 1.0) : 0.0;
    // (with channel lists: the mean number of blocks of a tile)
    const double all_blocks = a.d_clist ? (double)a.total_blocks / std::max(1, p.tiles_m) : (double)p.CB;
    const double blocks = std::ceil(all_blocks / p.KS);
    // Time of one channel block of one tile with the device full, and of what a tile costs besides its blocks
    // (epilogue, descriptors), microseconds, fitted to the nine VGG-16 shapes at batch 64: two workgroups that share
    // a compute unit take turns on its matrix cores, so each one's block lasts longer; rows of fewer than 56 pixels
    // mean narrower loads and stores.
    const bool narrow = a.W < 56;
    double block_us = kBlockUs[shape - 1], tile_us = 8.0;
    if (shape == 1) block_us = narrow ? 2.65 : 2.3;
    if (shape == 2) {
        const bool shared = per_cu == 2 && tiles > (long long)compute_units();
        block_us = shared ? (narrow ? 2.85 : 2.7) : 1.7;
        tile_us = shared ? 5.0 : 2.8;
    }
    if (shape == 3) tile_us = 5.0;
    if (shape == 4) {
        if (per_cu == 2 && tiles > (long long)compute_units()) block_us = 2.4;
        tile_us = 4.0;
    }
    // a split costs the round trip of the partial sums through memory and the last arriver's additions
    const double part_bytes = (double)tiles * (kShapes[shape - 1].wm * kShapes[shape - 1].af * 32) *
                              (kShapes[shape - 1].wn * kShapes[shape - 1].bf * 32) * 4.0;
    // (fitted to ResNet-50's 14 x 14 and 7 x 7 layers at batch 32 in 2, 4 and 8 parts)
    // (second pass: a launch, and the parts written once and read once -- fitted to ResNet-50's 3x3 and 1x1 layers
    // at batch 32: 4.5 TB/s, the parts of such layers staying in the memory-side cache)
    const double split_us = p.KS <= 1 ? 0.0 : a.second_pass ? 4.0 + 2.0 * part_bytes / 4.5e6
                                                             : 4.0 + 1.5 * (p.KS - 1) + part_bytes / 1.8e6;
    if (p.nt < 9) block_us *= (double)std::max(p.nt, 1) / 9.0;
    // A 1x1 layer with channel ranges in the place of taps multiplies for a fraction of the time that staging a
    // block takes its waves: 8 ki load instructions per lane and block with their address arithmetic, transposition
    // and LDS writes.  Fitted to ResNet-50's bottleneck layers at batch 32 (56 x 56 to 7 x 7 maps, 128 x 224 tiles):
    // 0.8 us + 0.1 us per load; 8 us per tile.  The other tile shapes stage twice the pieces per lane, or share the
    // compute unit, and lost on every one of those layers: they are priced out of the automatic choice.
    if (a.groups > 1) {
        const double staged_us = 0.8 + 0.1 * 8.0 * ki;
        return (rounds * (8.0 + blocks * staged_us) + split_us) * (shape == 3 ? 1.0 : 2.0);
    }
    return rounds * (tile_us + blocks * std::max(block_us, floor_us)) + split_us;
}

int mfma_workspace(const MfmaConv& a, size_t* floats, size_t* counters) {
    MfmaParams p;
    int lw = 0, ki = 0, grid = 0;
    size_t lds = 0;
    if (a.shape < 1 || a.shape > kMfmaShapes || !plan(a, a.shape - 1, a.rows, &p, &lw, &ki, &lds, &grid))
        return PCONV_EUNSUPPORTED;
    const Shape& sh = kShapes[a.shape - 1];
    const size_t tiles = (size_t)p.tiles_n * p.tiles_m;
    *floats = p.KS > 1 ? tiles * p.KS * (size_t)(sh.wm * sh.af * 32) * (size_t)(sh.wn * sh.bf * 32) : 0;
    *counters = p.KS > 1 ? tiles : 0;
    return PCONV_OK;
}

int launch_mfma_conv(const MfmaConv& a, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    MfmaParams p;
    int lw = 0, ki = 0, grid = 0;
    size_t lds = 0;
    const int shape = a.shape - 1;
    if (shape < 0 || shape >= kMfmaShapes) return PCONV_EUNSUPPORTED;
    if (!plan(a, shape, a.rows, &p, &lw, &ki, &lds, &grid)) return PCONV_EUNSUPPORTED;
    if (p.KS > 1 && (!p.ws || !p.counters)) return PCONV_EINVAL;
    int rc = PCONV_EUNSUPPORTED;
    switch (shape) {
        case 0: rc = launch_shape<2, 7, 2, 2>(p, lw, ki, lds, a.walk, kBlockUs[0], st); break;
        case 1: rc = launch_shape<1, 7, 2, 2>(p, lw, ki, lds, a.walk, kBlockUs[1], st); break;
        case 2: rc = launch_shape<1, 7, 4, 1>(p, lw, ki, lds, a.walk, kBlockUs[2], st); break;
        case 3: rc = launch_shape<1, 7, 2, 1>(p, lw, ki, lds, a.walk, kBlockUs[3], st); break;
    }
    if (rc != PCONV_OK || !p.second_pass) return rc;
    const Shape& sh = kShapes[shape];
    ReduceParams r{};
    r.ws = p.ws;
    r.y = p.y;
    r.N = p.N; r.F = p.F; r.Ho = p.Ho; r.Wo = p.Wo; r.relu = p.relu; r.nhwc = p.nhwc;
    r.KS = p.KS; r.R = p.R; r.tiles_m = p.tiles_m;
    r.AF = sh.af; r.BF = sh.bf; r.WM = sh.wm; r.WN = sh.wn;
    r.threads = (long long)p.tiles_n * p.tiles_m * (sh.wm * sh.wn) * sh.af * sh.bf * 4 * 64;
    const long long blocks = (r.threads + 255) / 256;
    if (blocks > 0x7FFFFFFF) return PCONV_EUNSUPPORTED;
    hipLaunchKernelGGL(mfma_split_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, r);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

int launch_mfma_arrange(const void* w_oihw, void* out, int F, int C, int mt, void* stream) {
    const int CB = (C + 15) / 16;
    const long long total = (long long)((F + mt - 1) / mt) * CB * 9 * 2 * mt * 8;
    const unsigned grid = (unsigned)std::min<long long>((total + 255) / 256, 65535);
    hipLaunchKernelGGL(mfma_arrange_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const unsigned short*>(w_oihw), static_cast<unsigned short*>(out), F, C, mt, CB, total);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

}  // namespace pconv
