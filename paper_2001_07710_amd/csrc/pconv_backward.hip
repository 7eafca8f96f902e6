// Weight gradient of the pruned 3x3 layer for fp16 storage on gfx950 (MI355X): G[f][c][ky][kx] = sum over the batch's
// output pixels of dy[n][f][oy][ox] * x[n][c][oy+ky-1][ox+kx-1] (stride 1, padding 1), kept for the weights the layer
// keeps (the primal step of section 5.1 of the paper trains those by SGD through the masked layer: dL/dW = G o M).
//
// Why a dense contraction again.  Per tap this is a matrix product over the pixels, [filter][pixel] x [pixel][channel],
// and on this chip the fp16 matrix cores run it 16 times faster than the vector ALU would run the kept products
// alone; the mask is applied when the result is gathered.  Both operands are pixel-minor in NCHW, which is the K
// layout v_mfma_f32_32x32x16_f16 wants: a lane's operand is 8 consecutive pixels of one filter (or channel), 16
// contiguous bytes.  No transposition anywhere.
//
// Tile.  A workgroup of four waves owns 64 filters x 64 channels x 9 taps (a wave: 32 x 32 x 9, 144 accumulators)
// and walks over chunks of the pixels: R output rows x Gc groups of 8 columns of one image.  Per chunk it stages
//   x   [input row r'][group g][channel][8 pixels]            rows oy0-1 .. oy0+R, one 16-byte piece per (channel, r', g)
//   dy  [row r][group j][filter][8 pixels]                    groups one left and one right more than x has
// 1040 bytes from one (row, group) to the next, so that neighbouring groups of one channel fall on different banks
// when they are written and the 32 filters (channels) of an operand read lie side by side.  The three taps of a
// kernel row share one read of x: the sum over ox of dy[ox] * x[ox+kx-1] is the sum over x's own columns ox' of
// dy[ox'+1-kx] * x[ox'], so kx = 1 multiplies x with dy's group as it is, and kx = 0 / 2 with the same eight pixels of
// dy moved by one with the first / last pixel of the neighbouring group (eight v_alignbyte_b32 per K step of nine
// MFMAs).  Those neighbour words are staged a second time, 8 bytes per (row, group, filter) side by side over the
// filters, so that dy is one 128-bit and one 64-bit read free of bank conflicts.  Zero padding is nothing but dy's
// zero halo: columns beyond the image, rows beyond it, filters beyond F and channels beyond C are loads at an
// offset outside the buffer descriptor.  The loads of the next chunk are in flight, in registers, while the current
// one is multiplied.  (First version: the shifts on the x side, three per kernel row -- 24 vector instructions, seven
// LDS reads and a dozen of address arithmetic per nine MFMAs, and the one wave a SIMD has here cannot issue that many
// beside its MFMAs: 19 to 26 % of the matrix cores' rate.)
//
// The pixels are split over S workgroups per tile; each writes its 9 x 64 x 64 partial sums to the workspace, a second
// kernel adds the S parts in order, and a third gathers the sums of the kept weights into the canonical entry order
// of the packed layer (deterministic: no atomics).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pconv_backward.h"
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

constexpr uint32_t kInvalid = 0x80000000u;
constexpr int kPitch = 64 * 16 + 16;          // bytes from one (row, group) of a staged operand to the next
constexpr int kPitchE = 64 * 8 + 8;           // the same for the neighbour words of dy (8 bytes per filter)
constexpr int kMaxX = 12, kMaxD = 10;         // 16-byte pieces per thread and chunk, at most: x, dy
constexpr int kTile = 64;

struct GwParams {
    const unsigned char* x;
    const unsigned char* dy;
    float* ws;
    int N, C, F, H, W;
    int R, Gc, NJ;            // output rows and column groups per chunk; NJ = Gc + 2 staged groups of dy
    int nrb, ncb;             // row blocks and column blocks per image
    int chunks;               // N * nrb * ncb
    int S;                    // workgroups per tile
    int tiles_c, tiles;       // channel tiles; all tiles
    int npx, npd;             // pieces per thread: x, dy
    unsigned x_img_bytes, dy_img_bytes;
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// eight consecutive fp16 elements from byte offset `off` (kInvalid: zeros), LW elements per load
template <int LW>
__device__ __forceinline__ uint4v load8(__amdgpu_buffer_rsrc_t r, const uint32_t (&off)[8 / LW]) {
    uint4v v;
    if constexpr (LW == 8) {
        v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off[0], 0, 0);
    } else if constexpr (LW == 4) {
        const uint2v a = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off[0], 0, 0);
        const uint2v b = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off[1], 0, 0);
        v = uint4v{a.x, a.y, b.x, b.y};
    } else if constexpr (LW == 2) {
        v.x = __builtin_amdgcn_raw_buffer_load_b32(r, (int)off[0], 0, 0);
        v.y = __builtin_amdgcn_raw_buffer_load_b32(r, (int)off[1], 0, 0);
        v.z = __builtin_amdgcn_raw_buffer_load_b32(r, (int)off[2], 0, 0);
        v.w = __builtin_amdgcn_raw_buffer_load_b32(r, (int)off[3], 0, 0);
    } else {
        unsigned h[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) h[u] = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)off[u], 0, 0);
        v = uint4v{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    }
    return v;
}

template <int LW>
__global__ __launch_bounds__(256, 1) void grad_weight_kernel(const GwParams p) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wf = wave >> 1, wc = wave & 1, li = lane & 31, lk = lane >> 5;
    const int tile = (int)blockIdx.x / p.S, split = (int)blockIdx.x - tile * p.S;
    const int tf = tile / p.tiles_c, tc = tile - tf * p.tiles_c;
    const int R = p.R, Gc = p.Gc, NJ = p.NJ, H = p.H, W = p.W;
    unsigned char* const dyL = lds;                               // [r][j < NJ][filter][8 pixels]
    unsigned char* const eL = dyL + R * NJ * kPitch;              // [r][j][filter]{left neighbours, right neighbours}
    unsigned char* const xL = eL + R * NJ * kPitchE;              // [r' < R + 2][g < Gc][channel][8 pixels]

    // ---- this thread's pieces of a chunk (the same for every chunk): where they go in LDS, and where they come
    // from relative to the chunk's first output row and column
    int xl[kMaxX], xrel[kMaxX], xrg[kMaxX];      // xrg: row r' | group g << 8
    int dl[kMaxD], drel[kMaxD], drj[kMaxD];      // drj: row r | group j << 8
#pragma unroll
    for (int i = 0; i < kMaxX; ++i) {
        const int idx = tid + i * 256;
        const int g = idx % Gc, q = idx / Gc, c = q & 63, r = q >> 6;
        const int chan = tc * kTile + c;
        const bool ok = r < R + 2 && chan < p.C;
        xl[i] = r < R + 2 ? (r * Gc + g) * kPitch + c * 16 : -1;
        xrel[i] = ok ? (chan * H * W + (r - 1) * W + g * 8) * 2 : (int)kInvalid;
        xrg[i] = r | (g << 8);
    }
#pragma unroll
    for (int i = 0; i < kMaxD; ++i) {
        const int idx = tid + i * 256;
        const int j = idx % NJ, q = idx / NJ, f = q & 63, r = q >> 6;
        const int filt = tf * kTile + f;
        const bool ok = r < R && filt < p.F;
        dl[i] = r < R ? (r * NJ + j) * kPitch + f * 16 : -1;
        drel[i] = ok ? (filt * H * W + r * W + (j - 1) * 8) * 2 : (int)kInvalid;
        drj[i] = r | (j << 8);
    }

    uint4v xs[kMaxX], ds[kMaxD];
    auto fetch = [&](int chunk) {
        const int cb = chunk % p.ncb, q = chunk / p.ncb, rb = q % p.nrb, n = q / p.nrb;
        const int oy0 = rb * R, col0 = cb * Gc * 8;
        const __amdgpu_buffer_rsrc_t xr = make_rsrc(p.x + (size_t)n * p.x_img_bytes, p.x_img_bytes);
        const __amdgpu_buffer_rsrc_t dr = make_rsrc(p.dy + (size_t)n * p.dy_img_bytes, p.dy_img_bytes);
        const int shift = (oy0 * W + col0) * 2;
#pragma unroll
        for (int i = 0; i < kMaxX; ++i) {
            if (i < p.npx) {
                const int iy = oy0 + (xrg[i] & 255) - 1, col = col0 + (xrg[i] >> 8) * 8;
                const bool row_ok = xrel[i] != (int)kInvalid && iy >= 0 && iy < H;
                uint32_t off[8 / LW];
#pragma unroll
                for (int u = 0; u < 8 / LW; ++u)
                    off[u] = (row_ok && col + u * LW < W) ? (uint32_t)(xrel[i] + shift + u * LW * 2) : kInvalid;
                xs[i] = load8<LW>(xr, off);
            }
        }
#pragma unroll
        for (int i = 0; i < kMaxD; ++i) {
            if (i < p.npd) {
                const int oy = oy0 + (drj[i] & 255), col = col0 + ((drj[i] >> 8) - 1) * 8;
                const bool row_ok = drel[i] != (int)kInvalid && oy < H;
                uint32_t off[8 / LW];
#pragma unroll
                for (int u = 0; u < 8 / LW; ++u) {
                    const int cc = col + u * LW;
                    off[u] = (row_ok && cc >= 0 && cc < W) ? (uint32_t)(drel[i] + shift + u * LW * 2) : kInvalid;
                }
                ds[i] = load8<LW>(dr, off);
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < kMaxX; ++i)
            if (i < p.npx && xl[i] >= 0) *reinterpret_cast<uint4v*>(xL + xl[i]) = xs[i];
#pragma unroll
        for (int i = 0; i < kMaxD; ++i)
            if (i < p.npd && dl[i] >= 0) {
                *reinterpret_cast<uint4v*>(dyL + dl[i]) = ds[i];
                // this piece's last two pixels are the left neighbours of the group to its right, its first two the
                // right neighbours of the group to its left (only groups 1 .. Gc are ever multiplied)
                const int j = drj[i] >> 8;
                const int e = (dl[i] / kPitch) * kPitchE + ((dl[i] % kPitch) >> 1);
                if (j < NJ - 1) *reinterpret_cast<unsigned*>(eL + e + kPitchE) = ds[i].w;
                if (j >= 1) *reinterpret_cast<unsigned*>(eL + e - kPitchE + 4) = ds[i].x;
            }
    };

    float16v acc[3][3];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int kx = 0; kx < 3; ++kx)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ky][kx][i] = 0.f;

    const int nk = R * Gc / 2;                  // K steps of 16 pixels per chunk (R*Gc is even)
    const int a_lane = (wf * 32 + li) * 16, b_lane = (wc * 32 + li) * 16;
    // This half-wave's items are lk, lk + 2, ...; item = r*Gc + g.  x has no halo groups, so an item's x slot is the
    // item number plus ky rows; its dy slot is r*NJ + g + 1, which skips the two halo groups at every row end.
    const bool one_group = Gc == 1;             // (then every item is a row of its own: three dy slots per item)
    const int a_slot0 = one_group ? lk * 3 + 1 : lk + 1;
    const int row_b = Gc * kPitch;
    struct RawA {
        uint4v cur;
        uint2v nb;
    };
    auto read_a = [&](int slot) {
        RawA w;
        w.cur = *reinterpret_cast<const uint4v*>(dyL + slot * kPitch + a_lane);
        w.nb = *reinterpret_cast<const uint2v*>(eL + slot * kPitchE + (a_lane >> 1));
        return w;
    };
    auto read_b = [&](int off, int ky) { return *reinterpret_cast<const half8*>(xL + off + ky * row_b); };

    int chunk = split;
    if (chunk < p.chunks) fetch(chunk);
    while (chunk < p.chunks) {
        stage();
        __syncthreads();
        const int next = chunk + p.S;
        if (next < p.chunks) fetch(next);
        // The operands of a K step are requested one step ahead, each as soon as its registers are free, so the LDS
        // has nine MFMAs' time to answer.  The shifts by one pixel are made on the dy side: the sum over ox of
        // dy[ox] * x[ox + kx - 1] is the sum over x's own columns ox' of dy[ox' + 1 - kx] * x[ox'], so one read of x
        // per kernel row serves its three taps, and dy is read once per step and moved left and right by one pixel
        // with its neighbour words (eight v_alignbyte_b32 per nine MFMAs; with the shifts on the x side it was 24
        // vector instructions per step, and a single wave per SIMD cannot issue that many beside its MFMAs).
        int g = lk, a_slot = a_slot0, b_off = lk * kPitch + b_lane;
        RawA ra = read_a(a_slot);
        half8 b[3];
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) b[ky] = read_b(b_off, ky);
        for (int k = 0; k < nk; ++k) {
            // the items after these (behind the last: the first again, whose operands are read and not used)
            g += 2;
            const bool wrap = g >= Gc;
            g = wrap ? g - Gc : g;
            a_slot += one_group ? 6 : wrap ? 4 : 2;
            b_off += 2 * kPitch;
            if (k + 1 == nk) {
                g = lk;
                a_slot = a_slot0;
                b_off = lk * kPitch + b_lane;
            }
            __builtin_amdgcn_sched_barrier(0);
            const uint4v cur = ra.cur;
            const unsigned l0 = __builtin_amdgcn_alignbyte(cur.x, ra.nb.x, 2);
            const unsigned l1 = __builtin_amdgcn_alignbyte(cur.y, cur.x, 2);
            const unsigned l2 = __builtin_amdgcn_alignbyte(cur.z, cur.y, 2);
            const unsigned l3 = __builtin_amdgcn_alignbyte(cur.w, cur.z, 2);
            const unsigned r3 = __builtin_amdgcn_alignbyte(ra.nb.y, cur.w, 2);
            const half8 a2 = __builtin_bit_cast(half8, uint4v{l0, l1, l2, l3});      // dy at column ox' - 1: tap kx = 2
            const half8 a1 = __builtin_bit_cast(half8, cur);                          // ox': kx = 1
            const half8 a0 = __builtin_bit_cast(half8, uint4v{l1, l2, l3, r3});      // ox' + 1: kx = 0
            ra = read_a(a_slot);
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) {
                __builtin_amdgcn_sched_barrier(0);
                acc[ky][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b[ky], acc[ky][0], 0, 0, 0);
                acc[ky][1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b[ky], acc[ky][1], 0, 0, 0);
                acc[ky][2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a2, b[ky], acc[ky][2], 0, 0, 0);
                b[ky] = read_b(b_off, ky);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        chunk = next;
    }

    // ---- partial sums: ws[split][tile][tap][filter in tile][channel in tile]; accumulator row i of a 32 x 32 block
    // is filter (i/4)*8 + (lane/32)*4 + i%4, its column (lane%32) the channel
    float* const out = p.ws + ((size_t)split * p.tiles + tile) * (9 * kTile * kTile);
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int kx = 0; kx < 3; ++kx)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int f = wf * 32 + (i >> 2) * 8 + lk * 4 + (i & 3), c = wc * 32 + li;
                out[((ky * 3 + kx) * kTile + f) * kTile + c] = acc[ky][kx][i];
            }
}

// The S parts of every tile added into part 0, in order: a dense pass, four neighbouring sums per thread, so the parts
// are read at the rate of a copy.  (Summed inside the gather below instead, one scattered 4-byte read per part and kept
// weight, the parts of a layer with a single tile -- 256 of them -- took 90 us.)
__global__ __launch_bounds__(256) void grad_weight_reduce_kernel(float* __restrict__ ws, long long n4, long long part4, int S,
                                                                 int step, int cnt) {
    // group blockIdx.y: parts (group*cnt + s)*step, s < cnt, as far as there are parts, added into the group's first
    typedef float float4v __attribute__((ext_vector_type(4)));
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    float4v* const w4 = reinterpret_cast<float4v*>(ws);
    const long long first = (long long)blockIdx.y * cnt * step;
    float4v sum = w4[first * part4 + i];
    for (int s = 1; s < cnt && first + (long long)s * step < S; ++s) sum += w4[(first + (long long)s * step) * part4 + i];
    w4[first * part4 + i] = sum;
}

// dw4[e][q] = sum over the S parts, in order, of the partial sum of entry e's filter and channel at the q-th tap of
// its pattern
__global__ __launch_bounds__(256) void grad_weight_gather_kernel(const float* __restrict__ ws, const uint32_t* __restrict__ canon,
                                                                 float* __restrict__ dw4, long long n4, int S, int tiles,
                                                                 int tiles_c) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    const long long e = i >> 2;
    const int q = (int)(i & 3);
    const uint32_t f = canon[e * 2], cm = canon[e * 2 + 1], c = cm & 0xFFFFu, mask = cm >> 16;
    int t = -1, seen = 0;
    for (int b = 0; b < 9; ++b)
        if ((mask >> b) & 1u) {
            if (seen == q) t = b;
            ++seen;
        }
    float sum = 0.f;
    if (t >= 0) {
        const int tile = (int)(f / kTile) * tiles_c + (int)(c / kTile);
        const size_t at = ((size_t)tile * 9 + t) * (kTile * kTile) + (f % kTile) * kTile + (c % kTile);
        for (int s = 0; s < S; ++s) sum += ws[(size_t)s * tiles * (9 * kTile * kTile) + at];
    }
    dw4[i] = sum;
}

// Chunk geometry and the split of the pixels for a layer shape; false if the kernel cannot take it.
bool plan(const pconv_packed* p, int N, int H, int W, GwParams* out, int* lw, size_t* lds, size_t* ws_floats) {
    GwParams g{};
    g.N = N; g.C = p->C; g.F = p->F; g.H = H; g.W = W;
    const int Gp = (W + 7) / 8;
    g.ncb = (Gp + 7) / 8;
    g.Gc = (Gp + g.ncb - 1) / g.ncb;
    g.NJ = g.Gc + 2;
    // rows per chunk: even (a K step is two items), as many as the pieces per thread allow, evened out over the image
    int R = 2;
    while (R + 2 <= 254 && ((R + 4) * g.Gc * 64 + 255) / 256 <= kMaxX && ((R + 2) * g.NJ * 64 + 255) / 256 <= kMaxD) R += 2;
    if (((R + 2) * g.Gc * 64 + 255) / 256 > kMaxX || (R * g.NJ * 64 + 255) / 256 > kMaxD) return false;
    int nrb = (H + R - 1) / R;
    R = std::min(R, ((H + nrb - 1) / nrb + 1) / 2 * 2);
    nrb = (H + R - 1) / R;
    g.R = R;
    g.nrb = nrb;
    const long long chunks = (long long)N * nrb * g.ncb;
    if (chunks > 0x7FFFFFFF) return false;
    g.chunks = (int)chunks;
    g.tiles_c = (p->C + kTile - 1) / kTile;
    g.tiles = g.tiles_c * ((p->F + kTile - 1) / kTile);
    const int cus = compute_units();
    g.S = (int)std::max<long long>(1, std::min<long long>(chunks, (cus + g.tiles - 1) / g.tiles));
    g.npx = ((R + 2) * g.Gc * 64 + 255) / 256;
    g.npd = (R * g.NJ * 64 + 255) / 256;
    const unsigned long long ximg = (unsigned long long)p->C * H * W * 2ull, dimg = (unsigned long long)p->F * H * W * 2ull;
    if (ximg >= 0x7FFFFFFFull || dimg >= 0x7FFFFFFFull) return false;
    g.x_img_bytes = (unsigned)ximg;
    g.dy_img_bytes = (unsigned)dimg;
    *lw = W % 8 == 0 ? 8 : W % 4 == 0 ? 4 : W % 2 == 0 ? 2 : 1;
    *lds = (size_t)(R * g.NJ + (R + 2) * g.Gc) * kPitch + (size_t)R * g.NJ * kPitchE;
    if (*lds > 160 * 1024) return false;
    *ws_floats = (size_t)g.S * g.tiles * 9 * kTile * kTile;
    *out = g;
    return true;
}

int check_args(const pconv_packed* p, int N, int H, int W, int stride, int pad) {
    if (!p) return PCONV_EINVAL;
    if (N < 0 || H <= 0 || W <= 0) return PCONV_ESHAPE;
    if (p->dtype != PCONV_F16 || stride != 1 || pad != 1 || p->is_1x1) return PCONV_EUNSUPPORTED;
    for (uint16_t m : p->lib)
        if (__builtin_popcount(m) != 4) return PCONV_EUNSUPPORTED;      // (a derived form, not a layer from pconv_pack)
    return PCONV_OK;
}

}  // namespace
}  // namespace pconv

using namespace pconv;

extern "C" int pconv_conv3x3_grad_weight_workspace(const pconv_packed* p, int N, int H, int W, int stride, int pad,
                                                   size_t* bytes) {
    if (!bytes) return PCONV_EINVAL;
    *bytes = 0;
    if (int rc = check_args(p, N, H, W, stride, pad)) return rc;
    if (N == 0 || p->n_kept == 0) return PCONV_OK;
    GwParams g;
    int lw = 0;
    size_t lds = 0, floats = 0;
    if (!plan(p, N, H, W, &g, &lw, &lds, &floats)) return PCONV_EUNSUPPORTED;
    *bytes = floats * sizeof(float);
    return PCONV_OK;
}

extern "C" int pconv_conv3x3_grad_weight(const void* x, const void* dy, const pconv_packed* p, float* dw4, int N, int H,
                                         int W, int stride, int pad, void* workspace, size_t workspace_bytes,
                                         void* stream) {
    if (int rc = check_args(p, N, H, W, stride, pad)) return rc;
    if (!x || !dy || !dw4) return PCONV_EINVAL;
    if (!p->d_canon) return PCONV_ESTATE;
    int dev = -1;
    PCONV_HIP(hipGetDevice(&dev));
    if (dev != p->device) return PCONV_ESTATE;
    if (p->n_kept == 0) return PCONV_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const long long n4 = (long long)p->n_kept * 4;
    GwParams g;
    int lw = 0;
    size_t lds = 0, floats = 0;
    if (!plan(p, std::max(N, 1), H, W, &g, &lw, &lds, &floats)) return PCONV_EUNSUPPORTED;
    if (!workspace || workspace_bytes < floats * sizeof(float)) return PCONV_EINVAL;
    if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(dy)) % 2) return PCONV_EINVAL;
    // (the widest loads that the pointers allow as well as the row length)
    while (lw > 1 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(dy)) % (2 * lw))) lw /= 2;
    g.x = static_cast<const unsigned char*>(x);
    g.dy = static_cast<const unsigned char*>(dy);
    g.ws = static_cast<float*>(workspace);
    g.N = N;
    if (N == 0) g.chunks = 0;          // (no pixels: the workgroups write zeros, the gather adds them)
    const dim3 grid((unsigned)(g.tiles * g.S));
#define PCONV_GW_CASE(LWv)                                                                                              \
    if (lw == LWv) {                                                                                                    \
        auto kern = grad_weight_kernel<LWv>;                                                                            \
        if (lds > 64 * 1024)                                                                                            \
            PCONV_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));    \
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, g);                                                          \
    }
    PCONV_GW_CASE(8) PCONV_GW_CASE(4) PCONV_GW_CASE(2) PCONV_GW_CASE(1)
#undef PCONV_GW_CASE
    PCONV_HIP(hipGetLastError());
    if (g.S > 1) {
        const long long part4 = (long long)g.tiles * 9 * kTile * kTile / 4;
        // (in two levels where there are many parts, so that the first level has workgroups enough: groups of 16
        // consecutive parts, then the groups' sums; the order of the additions is fixed either way)
        const unsigned blocks = (unsigned)((part4 + 255) / 256);
        const int groups = g.S > 16 ? (g.S + 15) / 16 : 1;
        if (groups > 1) {
            hipLaunchKernelGGL(grad_weight_reduce_kernel, dim3(blocks, (unsigned)groups), dim3(256), 0, st,
                               static_cast<float*>(workspace), part4, part4, g.S, 1, 16);
            PCONV_HIP(hipGetLastError());
        }
        hipLaunchKernelGGL(grad_weight_reduce_kernel, dim3(blocks, 1u), dim3(256), 0, st, static_cast<float*>(workspace),
                           part4, part4, g.S, groups > 1 ? 16 : 1, groups > 1 ? groups : g.S);
        PCONV_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(grad_weight_gather_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float*>(workspace), p->d_canon, dw4, n4, 1, g.tiles, g.tiles_c);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}
