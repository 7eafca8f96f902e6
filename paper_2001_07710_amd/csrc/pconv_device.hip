// Device side of libpconv for gfx950 (MI355X): kernels, launch selection, device upload of the packed weights.
//
// Kernels in this file
//   tiled_kernel    pattern-sparse 3x3 convolution at unit stride: one input column per lane, activations staged in
//                   LDS in a lane-shaped layout, one or two filters per wave, one generated code section per
//                   pattern; stride 2 runs through it on the layer re-packed over the four parity planes of the input
//   quad_kernel     the same with four input columns per lane (64 multiply-adds per kept kernel instead of 28,
//                   128-bit staging loads): for layers with enough output tiles to fill the chip with larger tiles
//   parity_planes_kernel  the split of the input into those planes
//   generic_kernel  the same sum for any stride and pad, one thread per output, straight from global memory
//   dense_kernel    dense 3x3 convolution of the same shape (comparison baseline)
//   maxpool_kernel  2x2 max-pool
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <type_traits>

#include "pconv_internal.h"

namespace pconv {

// ---------------------------------------------------------------------------------------------------------------
// error text
// ---------------------------------------------------------------------------------------------------------------

static thread_local char g_hip_error[256] = "";

void set_hip_error(const char* what, int hip_code) {
    std::snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString((hipError_t)hip_code));
}

#define PCONV_HIP(call)                                  \
    do {                                                 \
        hipError_t e_ = (call);                          \
        if (e_ != hipSuccess) {                          \
            pconv::set_hip_error(#call, (int)e_);        \
            return PCONV_EHIP;                           \
        }                                                \
    } while (0)

// ---------------------------------------------------------------------------------------------------------------
// upload / release
// ---------------------------------------------------------------------------------------------------------------

int upload_packed(pconv_packed* p) {
    int dev = -1;
    PCONV_HIP(hipGetDevice(&dev));
    const size_t n_ent = std::max<size_t>(p->ent.size(), 1);
    PCONV_HIP(hipMalloc((void**)&p->d_ent, n_ent * sizeof(DevEntry)));
    PCONV_HIP(hipMalloc((void**)&p->d_eptr, p->eptr.size() * sizeof(uint32_t)));
    PCONV_HIP(hipMalloc((void**)&p->d_forder, p->filter_order.size() * sizeof(uint32_t)));
    if (!p->ent.empty())
        PCONV_HIP(hipMemcpy(p->d_ent, p->ent.data(), p->ent.size() * sizeof(DevEntry), hipMemcpyHostToDevice));
    else
        PCONV_HIP(hipMemset(p->d_ent, 0, sizeof(DevEntry)));
    PCONV_HIP(hipMemcpy(p->d_eptr, p->eptr.data(), p->eptr.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    PCONV_HIP(hipMemcpy(p->d_forder, p->filter_order.data(), p->filter_order.size() * sizeof(uint32_t),
                        hipMemcpyHostToDevice));
    for (BalancedLayout& b : p->balanced) {
        PCONV_HIP(hipMalloc((void**)&b.d_ent, std::max<size_t>(b.ent.size(), 1) * sizeof(DevEntry)));
        PCONV_HIP(hipMalloc((void**)&b.d_eptr, b.eptr.size() * sizeof(uint32_t)));
        PCONV_HIP(hipMalloc((void**)&b.d_perm, std::max<size_t>(b.perm.size(), 1) * sizeof(uint32_t)));
        if (!b.ent.empty())
            PCONV_HIP(hipMemcpy(b.d_ent, b.ent.data(), b.ent.size() * sizeof(DevEntry), hipMemcpyHostToDevice));
        PCONV_HIP(hipMemcpy(b.d_eptr, b.eptr.data(), b.eptr.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
        if (!b.perm.empty())
            PCONV_HIP(hipMemcpy(b.d_perm, b.perm.data(), b.perm.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    }
    PCONV_HIP(hipMalloc((void**)&p->d_canon, std::max<size_t>(p->canon.size(), 2) * sizeof(uint32_t)));
    if (!p->canon.empty())
        PCONV_HIP(hipMemcpy(p->d_canon, p->canon.data(), p->canon.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
    for (MfmaWeights& m : p->mfma) {
        PCONV_HIP(hipMalloc(&m.d_w, std::max<size_t>(m.bytes(), 16)));
        if (m.bytes()) PCONV_HIP(hipMemcpy(m.d_w, m.w.data(), m.bytes(), hipMemcpyHostToDevice));
        if (!m.clist.empty()) {
            PCONV_HIP(hipMalloc((void**)&m.d_clist, m.clist.size() * sizeof(uint32_t)));
            PCONV_HIP(hipMemcpy(m.d_clist, m.clist.data(), m.clist.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
            PCONV_HIP(hipMalloc((void**)&m.d_tinfo, m.tinfo.size() * sizeof(uint32_t)));
            PCONV_HIP(hipMemcpy(m.d_tinfo, m.tinfo.data(), m.tinfo.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
        }
    }
    p->device = dev;
    return PCONV_OK;
}

void release_device(pconv_packed* p) {
    for (MfmaWeights& m : p->mfma) {
        if (m.d_w) (void)hipFree(m.d_w);
        if (m.d_clist) (void)hipFree(m.d_clist);
        if (m.d_tinfo) (void)hipFree(m.d_tinfo);
        m.d_w = nullptr;
        m.d_clist = nullptr;
        m.d_tinfo = nullptr;
    }
    if (p->d_canon) (void)hipFree(p->d_canon);
    p->d_canon = nullptr;
    if (p->d_ent) (void)hipFree(p->d_ent);
    if (p->d_eptr) (void)hipFree(p->d_eptr);
    if (p->d_forder) (void)hipFree(p->d_forder);
    for (BalancedLayout& b : p->balanced) {
        if (b.d_ent) (void)hipFree(b.d_ent);
        if (b.d_eptr) (void)hipFree(b.d_eptr);
        if (b.d_perm) (void)hipFree(b.d_perm);
        b.d_ent = nullptr;
        b.d_eptr = nullptr;
        b.d_perm = nullptr;
    }
    if (p->d_ws) (void)hipFree(p->d_ws);
    if (p->d_counters) (void)hipFree(p->d_counters);
    if (p->d_planes) (void)hipFree(p->d_planes);
    p->d_planes = nullptr;
    p->planes_bytes = 0;
    p->d_ws = nullptr;
    p->ws_floats = 0;
    p->d_counters = nullptr;
    p->n_counters = 0;
    p->d_ent = nullptr;
    p->d_eptr = nullptr;
    p->d_forder = nullptr;
    p->device = -1;
}

// Makes the handle's workspace at least `floats` partial sums and `counters` arrival counters large.  Counters are
// zero when allocated and every kernel leaves them zero.
static int ensure_workspace(const pconv_packed* p, size_t floats, size_t counters) {
    if (floats > p->ws_floats) {
        if (p->d_ws) PCONV_HIP(hipFree(p->d_ws));   // hipFree waits for work that may still use it
        p->d_ws = nullptr;
        p->ws_floats = 0;
        PCONV_HIP(hipMalloc(reinterpret_cast<void**>(&p->d_ws), floats * sizeof(float)));
        p->ws_floats = floats;
    }
    if (counters > p->n_counters) {
        if (p->d_counters) PCONV_HIP(hipFree(p->d_counters));
        p->d_counters = nullptr;
        p->n_counters = 0;
        PCONV_HIP(hipMalloc(reinterpret_cast<void**>(&p->d_counters), counters * sizeof(unsigned)));
        PCONV_HIP(hipMemset(p->d_counters, 0, counters * sizeof(unsigned)));
        p->n_counters = counters;
    }
    return PCONV_OK;
}

// ---------------------------------------------------------------------------------------------------------------
// the fixed arena of pconv_conv3x3_noalloc
//
// Callers that may not allocate (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc) get the
// channel split's partial sums and arrival counters from a file-scope device array instead of the handle's growing
// workspace.  Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends; the address is looked up once per device (hipGetSymbolAddress with that device current) and host code only
// ever uses the looked-up pointer.  Layout: kArenaCounters arrival counters, then kArenaFloats partial sums.
// ---------------------------------------------------------------------------------------------------------------

constexpr size_t kArenaCounters = 16384;            // one per output tile of a split launch
constexpr size_t kArenaFloats = (size_t)6 << 20;    // 24 MiB of partial sums
constexpr size_t kArenaBytes = kArenaCounters * sizeof(unsigned) + kArenaFloats * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kArenaBytes];

struct WsArena {
    float* ws;
    size_t floats;
    unsigned* counters;
    size_t n_counters;
};

constexpr int kMaxDevices = 64;
static std::mutex g_arena_mutex;
static void* g_arena_ptr[kMaxDevices] = {};

// The arena of the current device.
static int current_arena(WsArena* out) {
    int dev = -1;
    PCONV_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PCONV_EUNSUPPORTED;
    void* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_arena_mutex);
        if (!g_arena_ptr[dev]) {
            void* ptr = nullptr;
            PCONV_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            if (!ptr) return PCONV_EHIP;
            g_arena_ptr[dev] = ptr;
        }
        base = g_arena_ptr[dev];
    }
    out->counters = static_cast<unsigned*>(base);
    out->n_counters = kArenaCounters;
    out->ws = reinterpret_cast<float*>(static_cast<unsigned char*>(base) + kArenaCounters * sizeof(unsigned));
    out->floats = kArenaFloats;
    return PCONV_OK;
}

__global__ __launch_bounds__(256) void clear_counters_kernel(unsigned* counters, unsigned n) {
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i < n) counters[i] = 0u;
}

// Partial-sum workspace and arrival counters for a split launch: the handle's own (grown on demand) or, when the
// caller may not allocate, the fixed arena, whose counters are cleared on the launch stream first (the arena keeps
// what the last call left, and a launch that was aborted may have left counters that are not zero).
static int get_workspace(const pconv_packed* wp, const WsArena* arena, size_t floats, size_t counters, float** ws,
                         unsigned** cnt, hipStream_t stream) {
    if (!arena) {
        if (int rc = ensure_workspace(wp, floats, counters)) return rc;
        *ws = wp->d_ws;
        *cnt = wp->d_counters;
        return PCONV_OK;
    }
    if (floats > arena->floats || counters > arena->n_counters) return PCONV_ESCRATCH;
    hipLaunchKernelGGL(clear_counters_kernel, dim3((unsigned)((counters + 255) / 256)), dim3(256), 0, stream,
                       arena->counters, (unsigned)counters);
    PCONV_HIP(hipGetLastError());
    *ws = arena->ws;
    *cnt = arena->counters;
    return PCONV_OK;
}

// ---------------------------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------------------------

template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f32<__half>(__half v) { return __half2float(v); }

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ __half from_f32<__half>(float v) { return __float2half_rn(v); }

// Raw buffer descriptor over `bytes` bytes at `base`: loads whose per-lane offset is at or beyond `bytes` return
// zero without touching memory, which is how padding and ragged tiles are read.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

constexpr uint32_t kInvalidOffset = 0x80000000u;

// One element as it is stored, in the low bits of a 32-bit register.  Loading and widening are two steps on purpose:
// a conversion right behind the load would make the wave wait for the load at once, and the point of loading a chunk
// ahead is that it stays in flight while the chunk before it is multiplied.
template <typename T>
__device__ __forceinline__ unsigned buffer_load_raw(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff);
template <>
__device__ __forceinline__ unsigned buffer_load_raw<float>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0);
}
template <>
__device__ __forceinline__ unsigned buffer_load_raw<__half>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)voff, (int)soff, 0);
}
// Two neighbouring elements (an even and the following odd column) in one load, as stored: two registers for fp32,
// the two halves of `a` for fp16 (`b` is not written).  pair_to_f32 takes them apart, later, for the same reason.
template <typename T>
__device__ __forceinline__ void buffer_load_raw2(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff, unsigned& a,
                                                 unsigned& b);
template <>
__device__ __forceinline__ void buffer_load_raw2<float>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff,
                                                        unsigned& a, unsigned& b) {
    typedef unsigned v2u __attribute__((ext_vector_type(2)));
    const v2u v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, 0);
    a = v.x;
    b = v.y;
}
template <>
__device__ __forceinline__ void buffer_load_raw2<__half>(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff,
                                                         unsigned& a, unsigned&) {
    a = __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0);
}
template <typename T>
__device__ __forceinline__ float raw_to_f32(unsigned bits);
template <>
__device__ __forceinline__ float raw_to_f32<float>(unsigned bits) { return __builtin_bit_cast(float, bits); }
template <>
__device__ __forceinline__ float raw_to_f32<__half>(unsigned bits) {
    return __half2float(__builtin_bit_cast(__half, (unsigned short)bits));
}
// element `odd` (0: the even column, 1: the odd one) of what buffer_load_raw2 left in (a, b)
template <typename T>
__device__ __forceinline__ float pair_to_f32(unsigned a, unsigned b, int odd);
template <>
__device__ __forceinline__ float pair_to_f32<float>(unsigned a, unsigned b, int odd) {
    return __builtin_bit_cast(float, odd ? b : a);
}
template <>
__device__ __forceinline__ float pair_to_f32<__half>(unsigned a, unsigned, int odd) {
    return raw_to_f32<__half>(odd ? a >> 16 : a & 0xFFFFu);
}

// ---------------------------------------------------------------------------------------------------------------
// tiled kernel (unit stride; stride 2 through the parity form of the layer)
//
// Lane layout.  A wave owns S segments of LW lanes.  A segment is OWS consecutive output columns of R = 7
// consecutive output rows of one image, plus one halo lane on each side; lane t of a segment holds INPUT column
// ix = os + t - pad and, in registers, the R+2 input rows that its R output rows read.  A tap (ky,kx) of a kernel
// multiplies the lane's own column: acc[kx][r] += w * x[r + ky].  The three accumulator sets (one per kx) belong to
// output columns ix+1, ix, ix-1 (+pad-1) and are added across neighbouring lanes once, after the last channel.
// So the inner loop has no cross-lane traffic: 4*R multiply-adds per kept kernel.
//
// LDS layout.  tile[cc][lane][12]: channel-in-chunk, lane, patch row i = r + ky (R+2 = 9 rows padded to 12) so that
// a lane fetches its patch with 128-bit reads (twice the LDS rate of 32-bit reads on this chip); behind the tile,
// per wave and filter slot, the kept kernels ("entries") of that filter in the staged chunk.
//
// Work split.  A workgroup is one slot (the S segments) times FW*NF filters: wave w accumulates NF filters.  All
// waves share the staged activations.  Channels are staged in chunks of CC = CPW*FW = 16*NB (each wave copies CPW
// whole channels and the entries of its own filters); the global loads of chunk k+1 are in flight, in registers,
// while chunk k is being multiplied.
//
// Inner loop.  Threaded code, generated by gen_pattern_leaves.py into pattern_leaves.inc: one 256-byte code section
// per possible pattern; a section multiplies one kept kernel, fetches the next one and jumps straight to ITS
// section.  No branch tree (which costs several hundred clocks per kernel on this chip, against 112 clocks of
// multiply-adds), no divergence: the per-pattern generated access code of section 6.2 of the paper.  The sections
// are inline assembly with fixed registers; the accumulators sit above the register budget that the compiler is
// given for these kernels (amdgpu_num_vgpr).
// ---------------------------------------------------------------------------------------------------------------

#include "pattern_leaves.inc"
static_assert(PCONV_LEAF_STRIDE == kLeafStride, "host packer and generated code disagree on the section stride");

// Division of a 32-bit unsigned by a divisor that is fixed for the launch, as multiply-high and two shifts (Granlund
// and Montgomery's round-up method: exact for every 32-bit dividend).  The hardware has no integer divide, and the
// six divisions of the lane arithmetic below cost a workgroup a few thousand clocks at its start otherwise.
struct FastDiv {
    unsigned m, s1, s2;
};
static FastDiv make_fastdiv(unsigned d) {
    unsigned l = 0;
    while ((1ull << l) < d) ++l;   // ceil(log2 d)
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

struct TiledParams {
    const void* x;
    void* y;
    const DevEntry* ent;
    const uint32_t* eptr;
    const uint32_t* forder;
    const float* bias;
    int N, C, F, H, W, Ho, Wo, pad, relu;
    const uint32_t* perm;    // [groups][perm_stride] channel staged at each position, or null for channel order
    int perm_stride;
    int nbk;                 // eptr entries per filter position (buckets of 16 channels, or chunks of a balanced layout)
    int bpc;                 // eptr entries per chunk of the kernel (NB for buckets, 1 for a balanced layout)
    int LW, S, OWS, NCS, NRB, NSEG;
    int NG;                  // filter groups per slot
    int KS;                  // workgroups that share one output tile, each taking a range of the channel chunks
    float* ws;               // KS > 1: partial sums [KS][tiles][waves][NF][2][64 lanes][4]: a lane's output rows, as held
    unsigned ws_split_bytes; //         size of one split's partial sums
    unsigned* counters;      // KS > 1: [slots * NG] arrivals, zero between launches
    int nblocks;             // NG * slots * KS (the grid is padded to a multiple of 8)
    unsigned long long x_bytes;
    unsigned img_bytes;      // C*H*W*sizeof(T)
    unsigned plane_bytes;    // H*W*sizeof(T)
    FastDiv div_KS, div_NG, div_LW, div_segs_per_img, div_NCS;
    int pair;                // the layer is a parity form and x is the original input (kernels with PAIR staging)
};

// (By value on purpose: __builtin_bit_cast applied directly to an element of an ext_vector_type value reads element 0
// whatever the index, with this compiler.)
// The value the next lower / next higher lane of the wave holds (lane 0 / lane 63: zero): a data-parallel-primitive
// move across the whole wavefront, a plain vector instruction, where a shuffle would go through the LDS crossbar and
// come back a hundred clocks later.  The epilogues hand a lane's outermost partial sums to its neighbours with it.
__device__ __forceinline__ float from_lane_below(float v) {
    constexpr int kWaveShiftRight1 = 0x138;     // DPP control: lane i reads lane i - 1
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kWaveShiftRight1, 0xF, 0xF, true));
}
__device__ __forceinline__ float from_lane_above(float v) {
    constexpr int kWaveShiftLeft1 = 0x130;      // DPP control: lane i reads lane i + 1
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kWaveShiftLeft1, 0xF, 0xF, true));
}
__device__ __forceinline__ float bits_to_f32(unsigned u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ unsigned f32_to_bits(float f) { return __builtin_bit_cast(unsigned, f); }
typedef unsigned v4u __attribute__((ext_vector_type(4)));

constexpr int kR = 7;                       // output rows per lane
constexpr int kPR = 12;                     // patch rows per lane in LDS (R + 2, padded to a multiple of four)
constexpr int kChBytes = 64 * kPR * 4;      // one channel of one slot in LDS

// Packed weights and pointers never change while a kernel runs: reading them through the constant address space
// makes every such load a scalar load (wave-uniform address, result in scalar registers).
typedef const unsigned __attribute__((address_space(4)))* const_u32_ptr;
__device__ __forceinline__ unsigned scalar_load_u32(const uint32_t* p) {
    return *(const_u32_ptr)(unsigned long long)p;
}

template <int SLOT>
__device__ __forceinline__ void zero_acc() {
    if constexpr (SLOT == 0) asm volatile(PCONV_ACC_ZERO_S0 : : : PCONV_ACC_CLOBBERS_S0);
    else if constexpr (SLOT == 1) asm volatile(PCONV_ACC_ZERO_S1 : : : PCONV_ACC_CLOBBERS_S1);
    else asm volatile(PCONV_ACC_ZERO_S2 : : : PCONV_ACC_CLOBBERS_S2);
}

// An entry on its way from memory to LDS.  A lane holds dwords 2l, 2l+1 of an entry's eight (l = lane % 4); the lane
// with the header (dword 4: channel index in its low byte, pattern code above) turns it into what the entry loop
// uses as it is: the byte offset of the pattern's code section in a table of sections `leaf_stride` apart, and the
// byte offset of the channel in the staged chunk of CC channels of `ch_bytes` each.
template <int CC>
__device__ __forceinline__ uint2 staged_entry(uint2 e, int lane, unsigned leaf_stride, unsigned ch_bytes) {
    if ((lane & 3) == 2) return make_uint2((e.x >> 8) * leaf_stride, (e.x & (unsigned)(CC - 1)) * ch_bytes);
    return e;
}
// What stands behind a filter's last entry of a chunk: a header that leads out of the entry loop.
__device__ __forceinline__ uint2 end_marker(unsigned leaf_stride) { return make_uint2(PCONV_EXIT_CODE * leaf_stride, 0u); }

template <int SLOT>
__device__ __forceinline__ void read_acc(float (&a)[3][kR]) {
#define PCONV_ACC_OUTPUTS                                                                                           \
    "=v"(a[0][0]), "=v"(a[0][1]), "=v"(a[0][2]), "=v"(a[0][3]), "=v"(a[0][4]), "=v"(a[0][5]), "=v"(a[0][6]),        \
        "=v"(a[1][0]), "=v"(a[1][1]), "=v"(a[1][2]), "=v"(a[1][3]), "=v"(a[1][4]), "=v"(a[1][5]), "=v"(a[1][6]),    \
        "=v"(a[2][0]), "=v"(a[2][1]), "=v"(a[2][2]), "=v"(a[2][3]), "=v"(a[2][4]), "=v"(a[2][5]), "=v"(a[2][6])
    if constexpr (SLOT == 0) asm volatile(PCONV_ACC_READ_S0 : PCONV_ACC_OUTPUTS);
    else if constexpr (SLOT == 1) asm volatile(PCONV_ACC_READ_S1 : PCONV_ACC_OUTPUTS);
    else asm volatile(PCONV_ACC_READ_S2 : PCONV_ACC_OUTPUTS);
#undef PCONV_ACC_OUTPUTS
}

// Runs the entries stored in LDS from byte address `entry_addr` on (at least one), up to the end marker behind the
// last one, for the filter in slot SLOT of a kernel with NF slots.  `lane_addr` is the LDS byte address of this
// lane's patch of channel 0 of the chunk.  The entries are in the form staged_entry() gives them.
// ROWS8: the loop variant for layers whose kernels have no tap in their third row (a stride-2 layer over parity
// planes): patch row 8 is not fetched.
template <int NF, int SLOT, bool ROWS8>
__device__ __forceinline__ void run_entries(unsigned lane_addr, unsigned entry_addr) {
#define PCONV_LOOP_ASM(TEXT, NFv, Sv)                                                           \
    asm volatile(TEXT                                                                           \
                 :                                                                              \
                 : [vlane] "v"(lane_addr), [ventry] "v"(entry_addr)                             \
                 : "memory", PCONV_ENTRY_LOOP_CLOBBERS_NF##NFv##_S##Sv)
#define PCONV_LOOP(NFv, Sv)                                                                     \
    do {                                                                                        \
        if constexpr (ROWS8) PCONV_LOOP_ASM(PCONV_ENTRY_LOOP_ROWS8_NF##NFv##_S##Sv, NFv, Sv);   \
        else PCONV_LOOP_ASM(PCONV_ENTRY_LOOP_NF##NFv##_S##Sv, NFv, Sv);                         \
    } while (0)
    if constexpr (NF == 1) { PCONV_LOOP(1, 0); }
    else if constexpr (NF == 2 && SLOT == 0) { PCONV_LOOP(2, 0); }
    else { PCONV_LOOP(2, 1); }
#undef PCONV_LOOP
#undef PCONV_LOOP_ASM
}

// PAIR: a stride-2 layer in its parity form (see derive_for_stride2), staged straight from the original input.  The
// chunk's 32 channels are the four parity planes of 8 input channels; wave w stages the two column-parity planes of
// (input channel w/2, row parity w%2) with one two-element load per row, so no separate pass splits the input and
// the staging needs half the load instructions.  Needs even H and W, 16 waves, two channels per wave, channels in their own order.
template <int NF, int CPW, int NB, bool DB, bool PAIR, typename T>
__device__ __forceinline__ void tiled_body(const TiledParams& p) {
    static_assert(!PAIR || (CPW == 2 && NB == 2 && !DB), "the paired staging is built for 16 waves x 2 channels");
    constexpr int R = kR;
    constexpr int CC = 16 * NB;          // channels per chunk
    constexpr int FW = CC / CPW;         // waves per workgroup
    static_assert(CC % CPW == 0 && (FW == 4 || FW == 8 || FW == 16), "bad tiling");
    static_assert(NF >= 1 && NF <= 2, "one or two filters per wave");
    static_assert(CC == 16 || CC == 32, "the section code masks the channel index to the chunk size");
    // bytes of LDS for the entries of one filter and chunk; the loop reads (and ignores) up to two entries past the last
    constexpr unsigned kEntRegion = (CC + 2) * 32;
    constexpr unsigned kBuffers = DB ? 2 : 1;
    constexpr unsigned kTileBytes = CC * kChBytes;           // one chunk buffer
    constexpr unsigned kEntBase = kBuffers * kTileBytes;     // entries start behind the tile(s)
    constexpr unsigned kEntBytes = FW * NF * kEntRegion;     // entries of one buffer
    // [buffers][CC][64][12] floats, then [buffers][FW][NF][CC+2] entries
    extern __shared__ __align__(16) unsigned char lds[];
    const unsigned lds0 = (unsigned)(unsigned long long)lds; // LDS byte address of the allocation (low 32 bits)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // Consecutive workgroup ids go round-robin over the 8 XCDs; give each XCD a contiguous range of logical ids so
    // that the filter groups of one slot, which read the same activations, share one L2.
    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    // (An empty statement that "uses" the kernel arguments the start-up needs: the compiler then fetches them in
    // one batch, here, instead of three — one ahead of the test below, two on first use — each a round trip to
    // memory that the workgroup sits through before its first load.)
    asm volatile("" : : "s"(p.x), "s"(p.ent), "s"(p.eptr), "s"(p.forder), "s"(p.perm), "s"(p.perm_stride), "s"(p.nbk),
                 "s"(p.x_bytes), "s"(p.img_bytes), "s"(p.plane_bytes), "s"(p.nblocks), "s"(p.NSEG), "s"(p.C), "s"(p.H),
                 "s"(p.W), "s"(p.div_NCS.s2), "s"(p.pair));
    if (logical >= p.nblocks) return;
    const int tile = (int)fastdiv((unsigned)logical, p.div_KS);     // (slot, filter group)
    const int split = logical - tile * p.KS;
    const int slot = (int)fastdiv((unsigned)tile, p.div_NG);
    const int grp = tile - slot * p.NG;

    // lane -> (segment, column)
    const int s_local = (int)fastdiv((unsigned)lane, p.div_LW);
    const int t = lane - s_local * p.LW;
    const int gseg = slot * p.S + s_local;
    const bool active = (s_local < p.S) && (gseg < p.NSEG);
    const int segs_per_img = p.NCS * p.NRB;
    const int n0 = (int)fastdiv((unsigned)(slot * p.S), p.div_segs_per_img);   // image of the slot's first segment (uniform)
    const int gs = active ? gseg : slot * p.S;
    const int n = (int)fastdiv((unsigned)gs, p.div_segs_per_img);
    const int rem = gs - n * segs_per_img;
    const int rb = (int)fastdiv((unsigned)rem, p.div_NCS);
    const int cs = rem - rb * p.NCS;
    const int ox = cs * p.OWS + t - 1;
    const int ix = ox + 1 - p.pad;
    const int r0 = rb * R;

    // Byte offset of the lane's element in each of its R + 2 input rows, or an offset outside the descriptor.
    // PAIR: (iy, ix) index a parity plane; the load reads row 2*iy (+ the wave's row parity) and columns 2*ix,
    // 2*ix+1 of the original image, whose rows are 2*W long.
    unsigned voff[R + 2];
    {
        const bool col_in = active && ix >= 0 && ix < p.W;
        const int iy0 = r0 - p.pad;
        const unsigned row_bytes = (PAIR ? 4u : 1u) * (unsigned)p.W * (unsigned)sizeof(T);
        // (modulo 2^32: for rows above the image the product is negative and the offset is not used)
        const unsigned first = (unsigned)(n - n0) * p.img_bytes +
                               (unsigned)(PAIR ? 4 * iy0 * p.W + 2 * ix : iy0 * p.W + ix) * (unsigned)sizeof(T);
#pragma unroll
        for (int i = 0; i < R + 2; ++i)
            voff[i] = (col_in && (unsigned)(iy0 + i) < (unsigned)p.H) ? first + (unsigned)i * row_bytes : kInvalidOffset;
    }
    const unsigned long long base_off = (unsigned long long)n0 * p.img_bytes;
    const unsigned long long left = p.x_bytes - base_off;
    const __amdgpu_buffer_rsrc_t rsrc =
        make_rsrc(static_cast<const char*>(p.x) + base_off, (uint32_t)(left < 0x7FFFFFFFull ? left : 0x7FFFFFFFull));

    const unsigned lane_addr = lds0 + lane * (kPR * 4);

    const int pos_base = grp * (FW * NF) + wave;   // wave w takes positions pos_base + a*FW in the sorted filter order
    // What the first loads do not need is done behind them, while they are in flight: clearing the accumulators and
    // fetching the wave's filters and their biases (scalar registers, so that the epilogue does not wait for them).
    unsigned filt[NF];
    float filt_bias[NF];
    auto behind_first_loads = [&]() {
        if constexpr (NF > 0) zero_acc<0>();
        if constexpr (NF > 1) zero_acc<1>();
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const int pos = pos_base + a * FW;
            filt[a] = pos < p.F ? scalar_load_u32(p.forder + pos) : 0u;
            filt_bias[a] = (p.bias && pos < p.F)
                               ? __builtin_bit_cast(float, scalar_load_u32(reinterpret_cast<const uint32_t*>(p.bias + filt[a])))
                               : 0.f;
        }
    };
    const int nchunks = p.perm ? p.nbk : (p.C + CC - 1) / CC;
    // this workgroup's range of chunks (all of them unless the channels are split)
    const int k_begin = (int)fastdiv((unsigned)(split * nchunks), p.div_KS);   // split, nchunks < 65536
    const int k_end = (int)fastdiv((unsigned)((split + 1) * nchunks), p.div_KS);

    unsigned pre[CPW][R + 2];    // the wave's share of the next chunk's activations, in flight, as stored
    if constexpr (PAIR && sizeof(T) == 2) {   // a paired fp16 load fills pre[0] only
#pragma unroll
        for (int i = 0; i < R + 2; ++i) pre[1][i] = 0u;
    }
    uint2 epre[NF][NB];          // ... and of the next chunk's entries (lane l holds dwords 2l, 2l+1 of 16 entries)
    unsigned ecnt[NF];           // entries of each of the wave's filters in the chunk that is staged or in flight

    // channel staged at position `pos` of this workgroup's staging order (kNoChannel: nothing to stage there)
    auto channel_at = [&](int pos) -> unsigned {
        if (pos >= nchunks * CC) return kNoChannel;
        if (!p.perm) return pos < p.C ? (unsigned)pos : kNoChannel;
        return scalar_load_u32(p.perm + (size_t)grp * p.perm_stride + pos);
    };
    unsigned staged[CPW];        // channels in flight (kNoChannel: none)
    unsigned efirst[NF];         // first entry of each of the wave's filters in the chunk in flight
    auto fetch_entry_ranges = [&](int k) {
        const int b0 = k * p.bpc, b1 = min(p.nbk, b0 + p.bpc);
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const int pos = pos_base + a * FW;
            efirst[a] = 0u;
            ecnt[a] = 0u;
            if (pos < p.F) {
                efirst[a] = scalar_load_u32(p.eptr + pos * p.nbk + b0);
                ecnt[a] = scalar_load_u32(p.eptr + pos * p.nbk + b1) - efirst[a];
            }
        }
    };
    // The activations of the channels in staged[].  With two filters per wave and one chunk buffer the main loop
    // asks for them between the two filters' kept kernels and not in front of both: the address unit of the CU accepts
    // one wave's load per 16 clocks, and 16 waves that issue 18 loads each at the start of a multiply phase queue
    // there while nobody multiplies.
    constexpr bool kSplitLoads = NF > 1 && !DB;
    auto issue_row_loads = [&]() {
        if constexpr (PAIR) {
            const unsigned c = staged[0];
            if (c < (unsigned)p.C) {
                const unsigned soff = (c >> 2) * 4u * p.plane_bytes + ((c >> 1) & 1u) * 2u * p.W * (unsigned)sizeof(T);
#pragma unroll
                // kernels of a parity form have taps in their first two rows only: the last patch row is never read
                for (int i = 0; i < R + 1; ++i) buffer_load_raw2<T>(rsrc, voff[i], soff, pre[0][i], pre[1][i]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < CPW; ++j) {
                if (staged[j] < (unsigned)p.C) {
                    const unsigned soff = staged[j] * p.plane_bytes;
#pragma unroll
                    for (int i = 0; i < R + 2; ++i) pre[j][i] = buffer_load_raw<T>(rsrc, voff[i], soff);
                }
            }
        }
    };
    auto issue_loads = [&](int k, bool defer_rows = false) {
        if constexpr (PAIR) {
            // parity-form channel 4*c_in + 2*a at this wave's position of the staging order (+1: the odd columns)
            const unsigned c = channel_at(k * CC + 2 * wave);
            staged[0] = c < (unsigned)p.C ? c : kNoChannel;
            staged[1] = c < (unsigned)p.C ? c + 1 : kNoChannel;
        } else {
            // (what the scalar unit has to fetch first — which channels, where the entries are — is asked for in one
            // go, so that the wave waits for one round trip and not for one per channel and filter)
            unsigned cs[CPW];
            if (p.perm) {       // (k < nchunks: every position of the chunk is inside the group's order)
                const uint32_t* order = p.perm + (size_t)grp * p.perm_stride + k * CC + wave;
#pragma unroll
                for (int j = 0; j < CPW; ++j) cs[j] = scalar_load_u32(order + j * FW);
            } else {
#pragma unroll
                for (int j = 0; j < CPW; ++j) cs[j] = channel_at(k * CC + wave + j * FW);
            }
            fetch_entry_ranges(k);
#pragma unroll
            for (int j = 0; j < CPW; ++j) staged[j] = cs[j];
        }
        if constexpr (PAIR) fetch_entry_ranges(k);
        if (!(kSplitLoads && defer_rows)) issue_row_loads();
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const unsigned cnt = ecnt[a];
            const uint2* src = reinterpret_cast<const uint2*>(p.ent + efirst[a]);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                if ((unsigned)(lane >> 2) + 16u * j < cnt) epre[a][j] = src[lane + 64 * j];
        }
    };
    auto write_lds = [&](int buf) {
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            const int cc = PAIR ? 2 * wave + j : wave + j * FW;
            if (staged[j] < (unsigned)p.C) {
                float* dst = reinterpret_cast<float*>(lds + buf * kTileBytes + cc * kChBytes + lane * (kPR * 4));
                float v[R + 2];
#pragma unroll
                for (int i = 0; i < R + 2; ++i) {
                    if constexpr (PAIR) v[i] = i > R ? 0.f : pair_to_f32<T>(pre[0][i], pre[1][i], j);
                    else v[i] = raw_to_f32<T>(pre[j][i]);
                }
                *reinterpret_cast<float4*>(dst + 0) = make_float4(v[0], v[1], v[2], v[3]);
                *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
                if constexpr (!PAIR) *reinterpret_cast<float4*>(dst + 8) = make_float4(v[8], 0.f, 0.f, 0.f);
            }
        }
        // entries, and the end marker behind the last (at most CC entries; the region has room for CC + 2)
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            uint2* dst = reinterpret_cast<uint2*>(lds + kEntBase + buf * kEntBytes + (wave * NF + a) * kEntRegion);
#pragma unroll
            for (int j = 0; j < NB; ++j)
                if ((unsigned)(lane >> 2) + 16u * j < ecnt[a])
                    dst[lane + 64 * j] = staged_entry<CC>(epre[a][j], lane, PCONV_LEAF_STRIDE, kChBytes);
            if (lane == 0) dst[ecnt[a] * 4u + 2u] = end_marker(PCONV_LEAF_STRIDE);
        }
    };
    auto compute = [&](int buf, const unsigned (&cnt)[NF], bool rows_deferred = false) {
        const unsigned tile_addr = lane_addr + buf * kTileBytes;
        const unsigned ent_addr = lds0 + kEntBase + buf * kEntBytes + wave * NF * kEntRegion;
        if constexpr (NF > 0) { if (cnt[0]) run_entries<NF, 0, PAIR>(tile_addr, ent_addr + 0 * kEntRegion); }
        if constexpr (kSplitLoads) { if (rows_deferred) issue_row_loads(); }   // (uniform)
        if constexpr (NF > 1) { if (cnt[1]) run_entries<NF, 1, PAIR>(tile_addr, ent_addr + 1 * kEntRegion); }
    };

    unsigned cnt_now[NF];
    if constexpr (!DB) {
        issue_loads(k_begin);
        behind_first_loads();
        write_lds(0);
        __syncthreads();
        for (int k = k_begin; k < k_end; ++k) {
            const bool more = k + 1 < k_end;
#pragma unroll
            for (int a = 0; a < NF; ++a) cnt_now[a] = ecnt[a];
            if (more) issue_loads(k + 1, true);
            compute(0, cnt_now, more);
            __syncthreads();           // every wave is done reading chunk k
            if (more) {
                write_lds(0);
                __syncthreads();
            }
        }
    } else {
        // Three chunks are under way at a time: k is multiplied, k+1 is written to the other buffer at the START of
        // the step (its loads were issued a whole step earlier, and that buffer was last read before the previous
        // barrier), and the loads of k+2 are issued right after, so their latency runs beside the multiply-adds.
        unsigned cnt_next[NF];
        issue_loads(k_begin);
        behind_first_loads();
        write_lds(0);
#pragma unroll
        for (int a = 0; a < NF; ++a) cnt_now[a] = ecnt[a];
        if (k_begin + 1 < k_end) issue_loads(k_begin + 1);
        __syncthreads();
        for (int k = k_begin; k < k_end; ++k) {
            const int buf = (k - k_begin) & 1;
            if (k + 1 < k_end) {
                write_lds(buf ^ 1);
#pragma unroll
                for (int a = 0; a < NF; ++a) cnt_next[a] = ecnt[a];
                if (k + 2 < k_end) issue_loads(k + 2);
            }
            compute(buf, cnt_now);
#pragma unroll
            for (int a = 0; a < NF; ++a) cnt_now[a] = cnt_next[a];
            __syncthreads();           // chunk k+1 is complete in LDS, and nobody reads chunk k any more
        }
    }

    // ---- epilogue: add the three accumulator sets across neighbouring lanes, bias, ReLU, store
    T* __restrict__ y = static_cast<T*>(p.y);
    const bool col_ok = active && t >= 1 && t <= p.OWS && ox < p.Wo;
    const size_t plane_out = (size_t)p.Ho * p.Wo;
    auto combine = [&](const float (&acc)[3][R], float (&v)[R]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float from_left = from_lane_below(acc[0][r]);     // lane t-1 holds column ix-1: its kx=0 sum
            const float from_right = from_lane_above(acc[2][r]);  // lane t+1 holds column ix+1: its kx=2 sum
            v[r] = acc[1][r] + from_left + from_right;
        }
    };
    auto store_filter = [&](const float (&v)[R], unsigned f, float b) {
        const size_t ybase = ((size_t)n * p.F + f) * plane_out;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float o = v[r] + b;
            if (p.relu) o = fmaxf(o, 0.f);
            const int oy = r0 + r;
            if (col_ok && oy < p.Ho) y[ybase + (size_t)oy * p.Wo + ox] = from_f32<T>(o);
        }
    };
    float acc[3][R], v[R];
    if (p.KS == 1) {
#define PCONV_FINISH(a)                                                   \
        if (pos_base + a * FW < p.F) {   /* uniform per wave */            \
            read_acc<a>(acc);                                             \
            combine(acc, v);                                              \
            store_filter(v, filt[a], filt_bias[a]);                       \
        }
        if constexpr (NF > 0) { PCONV_FINISH(0) }
        if constexpr (NF > 1) { PCONV_FINISH(1) }
#undef PCONV_FINISH
        return;
    }

    // The channels of this tile are split over KS workgroups.  Each writes its partial sums to the workspace; the one
    // that arrives last adds them up, always in the order of the splits, so the result does not depend on which
    // workgroup that is.
    //
    // Partial sums and the arrival counter are accessed with device-scope atomic (relaxed) stores, loads and adds
    // only: such accesses are performed at the point where all compute units of the device agree, so no cache
    // write-back or invalidation is needed (a device-scope fence here writes back and invalidates the whole L2 and
    // costs more than the split saves).  Order: a wave's stores have been performed when its vmcnt is zero; the
    // barrier puts that before the arrival is counted; the last workgroup's loads are issued after its count returned.
    // The accesses go through buffer descriptors (one per split's partial sums) with the device-scope cache policy.
    // The workspace is laid out like the registers, not like the output: filter slot a of wave w of tile t has 2 KB
    // at (t*FW*NF + w*NF + a)*2048 of the split's part, rows 0..3 of lane l at + 16*l, rows 4..6 and a spare word
    // at + 1024 + 16*l -- every split of a tile has the same lanes on the same outputs, so two 128-bit stores and
    // two 128-bit loads per split move a lane's rows, each instruction covers 1 KB without gaps, and lanes without
    // an output need no special case.
    constexpr int kDeviceScope = 16;   // cache-policy bit "sc1" of gfx942/gfx950 buffer instructions
    auto ws_rsrc = [&](int s) {
        return make_rsrc(reinterpret_cast<const char*>(p.ws) + (size_t)s * p.ws_split_bytes, p.ws_split_bytes);
    };
    auto ws_offset = [&](int a) { return (unsigned)((tile * FW + wave) * NF + a) * 2048u + (unsigned)lane * 16u; };
    const __amdgpu_buffer_rsrc_t mine = ws_rsrc(split);
#define PCONV_PARTIAL(a)                                                                            \
    if (pos_base + a * FW < p.F) {                                                                  \
        read_acc<a>(acc);                                                                           \
        combine(acc, v);                                                                            \
        const v4u lo = {f32_to_bits(v[0]), f32_to_bits(v[1]), f32_to_bits(v[2]), f32_to_bits(v[3])}; \
        const v4u hi = {f32_to_bits(v[4]), f32_to_bits(v[5]), f32_to_bits(v[6]), 0u};               \
        __builtin_amdgcn_raw_buffer_store_b128(lo, mine, (int)ws_offset(a), 0, kDeviceScope);       \
        __builtin_amdgcn_raw_buffer_store_b128(hi, mine, (int)ws_offset(a) + 1024, 0, kDeviceScope);  \
    }
    if constexpr (NF > 0) { PCONV_PARTIAL(0) }
    if constexpr (NF > 1) { PCONV_PARTIAL(1) }
#undef PCONV_PARTIAL
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                 // (also: nobody reads the staged chunk any more, LDS can carry the flag)
    // (the flag goes through the first word of LDS with plain LDS instructions: a volatile access through the generic
    // pointer becomes a flat store and load, several hundred clocks slower, on a path every workgroup waits on)
    if (threadIdx.x == 0) {
        const unsigned arrived = __hip_atomic_fetch_add(p.counters + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = arrived == (unsigned)p.KS - 1u;
        // everybody has arrived: leave the counter ready for the next launch
        if (last) __hip_atomic_store(p.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("ds_write_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : : "v"(lds0), "v"(last ? 1u : 0u) : "memory");
    }
    __syncthreads();
    unsigned last_arrival;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(last_arrival) : "v"(lds0) : "memory");
    if (__builtin_amdgcn_readfirstlane(last_arrival) == 0u) return;   // (the same in every lane)
    // partial sums of up to four splits are requested together, then added in split order
#define PCONV_REDUCE(a)                                                                             \
    if (pos_base + a * FW < p.F) {                                                                  \
        static_assert(R == 7, "two 128-bit words per lane and filter");                             \
        read_acc<a>(acc);                                                                           \
        combine(acc, v);                                                                            \
        float sum[R];                                                                               \
        _Pragma("unroll") for (int r = 0; r < R; ++r) sum[r] = 0.f;                                 \
        for (int s0 = 0; s0 < p.KS; s0 += 4) {                                                      \
            float part[4][R];                                                                       \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                         \
                const int s = s0 + j;                                                               \
                if (s < p.KS && s != split) {   /* uniform: only the splits that exist, not this one's own */ \
                    const __amdgpu_buffer_rsrc_t theirs = ws_rsrc(s);                               \
                    const v4u lo = __builtin_amdgcn_raw_buffer_load_b128(theirs, (int)ws_offset(a), 0, kDeviceScope); \
                    const v4u hi = __builtin_amdgcn_raw_buffer_load_b128(theirs, (int)ws_offset(a) + 1024, 0, kDeviceScope); \
                    part[j][0] = bits_to_f32(lo[0]); part[j][1] = bits_to_f32(lo[1]);               \
                    part[j][2] = bits_to_f32(lo[2]); part[j][3] = bits_to_f32(lo[3]);               \
                    part[j][4] = bits_to_f32(hi[0]); part[j][5] = bits_to_f32(hi[1]);               \
                    part[j][6] = bits_to_f32(hi[2]);                                                \
                } else {                                                                            \
                    _Pragma("unroll") for (int r = 0; r < R; ++r) part[j][r] = 0.f;                 \
                }                                                                                   \
            }                                                                                       \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                         \
                const int s = s0 + j;                                                               \
                if (s < p.KS) {                                                                     \
                    _Pragma("unroll") for (int r = 0; r < R; ++r) {                                 \
                        const float q = s == split ? v[r] : part[j][r];                             \
                        sum[r] = s == 0 ? q : sum[r] + q;                                           \
                    }                                                                               \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
        store_filter(sum, filt[a], filt_bias[a]);                                                   \
    }
    if constexpr (NF > 0) { PCONV_REDUCE(0) }
    if constexpr (NF > 1) { PCONV_REDUCE(1) }
#undef PCONV_REDUCE
}

// The compiler may allocate 2*n vector registers under amdgpu_num_vgpr(n) on this target; the accumulators of the
// pattern sections sit above that: 21 registers per filter slot, ending at v127.
template <int CPW, int NB, bool DB, bool PAIR, typename T>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_num_vgpr(53))) void tiled_kernel_nf1(const TiledParams p) {
    static_assert(PCONV_ACC_BASE_S0 >= 2 * 53, "accumulators overlap the compiler's registers");
    tiled_body<1, CPW, NB, DB, PAIR, T>(p);
}
template <int CPW, int NB, bool DB, bool PAIR, typename T>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_num_vgpr(43))) void tiled_kernel_nf2(const TiledParams p) {
    static_assert(PCONV_ACC_BASE_S1 >= 2 * 43, "accumulators overlap the compiler's registers");
    tiled_body<2, CPW, NB, DB, PAIR, T>(p);
}

// ---------------------------------------------------------------------------------------------------------------
// quad kernel (unit stride, W a multiple of four)
//
// Lane layout.  A lane holds FOUR neighbouring input columns (a "quad") of the six input rows that four output rows
// read, and a wave holds BL = 64 / (W/4) row blocks of W/4 quads each: whole image rows, so there are no halo lanes
// and the zero padding left and right of the image needs no data at all.  A tap (ky,kx) of a kept kernel on the
// lane's column c (0..3) belongs to output column c + pad - kx of the quad, which is accumulator column
// j = c + 2 - kx of six (see gen_pattern_leaves.py); columns 0 and 5 are handed to the neighbouring lanes once, after
// the last channel.  64 multiply-adds per kept kernel and jump.
//
// LDS layout.  tile[cc][6 rows][64 lanes][4 columns]: every patch row is one 128-bit read with an immediate offset,
// neighbouring lanes read neighbouring 16 bytes.  Staging writes the same shape: wave w copies channel w of the
// 16-channel chunk, each lane its own six rows with 128-bit loads (64-bit for fp16 storage) -- a third of the load
// instructions per element of the one-column kernel, whose batch-1 chunks are bound by load issue.
//
// Work split.  Workgroup = one slot (the wave shape above) x 16 waves x NF filters; chunks of 16 channels in their
// own or in the workgroup's balanced order, one chunk buffer, two barriers per chunk.  Channels can be split over
// several workgroups per tile as in the one-column kernel; meant for layers with many tiles, where that is not needed.
// ---------------------------------------------------------------------------------------------------------------

struct QuadParams {
    const void* x;
    void* y;
    const DevEntry* ent;
    const uint32_t* eptr;
    const uint32_t* forder;
    const float* bias;
    int N, C, F, H, W, Ho, Wo, pad, relu;
    int nbk;                 // eptr entries per filter position: chunks of 16 channels
    const uint32_t* perm;    // [groups][perm_stride] channel staged at each position, or null for channel order
    int perm_stride;
    int QW, BL, NRB;         // quads per image row, row blocks per wave, row blocks per image
    int NBLK;                // N * NRB
    int NG;                  // filter groups per slot
    int KS;                  // workgroups per output tile (each takes a range of the chunks)
    int vec;                 // a lane's four outputs of a row are in range together and 16-byte aligned (pad 1, aligned y)
    int nblocks;             // NG * slots * KS (the grid is padded to a multiple of 8)
    float* ws;               // KS > 1: partial sums [KS][tiles][16 waves][NF][4 rows][64 lanes][4]: a lane's outputs, as held
    unsigned ws_split_bytes; //         size of one split's partial sums
    unsigned* counters;      // KS > 1: one arrival counter per tile, zero between launches
    unsigned long long x_bytes;
    unsigned img_bytes, plane_bytes;
    unsigned ent_bytes;      // size of ent[] (below 2^31: the kernel reads it through a buffer descriptor)
    int walkers;             // quad_walk_kernel: workgroups per filter group; one walks slots w, w + walkers, ...
    int slots;               //                   slots in all
    unsigned out_img_bytes;  //                   F*Ho*Wo*sizeof(T)
    unsigned long long y_bytes;
    FastDiv div_NG, div_KS, div_QW, div_NRB;
};

// four neighbouring elements as they are stored
template <typename T>
struct RawQuad;
template <>
struct RawQuad<float> {
    unsigned e0, e1, e2, e3;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        const v4u v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0);
        e0 = v[0];
        e1 = v[1];
        e2 = v[2];
        e3 = v[3];
    }
    __device__ __forceinline__ float4 widen() const {
        return make_float4(__builtin_bit_cast(float, e0), __builtin_bit_cast(float, e1), __builtin_bit_cast(float, e2),
                           __builtin_bit_cast(float, e3));
    }
};
template <>
struct RawQuad<__half> {
    unsigned lo, hi;   // elements 0, 1 and 2, 3
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
        typedef unsigned v2u __attribute__((ext_vector_type(2)));
        const v2u v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, 0);
        lo = v[0];
        hi = v[1];
    }
    __device__ __forceinline__ float4 widen() const {
        return make_float4(raw_to_f32<__half>(lo & 0xFFFFu), raw_to_f32<__half>(lo >> 16),
                           raw_to_f32<__half>(hi & 0xFFFFu), raw_to_f32<__half>(hi >> 16));
    }
};

template <int SLOT>
__device__ __forceinline__ void quad_zero_acc() {
    if constexpr (SLOT == 0) asm volatile(PCONV_QUAD_ACC_ZERO_S0 : : : PCONV_QUAD_ACC_CLOBBERS_S0);
    else asm volatile(PCONV_QUAD_ACC_ZERO_S1 : : : PCONV_QUAD_ACC_CLOBBERS_S1);
}

// Output row ROW of the six accumulator columns of filter slot SLOT.
template <int SLOT, int ROW>
__device__ __forceinline__ void quad_read_acc_row(float (&a)[6]) {
#define PCONV_QREAD(Sv, Rv)                                                                            \
    if constexpr (SLOT == Sv && ROW == Rv)                                                             \
        asm volatile(PCONV_QUAD_ACC_READ_ROW_S##Sv##_R##Rv                                             \
                     : "=v"(a[0]), "=v"(a[1]), "=v"(a[2]), "=v"(a[3]), "=v"(a[4]), "=v"(a[5]));
    PCONV_QREAD(0, 0) PCONV_QREAD(0, 1) PCONV_QREAD(0, 2) PCONV_QREAD(0, 3)
    PCONV_QREAD(1, 0) PCONV_QREAD(1, 1) PCONV_QREAD(1, 2) PCONV_QREAD(1, 3)
#undef PCONV_QREAD
}

template <int NF, int SLOT, int CC>
__device__ __forceinline__ void quad_run_entries(unsigned lane_addr, unsigned entry_addr, unsigned count) {
    const unsigned cnt = __builtin_amdgcn_readfirstlane(count);
#define PCONV_QLOOP(NFv, Sv)                                                                    \
    asm volatile(PCONV_QUAD_ENTRY_LOOP_NF##NFv##_S##Sv                                          \
                 :                                                                              \
                 : [vlane] "v"(lane_addr), [ventry] "v"(entry_addr), [cnt] "s"(cnt), [ccmask] "n"(CC - 1) \
                 : "memory", PCONV_QUAD_ENTRY_LOOP_CLOBBERS_NF##NFv##_S##Sv)
    if constexpr (NF == 1) { PCONV_QLOOP(1, 0); }
    else if constexpr (SLOT == 0) { PCONV_QLOOP(2, 0); }
    else { PCONV_QLOOP(2, 1); }
#undef PCONV_QLOOP
}

// FW waves, each with NF filters and one channel of every chunk of CC = FW channels.
template <int NF, int FW, typename T>
__device__ __forceinline__ void quad_body(const QuadParams& p) {
    constexpr int R = PCONV_QUAD_ROWS;
    constexpr int CC = FW;
    constexpr unsigned kChB = PCONV_QUAD_CH_BYTES;
    constexpr unsigned kRowB = 64 * 16;
    static_assert(kChB == (R + 2) * kRowB, "generated code and kernel disagree on the tile shape");
    constexpr unsigned kEntRegion = (CC + 2) * 32;
    constexpr unsigned kEntBase = CC * kChB;
    extern __shared__ __align__(16) unsigned char lds[];     // [CC][R+2][64] float4, then [FW][NF][CC+2] entries
    const unsigned lds0 = (unsigned)(unsigned long long)lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const int per_xcd = gridDim.x >> 3;   // see tiled_body: the filter groups of one slot share one XCD's L2
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    // (see tiled_body: the kernel arguments of the start-up in one batch)
    asm volatile("" : : "s"(p.x), "s"(p.ent), "s"(p.eptr), "s"(p.perm), "s"(p.perm_stride), "s"(p.nbk), "s"(p.x_bytes),
                 "s"(p.img_bytes), "s"(p.plane_bytes), "s"(p.ent_bytes), "s"(p.nblocks), "s"(p.NBLK), "s"(p.C), "s"(p.H),
                 "s"(p.W), "s"(p.div_NRB.s2));
    if (logical >= p.nblocks) return;
    const int tile = (int)fastdiv((unsigned)logical, p.div_KS);     // (slot, filter group)
    const int split = logical - tile * p.KS;
    const int slot = (int)fastdiv((unsigned)tile, p.div_NG);
    const int grp = tile - slot * p.NG;

    // lane -> (row block, quad), image and first output row.  Worked out twice, before the channel loop and again
    // behind it: a handful of instructions, instead of five registers held across the loop.
    const int g0 = slot * p.BL;                         // first row block of the slot (uniform)
    const int n0 = (int)fastdiv((unsigned)g0, p.div_NRB);
    struct LanePlace { int q, n, oy0; bool active; };
    auto place_of = [&](int ln) {
        LanePlace r;
        const int b = (int)fastdiv((unsigned)ln, p.div_QW);
        r.q = ln - b * p.QW;
        r.active = b < p.BL && g0 + b < p.NBLK;
        const int g = r.active ? g0 + b : g0;
        r.n = (int)fastdiv((unsigned)g, p.div_NRB);
        r.oy0 = (g - r.n * p.NRB) * R;
        return r;
    };
    const LanePlace early = place_of(lane);

    unsigned voff[R + 2];
#pragma unroll
    for (int i = 0; i < R + 2; ++i) {
        const int iy = early.oy0 - p.pad + i;
        const bool ok = early.active && iy >= 0 && iy < p.H;
        voff[i] = ok ? (unsigned)(early.n - n0) * p.img_bytes + (unsigned)(iy * p.W + 4 * early.q) * (unsigned)sizeof(T)
                     : kInvalidOffset;
    }
    const unsigned long long base_off = (unsigned long long)n0 * p.img_bytes;
    const unsigned long long left = p.x_bytes - base_off;
    const __amdgpu_buffer_rsrc_t rsrc =
        make_rsrc(static_cast<const char*>(p.x) + base_off, (uint32_t)(left < 0x7FFFFFFFull ? left : 0x7FFFFFFFull));

    const unsigned lane_addr = lds0 + lane * 16;
    if constexpr (NF > 0) quad_zero_acc<0>();
    if constexpr (NF > 1) quad_zero_acc<1>();

    const int pos_base = grp * (FW * NF) + wave;
    const int nchunks = p.nbk;
    // this workgroup's range of chunks (all of them unless the channels are split)
    const int k_begin = (int)fastdiv((unsigned)(split * nchunks), p.div_KS);   // split, nchunks < 65536
    const int k_end = (int)fastdiv((unsigned)((split + 1) * nchunks), p.div_KS);

    // The loads of a chunk and their use below are unconditional (lanes and waves with nothing to fetch use an offset
    // outside the descriptor and get zeros): with loads or uses under branches the compiler has to assume that a
    // load of the previous chunk may still be pending when the next ones are issued, and waits for all of them
    // there, in front of the multiply-adds that are meant to cover their latency.
    RawQuad<T> pre[R + 2];       // the wave's channel of the next chunk, in flight
    uint2 epre[NF];              // ... and the wave's entries of the next chunk (lane l: dwords 2l, 2l+1)
    unsigned ecnt[NF];
    const __amdgpu_buffer_rsrc_t ent_rsrc = make_rsrc(p.ent, p.ent_bytes);
    // Where a chunk's entries and channel are (scalar loads) is fetched one chunk ahead of the vector loads that need
    // it: issued back to back, the two dependent rounds of scalar loads cost every wave about 1500 clocks per chunk
    // in which the multiply-add units have nothing to do.
    unsigned meta_e0[NF], meta_e1[NF], meta_c;
    auto fetch_meta = [&](int k) {
        const bool chunk = k < k_end;
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const int pos = pos_base + a * FW;
            meta_e0[a] = meta_e1[a] = 0;
            if (chunk && pos < p.F) {
                meta_e0[a] = scalar_load_u32(p.eptr + pos * p.nbk + k);
                meta_e1[a] = scalar_load_u32(p.eptr + pos * p.nbk + k + 1);
            }
        }
        // the channel at this wave's position of the workgroup's staging order (kNoChannel: nothing to stage there)
        meta_c = !chunk ? kNoChannel
                 : p.perm ? scalar_load_u32(p.perm + (size_t)grp * p.perm_stride + k * CC + wave)
                          : (unsigned)(k * CC + wave);
    };
    // The loads of a chunk, in two parts: the address unit of the CU accepts one wave's load per 16 clocks, so 16 waves
    // that issue all their loads at the start of a multiply phase queue for 2 k clocks before the last of them
    // multiplies.  With two filters per wave the patch rows are requested between the two filters' entries instead,
    // when the waves are out of step and the unit is idle (the entries stay in front: moving them too costs 2 %).
    constexpr bool kSplit = NF > 1;
    unsigned load_soff = 0u;
    bool load_staged = false;
    auto issue_row_loads = [&]() {
#pragma unroll
        for (int i = 0; i < R + 2; ++i) pre[i].load(rsrc, load_staged ? voff[i] : kInvalidOffset, load_soff);
    };
    auto issue_loads_first = [&]() {     // the chunk of the last fetch_meta
        unsigned e0[NF];
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            e0[a] = meta_e0[a];
            ecnt[a] = meta_e1[a] - e0[a];
        }
        const unsigned c = meta_c;
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const unsigned eoff = (unsigned)(lane >> 2) < ecnt[a] ? e0[a] * 32u + (unsigned)lane * 8u : kInvalidOffset;
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            const v2u e = __builtin_amdgcn_raw_buffer_load_b64(ent_rsrc, (int)eoff, 0, 0);
            epre[a] = make_uint2(e[0], e[1]);
        }
        load_staged = c < (unsigned)p.C;
        load_soff = load_staged ? c * p.plane_bytes : 0u;
        if constexpr (!kSplit) issue_row_loads();
    };
    auto issue_loads_rest = [&]() {      // (nothing fetches metadata between the two parts)
        if constexpr (kSplit) issue_row_loads();
    };
    auto issue_loads = [&]() {
        issue_loads_first();
        issue_loads_rest();
    };
    auto write_lds = [&]() {
        float4* dst = reinterpret_cast<float4*>(lds + wave * kChB + lane * 16);
#pragma unroll
        for (int i = 0; i < R + 2; ++i) dst[i * (kRowB / 16)] = pre[i].widen();
        // 64 lanes x 8 bytes: 16 entries, of which the chunk's first ecnt are real; the region holds CC + 2
        static_assert(kEntRegion >= 64 * 8, "entry region smaller than one wave's write");
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            uint2* e = reinterpret_cast<uint2*>(lds + kEntBase + (wave * NF + a) * kEntRegion);
            e[lane] = epre[a];
        }
    };

    unsigned cnt_now[NF];
    fetch_meta(k_begin);
    issue_loads();
    fetch_meta(k_begin + 1);
    write_lds();
    __syncthreads();
    for (int k = k_begin; k < k_end; ++k) {
        const bool more = k + 1 < k_end;
#pragma unroll
        for (int a = 0; a < NF; ++a) cnt_now[a] = ecnt[a];
        if (more) issue_loads_first();   // chunk k + 1
        const unsigned ent_addr = lds0 + kEntBase + wave * NF * kEntRegion;
        if constexpr (NF > 0) { if (cnt_now[0]) quad_run_entries<NF, 0, CC>(lane_addr, ent_addr, cnt_now[0]); }
        if (more) issue_loads_rest();
        if constexpr (NF > 1) { if (cnt_now[1]) quad_run_entries<NF, 1, CC>(lane_addr, ent_addr + kEntRegion, cnt_now[1]); }
        fetch_meta(k + 2);               // lands while the workgroup meets at the barriers
        __syncthreads();
        if (more) {
            write_lds();
            __syncthreads();
        }
    }

    // ---- epilogue: accumulator columns 0 and 5 go to the neighbouring quads; bias, ReLU, store
    T* __restrict__ y = static_cast<T*>(p.y);
    int lane_again = lane;
    asm volatile("" : "+v"(lane_again));               // keeps the compiler from carrying the first result over
    const LanePlace late = place_of(lane_again);
    const int q = late.q, n = late.n, oy0 = late.oy0;
    const bool active = late.active;
    const bool has_left = q > 0, has_right = q + 1 < p.QW;
    const int o0 = 4 * q + p.pad - 1;                  // output column of accumulator column 1
    // the four sums of output row `row` of one filter slot
    auto row_sums = [&](auto slot_c, auto row_c, float (&v)[4]) {
        float a[6];
        quad_read_acc_row<decltype(slot_c)::value, decltype(row_c)::value>(a);
        const float from_left = from_lane_below(a[5]);     // the left quad's column 5 is this quad's column 1
        const float from_right = from_lane_above(a[0]);  // the right quad's column 0 is this quad's column 4
        v[0] = a[1] + (has_left ? from_left : 0.f);
        v[1] = a[2];
        v[2] = a[3];
        v[3] = a[4] + (has_right ? from_right : 0.f);
    };
    auto store_row = [&](const float (&v)[4], unsigned f, float bias, int r) {
        const int oy = oy0 + r;
        const size_t at = (((size_t)n * p.F + f) * p.Ho + oy) * (size_t)p.Wo;
        float o[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            o[m] = v[m] + bias;
            if (p.relu) o[m] = fmaxf(o[m], 0.f);
        }
        if (p.vec) {             // uniform: one 128-bit (fp16: 64-bit) store per lane and row
            if (active && oy < p.Ho) {
                if constexpr (sizeof(T) == 4) {
                    *reinterpret_cast<float4*>(y + at + o0) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
                    const unsigned lo = (unsigned)__half_as_ushort(__float2half_rn(o[0])) |
                                        ((unsigned)__half_as_ushort(__float2half_rn(o[1])) << 16);
                    const unsigned hi = (unsigned)__half_as_ushort(__float2half_rn(o[2])) |
                                        ((unsigned)__half_as_ushort(__float2half_rn(o[3])) << 16);
                    *reinterpret_cast<uint2*>(y + at + o0) = make_uint2(lo, hi);
                }
            }
            return;
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int ox = o0 + m;
            if (active && oy < p.Ho && ox >= 0 && ox < p.Wo) y[at + ox] = from_f32<T>(o[m]);
        }
    };
    unsigned filt[NF];
    float filt_bias[NF];
#pragma unroll
    for (int a = 0; a < NF; ++a) {
        const int pos = pos_base + a * FW;
        filt[a] = pos < p.F ? scalar_load_u32(p.forder + pos) : 0u;
        filt_bias[a] = (p.bias && pos < p.F)
                           ? __builtin_bit_cast(float, scalar_load_u32(reinterpret_cast<const uint32_t*>(p.bias + filt[a])))
                           : 0.f;
    }
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;
#define PCONV_QROWS(BODY) { BODY(I0{}, 0) BODY(I1{}, 1) BODY(I2{}, 2) BODY(I3{}, 3) }
    float v[4];
    if (p.KS == 1) {
#define PCONV_QSTORE(rc, r) row_sums(slot_c, rc, v); store_row(v, filt[a], filt_bias[a], r);
#define PCONV_QFINISH(Sv)                                              \
        if (pos_base + Sv * FW < p.F) {   /* uniform per wave */        \
            constexpr int a = Sv;                                      \
            const std::integral_constant<int, Sv> slot_c{};            \
            PCONV_QROWS(PCONV_QSTORE)                                  \
        }
        if constexpr (NF > 0) { PCONV_QFINISH(0) }
        if constexpr (NF > 1) { PCONV_QFINISH(1) }
#undef PCONV_QFINISH
#undef PCONV_QSTORE
        return;
    }

    // The channels of this tile are split over KS workgroups: partial sums go to the workspace, the workgroup that
    // arrives last adds them up in the order of the splits (see tiled_body for the memory-ordering argument; the
    // accesses here are the same kind: device-scope buffer stores and loads, one relaxed device-scope atomic).
    // The workspace is laid out like the registers: filter slot a of wave w of tile t has 4 KB at
    // (t*FW*NF + w*NF + a)*4096 of the split's part, output row r of lane l at + 1024*r + 16*l (one 128-bit access
    // per lane and row, 1 KB without gaps per instruction).
    constexpr int kDeviceScope = 16;   // cache-policy bit "sc1" of gfx942/gfx950 buffer instructions
    auto ws_rsrc = [&](int s) {
        return make_rsrc(reinterpret_cast<const char*>(p.ws) + (size_t)s * p.ws_split_bytes, p.ws_split_bytes);
    };
    auto ws_offset = [&](int a, int r) {
        return (unsigned)((tile * FW + wave) * NF + a) * 4096u + 1024u * r + (unsigned)lane * 16u;
    };
    const __amdgpu_buffer_rsrc_t mine = ws_rsrc(split);
#define PCONV_QPART(rc, r)                                                                          \
    {                                                                                               \
        row_sums(slot_c, rc, v);                                                                    \
        const v4u q4 = {f32_to_bits(v[0]), f32_to_bits(v[1]), f32_to_bits(v[2]), f32_to_bits(v[3])}; \
        __builtin_amdgcn_raw_buffer_store_b128(q4, mine, (int)ws_offset(a, r), 0, kDeviceScope);    \
    }
#define PCONV_QPARTIAL(Sv)                                             \
    if (pos_base + Sv * FW < p.F) {                                    \
        constexpr int a = Sv;                                          \
        const std::integral_constant<int, Sv> slot_c{};                \
        PCONV_QROWS(PCONV_QPART)                                       \
    }
    if constexpr (NF > 0) { PCONV_QPARTIAL(0) }
    if constexpr (NF > 1) { PCONV_QPARTIAL(1) }
#undef PCONV_QPARTIAL
#undef PCONV_QPART
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                 // (also: nobody reads the staged chunk any more, LDS can carry the flag)
    // (the flag goes through the first word of LDS with plain LDS instructions: a volatile access through the generic
    // pointer becomes a flat store and load, several hundred clocks slower, on a path every workgroup waits on)
    if (threadIdx.x == 0) {
        const unsigned arrived = __hip_atomic_fetch_add(p.counters + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = arrived == (unsigned)p.KS - 1u;
        // everybody has arrived: leave the counter ready for the next launch
        if (last) __hip_atomic_store(p.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("ds_write_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : : "v"(lds0), "v"(last ? 1u : 0u) : "memory");
    }
    __syncthreads();
    unsigned last_arrival;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(last_arrival) : "v"(lds0) : "memory");
    if (__builtin_amdgcn_readfirstlane(last_arrival) == 0u) return;   // (the same in every lane)
    // partial sums of up to four splits are requested together (this workgroup's own among them: its stores have
    // been performed), then added in split order
#define PCONV_QRED(rc, r)                                                                           \
    {                                                                                               \
        float sum[4] = {0.f, 0.f, 0.f, 0.f};                                                        \
        for (int s0 = 0; s0 < p.KS; s0 += 4) {                                                      \
            float part[4][4];                                                                       \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                         \
                if (s0 + j < p.KS) {            /* uniform: only the splits that exist */           \
                    const v4u q4 = __builtin_amdgcn_raw_buffer_load_b128(ws_rsrc(s0 + j), (int)ws_offset(a, r), 0, kDeviceScope); \
                    part[j][0] = bits_to_f32(q4[0]);                                                \
                    part[j][1] = bits_to_f32(q4[1]);                                                \
                    part[j][2] = bits_to_f32(q4[2]);                                                \
                    part[j][3] = bits_to_f32(q4[3]);                                                \
                } else {                                                                            \
                    part[j][0] = part[j][1] = part[j][2] = part[j][3] = 0.f;                        \
                }                                                                                   \
            }                                                                                       \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                         \
                const int s = s0 + j;                                                               \
                if (s < p.KS) {                                                                     \
                    _Pragma("unroll") for (int m = 0; m < 4; ++m)                                   \
                        sum[m] = s == 0 ? part[j][m] : sum[m] + part[j][m];                         \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
        store_row(sum, filt[a], filt_bias[a], r);                                                   \
    }
#define PCONV_QREDUCE(Sv)                                              \
    if (pos_base + Sv * FW < p.F) {                                    \
        constexpr int a = Sv;                                          \
        PCONV_QROWS(PCONV_QRED)                                        \
    }
    if constexpr (NF > 0) { PCONV_QREDUCE(0) }
    if constexpr (NF > 1) { PCONV_QREDUCE(1) }
#undef PCONV_QREDUCE
#undef PCONV_QRED
#undef PCONV_QROWS
}

// The quad kernel for layers whose input channels fit one chunk (a network's first layer) and that have many slots:
// an ordinary workgroup would load three channels, do three kept kernels per wave and store, one dependent step after
// the other and all of it start-up.  Here a workgroup keeps its 16 filters (one per wave) and their entries in LDS
// and walks over the slots w, w + walkers, ...; the loads of the next slot are in flight while the current one is
// multiplied and stored.  Loads and stores are unconditional (lanes with nothing to do use an offset outside the
// descriptor): the wait for a slot's loads must not include the stores issued behind them, and the compiler can
// only count those when no branch surrounds them.  Needs pad 1 and a 16-byte aligned y (one store per lane and row).
template <int NF, typename T>
__device__ __forceinline__ void quad_walk_body(const QuadParams& p) {
    constexpr int R = PCONV_QUAD_ROWS, FW = 16, CC = 16;
    constexpr unsigned kChB = PCONV_QUAD_CH_BYTES;
    constexpr unsigned kRowB = 64 * 16;
    constexpr unsigned kEntRegion = (CC + 2) * 32;
    constexpr unsigned kEntBase = CC * kChB;
    extern __shared__ __align__(16) unsigned char lds[];     // as in quad_body
    const unsigned lds0 = (unsigned)(unsigned long long)lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const int per_xcd = gridDim.x >> 3;   // the filter groups of one walker read the same slots: same XCD, same L2
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= p.nblocks) return;
    const int walker = (int)fastdiv((unsigned)logical, p.div_NG);
    const int grp = logical - walker * p.NG;

    struct LanePlace { int q, n, n0, oy0; bool active; };
    auto place_of = [&](int ln, int slot) {
        LanePlace r;
        const int g0 = slot * p.BL;                     // first row block of the slot (uniform)
        r.n0 = (int)fastdiv((unsigned)g0, p.div_NRB);
        const int b = (int)fastdiv((unsigned)ln, p.div_QW);
        r.q = ln - b * p.QW;
        r.active = b < p.BL && g0 + b < p.NBLK;
        const int g = r.active ? g0 + b : g0;
        r.n = (int)fastdiv((unsigned)g, p.div_NRB);
        r.oy0 = (g - r.n * p.NRB) * R;
        return r;
    };

    // the wave's filters, their entries (staged once) and its channel of the one chunk
    const int pos_base = grp * (FW * NF) + wave;
    bool has_filter[NF];
    unsigned filt[NF], cnt[NF];
    float filt_bias[NF];
#pragma unroll
    for (int a = 0; a < NF; ++a) {
        const int pos = pos_base + a * FW;
        has_filter[a] = pos < p.F;
        unsigned e0 = 0, e1 = 0;
        if (has_filter[a]) {
            e0 = scalar_load_u32(p.eptr + pos * p.nbk);
            e1 = scalar_load_u32(p.eptr + pos * p.nbk + 1);
        }
        filt[a] = has_filter[a] ? scalar_load_u32(p.forder + pos) : 0u;
        filt_bias[a] = (p.bias && has_filter[a])
                           ? __builtin_bit_cast(float, scalar_load_u32(reinterpret_cast<const uint32_t*>(p.bias + filt[a])))
                           : 0.f;
        cnt[a] = __builtin_amdgcn_readfirstlane(e1 - e0);
        const __amdgpu_buffer_rsrc_t ent_rsrc = make_rsrc(p.ent, p.ent_bytes);
        const unsigned eoff = (unsigned)(lane >> 2) < cnt[a] ? e0 * 32u + (unsigned)lane * 8u : kInvalidOffset;
        typedef unsigned v2u __attribute__((ext_vector_type(2)));
        const v2u e = __builtin_amdgcn_raw_buffer_load_b64(ent_rsrc, (int)eoff, 0, 0);
        static_assert(kEntRegion >= 64 * 8, "entry region smaller than one wave's write");
        reinterpret_cast<uint2*>(lds + kEntBase + (wave * NF + a) * kEntRegion)[lane] = make_uint2(e[0], e[1]);
    }
    const unsigned c = p.perm ? scalar_load_u32(p.perm + (size_t)grp * p.perm_stride + wave) : (unsigned)wave;
    const bool staged = c < (unsigned)p.C;
    const unsigned soff = staged ? c * p.plane_bytes : 0u;
    const unsigned lane_addr = lds0 + lane * 16;
    const unsigned ent_addr = lds0 + kEntBase + wave * NF * kEntRegion;

    RawQuad<T> pre[R + 2];
    // (`wanted` and `staged` are the same for the whole wave; they reach the offsets through a vector register the
    // compiler knows nothing about, or it splits the six loads over branches, with a wait in front of each.)
    auto issue_loads = [&](int slot, bool wanted) {
        int fetch = (wanted && staged) ? 1 : 0;
        asm volatile("" : "+v"(fetch));
        const LanePlace pl = place_of(lane, slot);
        const unsigned long long base_off = (unsigned long long)pl.n0 * p.img_bytes;
        const unsigned long long left = p.x_bytes - base_off;
        const __amdgpu_buffer_rsrc_t rsrc =
            make_rsrc(static_cast<const char*>(p.x) + base_off, (uint32_t)(left < 0x7FFFFFFFull ? left : 0x7FFFFFFFull));
#pragma unroll
        for (int i = 0; i < R + 2; ++i) {
            const int iy = pl.oy0 - p.pad + i;
            const bool ok = fetch != 0 && pl.active && iy >= 0 && iy < p.H;
            const unsigned voff = ok ? (unsigned)(pl.n - pl.n0) * p.img_bytes +
                                           (unsigned)(iy * p.W + 4 * pl.q) * (unsigned)sizeof(T)
                                     : kInvalidOffset;
            pre[i].load(rsrc, voff, soff);
        }
    };

    int slot = walker;                 // walker < walkers <= slots
    issue_loads(slot, true);
    {
        // Stores that store nothing (their offset is outside the descriptor), as many as a slot has, so that the loop is
        // entered the way it is re-entered: six loads with a slot's stores behind them.  The compiler's count of what may still be
        // pending at the top of the loop is the merge of both ways in, and without these it waits for the stores of
        // the slot before along with the loads.
        const __amdgpu_buffer_rsrc_t none = make_rsrc(p.y, 0u);
#pragma unroll
        for (int r = 0; r < R * NF; ++r) {
            if constexpr (sizeof(T) == 4) {
                v4u z = {0u, 0u, 0u, 0u};
                __builtin_amdgcn_raw_buffer_store_b128(z, none, (int)(kInvalidOffset + 16u * r), 0, 0);   // (four different ones)
            } else {
                typedef unsigned v2u __attribute__((ext_vector_type(2)));
                v2u z = {0u, 0u};
                __builtin_amdgcn_raw_buffer_store_b64(z, none, (int)(kInvalidOffset + 16u * r), 0, 0);
            }
        }
    }
    for (;;) {
        float4* dst = reinterpret_cast<float4*>(lds + wave * kChB + lane * 16);
#pragma unroll
        for (int i = 0; i < R + 2; ++i) dst[i * (kRowB / 16)] = pre[i].widen();
        __syncthreads();
        const int next = slot + p.walkers;
        const bool more = next < p.slots;
        issue_loads(more ? next : slot, more);
        if constexpr (NF > 0) {
            quad_zero_acc<0>();
            if (cnt[0]) quad_run_entries<NF, 0, CC>(lane_addr, ent_addr, cnt[0]);
        }
        if constexpr (NF > 1) {
            quad_zero_acc<1>();
            if (cnt[1]) quad_run_entries<NF, 1, CC>(lane_addr, ent_addr + kEntRegion, cnt[1]);
        }

        // the slot's outputs: accumulator columns 0 and 5 go to the neighbouring quads; bias, ReLU, store
        int lane_again = lane;
        asm volatile("" : "+v"(lane_again));
        const LanePlace pl = place_of(lane_again, slot);
        const bool has_left = pl.q > 0, has_right = pl.q + 1 < p.QW;
        const unsigned long long ybase = (unsigned long long)pl.n0 * p.out_img_bytes;
        const unsigned long long yleft = p.y_bytes - ybase;
        const __amdgpu_buffer_rsrc_t yrsrc =
            make_rsrc(static_cast<char*>(p.y) + ybase, (uint32_t)(yleft < 0x7FFFFFFFull ? yleft : 0x7FFFFFFFull));
        const unsigned plane_out = (unsigned)(p.Ho * p.Wo) * (unsigned)sizeof(T);
        const unsigned at_img = (unsigned)(pl.n - pl.n0) * p.out_img_bytes +
                                (unsigned)(pl.oy0 * p.Wo + 4 * pl.q) * (unsigned)sizeof(T);
        auto finish_row = [&](auto slot_c, auto row_c) {
            constexpr int a = decltype(slot_c)::value;
            constexpr int r = decltype(row_c)::value;
            int keep = has_filter[a] ? 1 : 0;        // (as `fetch` above)
            asm volatile("" : "+v"(keep));
            float acc[6];
            quad_read_acc_row<a, r>(acc);
            const float from_left = from_lane_below(acc[5]);
            const float from_right = from_lane_above(acc[0]);
            float o[4] = {acc[1] + (has_left ? from_left : 0.f), acc[2], acc[3], acc[4] + (has_right ? from_right : 0.f)};
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                o[m] += filt_bias[a];
                if (p.relu) o[m] = fmaxf(o[m], 0.f);
            }
            const bool ok = keep != 0 && pl.active && pl.oy0 + r < p.Ho;
            const unsigned off = ok ? at_img + filt[a] * plane_out + (unsigned)(r * p.Wo) * (unsigned)sizeof(T)
                                    : kInvalidOffset;
            if constexpr (sizeof(T) == 4) {
                v4u q4;
                q4[0] = f32_to_bits(o[0]);
                q4[1] = f32_to_bits(o[1]);
                q4[2] = f32_to_bits(o[2]);
                q4[3] = f32_to_bits(o[3]);
                __builtin_amdgcn_raw_buffer_store_b128(q4, yrsrc, (int)off, 0, 0);
            } else {
                typedef unsigned v2u __attribute__((ext_vector_type(2)));
                v2u q2;
                q2[0] = (unsigned)__half_as_ushort(__float2half_rn(o[0])) |
                        ((unsigned)__half_as_ushort(__float2half_rn(o[1])) << 16);
                q2[1] = (unsigned)__half_as_ushort(__float2half_rn(o[2])) |
                        ((unsigned)__half_as_ushort(__float2half_rn(o[3])) << 16);
                __builtin_amdgcn_raw_buffer_store_b64(q2, yrsrc, (int)off, 0, 0);
            }
        };
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        using I3 = std::integral_constant<int, 3>;
        if constexpr (NF > 0) { finish_row(I0{}, I0{}); finish_row(I0{}, I1{}); finish_row(I0{}, I2{}); finish_row(I0{}, I3{}); }
        if constexpr (NF > 1) { finish_row(I1{}, I0{}); finish_row(I1{}, I1{}); finish_row(I1{}, I2{}); finish_row(I1{}, I3{}); }
        __syncthreads();               // nobody reads the staged slot any more
        if (!more) break;
        slot = next;
    }
}

// The walking workgroup for layers of several chunks: the chunk loop of quad_body run over the (tile, chunk) pairs of
// all the workgroup's tiles as one sequence, so that the first chunk of the next tile is loaded while the last chunk
// of the current one is multiplied, and its outputs are stored while the next tile is under way; what a workgroup
// pays once per tile otherwise — kernel start, scalar metadata, a memory round trip before the first multiply-add,
// the stores' acknowledgement at the end — it pays once.  Entries are staged per chunk as in quad_body (they are the
// same for every tile and come from the L2).  The outputs of a tile are stored between the two barriers that end
// its last chunk, behind the LDS write of the next chunk: by then the loads in flight have been waited for, so no
// later wait for a load has younger stores to account for, and the stores have a whole chunk's time to complete
// before the next wait (gfx950 counts loads and stores with one counter, in order).
template <int NF, typename T>
__device__ __forceinline__ void quad_stream_body(const QuadParams& p) {
    constexpr int R = PCONV_QUAD_ROWS, FW = 16, CC = 16;
    constexpr unsigned kChB = PCONV_QUAD_CH_BYTES;
    constexpr unsigned kRowB = 64 * 16;
    constexpr unsigned kEntRegion = (CC + 2) * 32;
    constexpr unsigned kEntBase = CC * kChB;
    extern __shared__ __align__(16) unsigned char lds[];     // as in quad_body
    const unsigned lds0 = (unsigned)(unsigned long long)lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    const int per_xcd = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= p.nblocks) return;
    const int walker = (int)fastdiv((unsigned)logical, p.div_NG);
    const int g0 = logical - walker * p.NG;
    const int K = p.nbk;                                      // chunks per tile
    // The filter groups are in the packed order, most kept kernels first, so a workgroup that stayed with one group
    // would do up to 15 % more or less than the average; it takes group g0 for its even tiles and NG-1-g0 for its odd
    // ones instead.  (At any time the NG workgroups of a walker are still on the same tile, one per group.)
    auto group_of = [&](int j) { return (j & 1) ? p.NG - 1 - g0 : g0; };

    struct LanePlace { int q, n, n0, oy0; bool active; };
    auto place_of = [&](int ln, int slot) {
        LanePlace r;
        const int g0 = slot * p.BL;
        r.n0 = (int)fastdiv((unsigned)g0, p.div_NRB);
        const int b = (int)fastdiv((unsigned)ln, p.div_QW);
        r.q = ln - b * p.QW;
        r.active = b < p.BL && g0 + b < p.NBLK;
        const int g = r.active ? g0 + b : g0;
        r.n = (int)fastdiv((unsigned)g, p.div_NRB);
        r.oy0 = (g - r.n * p.NRB) * R;
        return r;
    };

    // Input offsets and descriptor of the tile whose chunks are being loaded: the offset of the lane's quad in patch
    // row 0 (modulo 2^32 where that row is above the image) and which of the six rows exist — two registers held
    // across the loop instead of six offsets.
    unsigned first_off, rows_ok;
    __amdgpu_buffer_rsrc_t rsrc;
    auto aim_at = [&](int slot) {
        const LanePlace pl = place_of(lane, slot);
        const int iy0 = pl.oy0 - p.pad;
        first_off = (unsigned)(pl.n - pl.n0) * p.img_bytes + (unsigned)(iy0 * p.W + 4 * pl.q) * (unsigned)sizeof(T);
        rows_ok = 0u;
#pragma unroll
        for (int i = 0; i < R + 2; ++i)
            if (pl.active && iy0 + i >= 0 && iy0 + i < p.H) rows_ok |= 1u << i;
        const unsigned long long base_off = (unsigned long long)pl.n0 * p.img_bytes;
        const unsigned long long left = p.x_bytes - base_off;
        rsrc = make_rsrc(static_cast<const char*>(p.x) + base_off, (uint32_t)(left < 0x7FFFFFFFull ? left : 0x7FFFFFFFull));
    };
    const unsigned row_bytes = (unsigned)p.W * (unsigned)sizeof(T);

    const unsigned lane_addr = lds0 + lane * 16;
    const unsigned ent_addr = lds0 + kEntBase + wave * NF * kEntRegion;
    // filters and biases of the tile that is multiplied (fetched when its first chunk starts)
    unsigned filt[NF];
    float filt_bias[NF];
    bool has_filter[NF];
    auto fetch_filters = [&](int grp) {
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const int pos = grp * (FW * NF) + wave + a * FW;
            has_filter[a] = pos < p.F;
            filt[a] = has_filter[a] ? scalar_load_u32(p.forder + pos) : 0u;
            filt_bias[a] = (p.bias && has_filter[a])
                               ? __builtin_bit_cast(float, scalar_load_u32(reinterpret_cast<const uint32_t*>(p.bias + filt[a])))
                               : 0.f;
        }
    };

    // (see quad_body for why loads and their use are unconditional and the metadata runs a chunk ahead)
    RawQuad<T> pre[R + 2];
    uint2 epre[NF];
    unsigned ecnt[NF];
    const __amdgpu_buffer_rsrc_t ent_rsrc = make_rsrc(p.ent, p.ent_bytes);
    unsigned meta_e0[NF], meta_e1[NF], meta_c;
    auto fetch_meta = [&](int grp, int k, bool any) {      // chunk k of the group, or nothing
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const int pos = grp * (FW * NF) + wave + a * FW;
            meta_e0[a] = meta_e1[a] = 0;
            if (any && pos < p.F) {
                meta_e0[a] = scalar_load_u32(p.eptr + pos * p.nbk + k);
                meta_e1[a] = scalar_load_u32(p.eptr + pos * p.nbk + k + 1);
            }
        }
        meta_c = !any ? kNoChannel
                 : p.perm ? scalar_load_u32(p.perm + (size_t)grp * p.perm_stride + k * CC + wave)
                          : (unsigned)(k * CC + wave);
    };
    // (the loads of a chunk in two parts, as in quad_body: entries in front of the first filter's kept kernels, patch
    // rows behind them)
    constexpr bool kSplit = NF > 1;               // loads issued behind the first filter's entries
    unsigned load_soff = 0u, load_rows = 0u;
    auto issue_entry_loads = [&]() {
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            const unsigned eoff = (unsigned)(lane >> 2) < ecnt[a] ? meta_e0[a] * 32u + (unsigned)lane * 8u : kInvalidOffset;
            typedef unsigned v2u __attribute__((ext_vector_type(2)));
            const v2u e = __builtin_amdgcn_raw_buffer_load_b64(ent_rsrc, (int)eoff, 0, 0);
            epre[a] = make_uint2(e[0], e[1]);
        }
    };
    auto issue_row_loads = [&]() {
#pragma unroll
        for (int i = 0; i < R + 2; ++i)
            pre[i].load(rsrc, ((load_rows >> i) & 1u) ? first_off + (unsigned)i * row_bytes : kInvalidOffset, load_soff);
    };
    auto issue_loads_first = [&]() {              // the chunk of the last fetch_meta, of the tile last aimed at
#pragma unroll
        for (int a = 0; a < NF; ++a) ecnt[a] = meta_e1[a] - meta_e0[a];
        const bool staged = meta_c < (unsigned)p.C;
        load_soff = staged ? meta_c * p.plane_bytes : 0u;
        load_rows = staged ? rows_ok : 0u;
        issue_entry_loads();                      // (measured: moving these back as well costs 2 %)
        if constexpr (!kSplit) issue_row_loads();
    };
    auto issue_loads_rest = [&]() {               // (nothing fetches metadata between the two parts)
        if constexpr (kSplit) issue_row_loads();
    };
    auto issue_loads = [&]() {
        issue_loads_first();
        issue_loads_rest();
    };
    auto write_lds = [&]() {
        float4* dst = reinterpret_cast<float4*>(lds + wave * kChB + lane * 16);
#pragma unroll
        for (int i = 0; i < R + 2; ++i) dst[i * (kRowB / 16)] = pre[i].widen();
        static_assert(kEntRegion >= 64 * 8, "entry region smaller than one wave's write");
#pragma unroll
        for (int a = 0; a < NF; ++a) {
            uint2* e = reinterpret_cast<uint2*>(lds + kEntBase + (wave * NF + a) * kEntRegion);
            e[lane] = epre[a];
        }
    };
    // outputs of the tile `slot`, from the accumulators
    auto store_tile = [&](int slot) {
        int lane_again = lane;
        asm volatile("" : "+v"(lane_again));
        const LanePlace pl = place_of(lane_again, slot);
        const bool has_left = pl.q > 0, has_right = pl.q + 1 < p.QW;
        const unsigned long long ybase = (unsigned long long)pl.n0 * p.out_img_bytes;
        const unsigned long long yleft = p.y_bytes - ybase;
        const __amdgpu_buffer_rsrc_t yrsrc =
            make_rsrc(static_cast<char*>(p.y) + ybase, (uint32_t)(yleft < 0x7FFFFFFFull ? yleft : 0x7FFFFFFFull));
        const unsigned plane_out = (unsigned)(p.Ho * p.Wo) * (unsigned)sizeof(T);
        const unsigned at_img = (unsigned)(pl.n - pl.n0) * p.out_img_bytes +
                                (unsigned)(pl.oy0 * p.Wo + 4 * pl.q) * (unsigned)sizeof(T);
        auto finish_row = [&](auto slot_c, auto row_c) {
            constexpr int a = decltype(slot_c)::value;
            constexpr int r = decltype(row_c)::value;
            float acc[6];
            quad_read_acc_row<a, r>(acc);
            const float from_left = from_lane_below(acc[5]);
            const float from_right = from_lane_above(acc[0]);
            float o[4] = {acc[1] + (has_left ? from_left : 0.f), acc[2], acc[3], acc[4] + (has_right ? from_right : 0.f)};
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                o[m] += filt_bias[a];
                if (p.relu) o[m] = fmaxf(o[m], 0.f);
            }
            const bool ok = has_filter[a] && pl.active && pl.oy0 + r < p.Ho;
            const unsigned off = ok ? at_img + filt[a] * plane_out + (unsigned)(r * p.Wo) * (unsigned)sizeof(T)
                                    : kInvalidOffset;
            if constexpr (sizeof(T) == 4) {
                v4u q4;
                q4[0] = f32_to_bits(o[0]);
                q4[1] = f32_to_bits(o[1]);
                q4[2] = f32_to_bits(o[2]);
                q4[3] = f32_to_bits(o[3]);
                __builtin_amdgcn_raw_buffer_store_b128(q4, yrsrc, (int)off, 0, 0);
            } else {
                typedef unsigned v2u __attribute__((ext_vector_type(2)));
                v2u q2;
                q2[0] = (unsigned)__half_as_ushort(__float2half_rn(o[0])) |
                        ((unsigned)__half_as_ushort(__float2half_rn(o[1])) << 16);
                q2[1] = (unsigned)__half_as_ushort(__float2half_rn(o[2])) |
                        ((unsigned)__half_as_ushort(__float2half_rn(o[3])) << 16);
                __builtin_amdgcn_raw_buffer_store_b64(q2, yrsrc, (int)off, 0, 0);
            }
        };
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        using I3 = std::integral_constant<int, 3>;
        if constexpr (NF > 0) { finish_row(I0{}, I0{}); finish_row(I0{}, I1{}); finish_row(I0{}, I2{}); finish_row(I0{}, I3{}); }
        if constexpr (NF > 1) { finish_row(I1{}, I0{}); finish_row(I1{}, I1{}); finish_row(I1{}, I2{}); finish_row(I1{}, I3{}); }
    };

    // The sequence: tiles number j = 0, 1, ... of this workgroup (slot walker + j * walkers < slots), K chunks each.
    // Three positions move along it: (fj, fk) the pair whose metadata is fetched next, (lj, lk) the pair whose loads
    // are issued next, (cj, k) the pair that is multiplied.
    auto slot_of = [&](int j) { return walker + j * p.walkers; };
    auto step = [&](int& j, int& c) {
        if (++c == K) {
            c = 0;
            ++j;
        }
    };
    int cj = 0, k = 0, lj = 0, lk = 0, fj = 0, fk = 0;
    if constexpr (NF > 0) quad_zero_acc<0>();
    if constexpr (NF > 1) quad_zero_acc<1>();
    aim_at(slot_of(0));
    fetch_meta(group_of(0), 0, true);      // walker < walkers <= slots: the first pair exists
    step(fj, fk);
    issue_loads();
    step(lj, lk);
    fetch_meta(group_of(fj), fk, slot_of(fj) < p.slots);
    step(fj, fk);
    write_lds();
    __syncthreads();
    unsigned cnt_now[NF];
    for (;;) {
        const bool more = slot_of(lj) < p.slots;   // a pair behind the current one
#pragma unroll
        for (int a = 0; a < NF; ++a) cnt_now[a] = ecnt[a];
        if (more) {
            if (lk == 0) aim_at(slot_of(lj));      // (uniform)
            issue_loads_first();
        }
        step(lj, lk);
        if (k == 0) fetch_filters(group_of(cj));   // (uniform) needed when the tile is stored
        if constexpr (NF > 0) { if (cnt_now[0]) quad_run_entries<NF, 0, CC>(lane_addr, ent_addr, cnt_now[0]); }
        if (more) issue_loads_rest();
        if constexpr (NF > 1) { if (cnt_now[1]) quad_run_entries<NF, 1, CC>(lane_addr, ent_addr + kEntRegion, cnt_now[1]); }
        fetch_meta(group_of(fj), fk, slot_of(fj) < p.slots);
        step(fj, fk);
        __syncthreads();                   // every wave is done reading the staged chunk
        if (more) write_lds();
        if (k == K - 1) {                  // (uniform) the tile is complete
            store_tile(slot_of(cj));
            if constexpr (NF > 0) quad_zero_acc<0>();
            if constexpr (NF > 1) quad_zero_acc<1>();
        }
        if (!more) break;
        __syncthreads();
        step(cj, k);
    }
}

template <typename T>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_num_vgpr(36))) void quad_stream_kernel_nf1(const QuadParams p) {
    static_assert(PCONV_QUAD_SCRATCH_FIRST_NF1 >= 2 * 36, "the entry loop's registers overlap the compiler's");
    quad_stream_body<1, T>(p);
}
template <typename T>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_num_vgpr(24))) void quad_stream_kernel_nf2(const QuadParams p) {
    static_assert(PCONV_QUAD_SCRATCH_FIRST_NF2 >= 2 * 24, "the entry loop's registers overlap the compiler's");
    quad_stream_body<2, T>(p);
}

template <typename T>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_num_vgpr(36))) void quad_walk_kernel_nf1(const QuadParams p) {
    static_assert(PCONV_QUAD_SCRATCH_FIRST_NF1 >= 2 * 36, "the entry loop's registers overlap the compiler's");
    quad_walk_body<1, T>(p);
}
template <typename T>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_num_vgpr(24))) void quad_walk_kernel_nf2(const QuadParams p) {
    static_assert(PCONV_QUAD_SCRATCH_FIRST_NF2 >= 2 * 24, "the entry loop's registers overlap the compiler's");
    quad_walk_body<2, T>(p);
}

template <int FW, typename T>
__global__ __launch_bounds__(FW * 64) __attribute__((amdgpu_num_vgpr(36))) void quad_kernel_nf1(const QuadParams p) {
    static_assert(PCONV_QUAD_SCRATCH_FIRST_NF1 >= 2 * 36, "the entry loop's registers overlap the compiler's");
    quad_body<1, FW, T>(p);
}
template <int FW, typename T>
__global__ __launch_bounds__(FW * 64) __attribute__((amdgpu_num_vgpr(24))) void quad_kernel_nf2(const QuadParams p) {
    static_assert(PCONV_QUAD_SCRATCH_FIRST_NF2 >= 2 * 24, "the entry loop's registers overlap the compiler's");
    quad_body<2, FW, T>(p);
}

// ---------------------------------------------------------------------------------------------------------------
// generic kernel: any stride / pad; one thread per output, one filter per workgroup row
// ---------------------------------------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(256) void generic_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                      const DevEntry* __restrict__ ent,
                                                      const uint32_t* __restrict__ eptr,
                                                      const uint32_t* __restrict__ forder,
                                                      const float* __restrict__ bias, int C, int F, int H, int W, int Ho,
                                                      int Wo, int stride, int pad, int nch, int relu) {
    const int pos = blockIdx.y, n = blockIdx.z;
    const int pix = blockIdx.x * 256 + threadIdx.x;
    const bool ok = pix < Ho * Wo;
    const int oy = ok ? pix / Wo : 0, ox = ok ? pix - (pix / Wo) * Wo : 0;
    const unsigned f = forder[pos];
    const unsigned e0 = eptr[pos * nch], e1 = eptr[(pos + 1) * nch];
    const size_t plane = (size_t)H * W;
    const T* xn = x + (size_t)n * C * plane;
    float acc = 0.f;
    for (unsigned e = e0; e < e1; ++e) {
        const DevEntry d = ent[e];   // wave-uniform address
        const T* xc = xn + (size_t)d.c * plane;
        int q = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if ((d.mask9 >> t) & 1u) {
                const int iy = oy * stride + t / 3 - pad, ix = ox * stride + t % 3 - pad;
                const float wv = q == 0 ? d.w[0] : q == 1 ? d.w[1] : q == 2 ? d.w[2] : d.w[3];
                if (ok && iy >= 0 && iy < H && ix >= 0 && ix < W) acc = fmaf(wv, to_f32<T>(xc[(size_t)iy * W + ix]), acc);
                ++q;
            }
        }
    }
    if (ok) {
        float v = acc + (bias ? bias[f] : 0.f);
        if (relu) v = fmaxf(v, 0.f);
        y[(((size_t)n * F + f) * Ho + oy) * (size_t)Wo + ox] = from_f32<T>(v);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// dense 3x3 baseline: one thread per output, one filter per workgroup row, all nine taps of all channels
// ---------------------------------------------------------------------------------------------------------------

template <typename T>
__global__ __launch_bounds__(256) void dense_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                    const T* __restrict__ w, const float* __restrict__ bias, int C,
                                                    int F, int H, int W, int Ho, int Wo, int stride, int pad, int relu) {
    const int f = blockIdx.y, n = blockIdx.z;
    const int pix = blockIdx.x * 256 + threadIdx.x;
    const bool ok = pix < Ho * Wo;
    const int oy = ok ? pix / Wo : 0, ox = ok ? pix - (pix / Wo) * Wo : 0;
    const size_t plane = (size_t)H * W;
    const T* xn = x + (size_t)n * C * plane;
    const T* wf = w + (size_t)f * C * 9;
    float acc = 0.f;
    for (int c = 0; c < C; ++c) {
        const T* xc = xn + (size_t)c * plane;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int iy = oy * stride + t / 3 - pad, ix = ox * stride + t % 3 - pad;
            const float wv = to_f32<T>(wf[c * 9 + t]);
            if (ok && iy >= 0 && iy < H && ix >= 0 && ix < W) acc = fmaf(wv, to_f32<T>(xc[(size_t)iy * W + ix]), acc);
        }
    }
    if (ok) {
        float v = acc + (bias ? bias[f] : 0.f);
        if (relu) v = fmaxf(v, 0.f);
        y[(((size_t)n * F + f) * Ho + oy) * (size_t)Wo + ox] = from_f32<T>(v);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool_kernel(const T* __restrict__ x, T* __restrict__ y, long long planes,
                                                      int H, int W) {
    const int Ho = H / 2, Wo = W / 2;
    const long long total = planes * Ho * Wo;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        const int ox = (int)(i % Wo);
        const long long r = i / Wo;
        const int oy = (int)(r % Ho);
        const long long pl = r / Ho;
        const T* xp = x + (pl * H + 2 * oy) * (long long)W + 2 * ox;
        const float a = to_f32<T>(xp[0]), b = to_f32<T>(xp[1]), c = to_f32<T>(xp[W]), d = to_f32<T>(xp[W + 1]);
        y[i] = from_f32<T>(fmaxf(fmaxf(a, b), fmaxf(c, d)));
    }
}

// Splits every input plane into its four row/column parity planes: out[pl][2a+b][i][j] = x[pl][2i+a][2j+b] (zero
// where that is outside the image).  A stride-2 convolution reads each parity plane at unit stride.
// One workgroup per input plane and band of 4 plane rows; thread (ty, tx) walks the columns in steps of 64.
template <typename T>
__global__ __launch_bounds__(256) void parity_planes_kernel(const T* __restrict__ x, T* __restrict__ out, int H, int W,
                                                            int Hs, int Ws) {
    const long long pl = blockIdx.x;
    const int i = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (i >= Hs) return;
    const T* src = x + pl * (long long)H * W;
    T* dst = out + pl * 4ll * Hs * Ws;
    const T zero = from_f32<T>(0.f);
    const bool row1 = 2 * i + 1 < H;
    for (int j = threadIdx.x & 63; j < Ws; j += 64) {
        const bool col1 = 2 * j + 1 < W;
        const T* s0 = src + (long long)(2 * i) * W + 2 * j;
        const T v00 = s0[0];
        const T v01 = col1 ? s0[1] : zero;
        const T v10 = row1 ? s0[W] : zero;
        const T v11 = (row1 && col1) ? s0[W + 1] : zero;
        const long long o = (long long)i * Ws + j, ps = (long long)Hs * Ws;
        dst[o] = v00;
        dst[ps + o] = v01;
        dst[2 * ps + o] = v10;
        dst[3 * ps + o] = v11;
    }
}

// ---------------------------------------------------------------------------------------------------------------
// launch selection
// ---------------------------------------------------------------------------------------------------------------

// Dynamic LDS above 64 KiB has to be allowed per kernel function.  The attribute is set on every launch that needs
// it: it is a cheap host-side call and keeps the library free of global mutable state.
static hipError_t allow_big_lds(const void* fn, size_t lds) {
    if (lds <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
}

template <typename K>
static int launch_tiled_inst(K kern, const TiledParams& p, int waves, int NF, int CC, int buffers, hipStream_t stream) {
    const int grid = (p.nblocks + 7) / 8 * 8;
    const size_t lds = (size_t)buffers * ((size_t)CC * kChBytes + (size_t)waves * NF * (CC + 2) * 32);
    if (lds > 160 * 1024) return PCONV_EUNSUPPORTED;
    PCONV_HIP(allow_big_lds((const void*)kern, lds));
    hipLaunchKernelGGL(kern, dim3(grid), dim3(waves * 64), lds, stream, p);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

template <typename T>
static int launch_tiled(TiledParams& p, const pconv_packed* wp, int NF, int waves, int CPW, int KS, int buffers,
                        hipStream_t stream, const WsArena* arena) {
    const int CC = CPW * waves;
    if (CC % kBucket != 0) return PCONV_EUNSUPPORTED;   // a chunk is a whole number of buckets
    const int NB = CC / kBucket;
    // tile geometry
    const int Wo = p.Wo, Ho = p.Ho;
    const int ncs = (Wo + 61) / 62;
    p.OWS = (Wo + ncs - 1) / ncs;
    p.NCS = (Wo + p.OWS - 1) / p.OWS;
    p.LW = p.OWS + 2;
    p.S = 64 / p.LW;
    p.NRB = (Ho + kR - 1) / kR;
    const long long nseg = (long long)p.N * p.NRB * p.NCS;
    if (nseg > 0x7FFFFFFF) return PCONV_ESHAPE;
    p.NSEG = (int)nseg;
    const int slots = (int)((nseg + p.S - 1) / p.S);
    p.NG = (p.F + waves * NF - 1) / (waves * NF);
    const int nchunks = p.perm ? p.nbk : (p.C + CC - 1) / CC;
    if (KS == 0) {
        // Automatic: one round of workgroups over the compute units when the tiles alone are fewer than that
        const long long tiles = (long long)slots * p.NG;
        KS = (int)std::max<long long>(1, std::min<long long>(compute_units() / std::max<long long>(tiles, 1), 16));
        KS = std::min(KS, nchunks);
    }
    if (KS < 1 || KS > nchunks || KS > 64) return PCONV_EUNSUPPORTED;
    const long long nb = (long long)slots * p.NG * KS;
    if (nb > 0x7FFFFFF0) return PCONV_ESHAPE;
    p.nblocks = (int)nb;
    p.KS = KS;
    p.div_KS = make_fastdiv((unsigned)KS);
    p.div_NG = make_fastdiv((unsigned)p.NG);
    p.div_LW = make_fastdiv((unsigned)p.LW);
    p.div_segs_per_img = make_fastdiv((unsigned)(p.NCS * p.NRB));
    p.div_NCS = make_fastdiv((unsigned)p.NCS);
    p.ws = nullptr;
    p.counters = nullptr;
    if (KS > 1) {
        // eight words per lane, filter slot and wave of every tile; one split's part is addressed with 32-bit offsets
        const size_t split_bytes = (size_t)slots * p.NG * waves * NF * 64 * 8 * sizeof(float);
        if (split_bytes >= kInvalidOffset) return PCONV_EUNSUPPORTED;
        if (int rc = get_workspace(wp, arena, (size_t)KS * split_bytes / sizeof(float), (size_t)slots * p.NG, &p.ws,
                                   &p.counters, stream))
            return rc;
        p.ws_split_bytes = (unsigned)split_bytes;
    }
    // (filters per wave, channels per wave and chunk, buckets per chunk); waves = 16 * NB / CPW
#define PCONV_CASE(FF, PP, BB) \
    if (NF == FF && CPW == PP && NB == BB && buffers == 1) \
        return launch_tiled_inst(tiled_kernel_nf##FF<PP, BB, false, false, T>, p, waves, NF, CC, 1, stream);
#define PCONV_CASE_DB(FF, PP) \
    if (NF == FF && CPW == PP && NB == 1 && buffers == 2) \
        return launch_tiled_inst(tiled_kernel_nf##FF<PP, 1, true, false, T>, p, waves, NF, CC, 2, stream);
    if (p.pair) {
        if (CPW != 2 || NB != 2 || buffers != 1 || p.perm) return PCONV_EUNSUPPORTED;
        if (NF == 1) return launch_tiled_inst(tiled_kernel_nf1<2, 2, false, true, T>, p, waves, NF, CC, 1, stream);
        if (NF == 2) return launch_tiled_inst(tiled_kernel_nf2<2, 2, false, true, T>, p, waves, NF, CC, 1, stream);
        return PCONV_EUNSUPPORTED;
    }
    PCONV_CASE(1, 1, 1) PCONV_CASE(1, 2, 1) PCONV_CASE(1, 4, 1) PCONV_CASE(1, 2, 2) PCONV_CASE(1, 4, 2)
    PCONV_CASE(2, 1, 1) PCONV_CASE(2, 2, 1) PCONV_CASE(2, 2, 2)
    PCONV_CASE_DB(1, 1) PCONV_CASE_DB(1, 2) PCONV_CASE_DB(2, 1) PCONV_CASE_DB(2, 2)
#undef PCONV_CASE
#undef PCONV_CASE_DB
    return PCONV_EUNSUPPORTED;
}

// walk: 0 = automatic, 1 = never, 2 = always: quad_walk_kernel instead of quad_kernel_nf1
template <typename T>
static int launch_quad(QuadParams& p, const pconv_packed* wp, int NF, int FW, int KS, int walk, hipStream_t stream,
                       const WsArena* arena) {
    constexpr int R = PCONV_QUAD_ROWS;
    if (p.W % 4 != 0 || p.W / 4 > 64) return PCONV_EUNSUPPORTED;
    if (NF != 1 && NF != 2) return PCONV_EUNSUPPORTED;   // NG below is computed for the kernels that exist
    p.QW = p.W / 4;
    p.BL = 64 / p.QW;
    p.NRB = (p.Ho + R - 1) / R;
    const long long nblk = (long long)p.N * p.NRB;
    if (nblk > 0x7FFFFFFF) return PCONV_ESHAPE;
    p.NBLK = (int)nblk;
    const long long slots = (nblk + p.BL - 1) / p.BL;
    // Only workgroups of 16 waves are built: eight waves with eight-channel chunks (two workgroups per CU) measured
    // within 3 % of them on the VGG-16 shapes at batch 64, slower on most.
    if (FW != 16) return PCONV_EUNSUPPORTED;
    p.NG = (p.F + FW * NF - 1) / (FW * NF);
    const bool ks_auto = KS == 0;      // decided below, once it is clear that the workgroups do not walk
    KS = std::max(1, std::min(KS, p.nbk));
    if (slots * p.NG * KS > 0x7FFFFFF0) return PCONV_ESHAPE;
    // pad 1: Wo == W, so a lane's four outputs of a row start at a multiple of four columns and are all inside
    p.vec = (p.pad == 1 && reinterpret_cast<uintptr_t>(p.y) % 16 == 0) ? 1 : 0;
    p.ws = nullptr;
    p.counters = nullptr;
    // 32-bit byte offsets inside the buffer descriptor: the images one slot can span
    const unsigned long long span = (unsigned long long)((p.BL + p.NRB - 1) / p.NRB + 1);
    if ((unsigned long long)p.img_bytes * span >= 0x7FFFFFFFull) return PCONV_EUNSUPPORTED;
    p.div_NG = make_fastdiv((unsigned)p.NG);
    p.div_QW = make_fastdiv((unsigned)p.QW);
    p.div_NRB = make_fastdiv((unsigned)p.NRB);
    const size_t lds = (size_t)FW * PCONV_QUAD_CH_BYTES + (size_t)FW * NF * (FW + 2) * 32;
    // One chunk of channels and many slots: workgroups that keep their filters and walk over the slots, as many as
    // give every CU one.  (The outputs go through a buffer descriptor there, too.)
    const unsigned long long out_img = (unsigned long long)p.F * p.Ho * p.Wo * sizeof(T);
    // (two filters per wave: fp16 storage only; with fp32 the six rows in flight do not fit the registers left)
    const bool can_walk = KS == 1 && p.vec && p.NG <= 256 && out_img * span < 0x7FFFFFFFull && slots < 0x7FFF0000ll &&
                          (NF == 1 || sizeof(T) == 2);
    if (walk < 0 || walk > 2) return PCONV_EINVAL;
    if (walk == 2 && !can_walk) return PCONV_EUNSUPPORTED;
    const int cus = compute_units();
    const long long walkers = std::min<long long>(slots, std::max(1, cus / p.NG));
    // Cost of one workgroup per tile, in chunks: the rounds of 256 workgroups times a workgroup's chunks plus half a
    // chunk for what it cannot overlap at its start and end, plus 1.2 for partial sums and their reduction if the
    // channels are split.  A split (automatic: 2 or 4) is taken where it evens out the rounds — 800 tiles are 3.1
    // rounds, so four; 1600 half-length workgroups are 6.25, so seven halves — from 3 % predicted gain on.
    const long long tiles = slots * p.NG;
    auto tile_cost = [&](int ks) {
        const double rounds = (double)((tiles * ks + cus - 1) / cus);
        return rounds * ((double)((p.nbk + ks - 1) / ks) + 0.5 + (ks > 1 ? 1.2 : 0.0));
    };
    double best_tile = tile_cost(KS);
    if (ks_auto)
        for (int ks = 2; ks <= std::min(4, p.nbk); ks *= 2) {
            if ((unsigned long long)tiles * FW * NF * 4096ull >= kInvalidOffset) break;
            if (tile_cost(ks) < 0.97 * best_tile) {
                best_tile = tile_cost(ks);
                KS = ks;
            }
        }
    // Walking workgroups, automatic.  One chunk: from 1.5 tiles per workgroup on (13 to 32 % faster at batch 4 to 64).
    // Several chunks: a walker runs its tiles back to back and pays the half chunk once; with an odd number of
    // tiles the alternation between a heavy and a light filter group leaves it 7 % of a tile off balance.  Measured
    // on the VGG-16 layers at batch 4 to 64: 2 to 16 % faster where this estimate says so, level elsewhere.
    bool walking = walk == 2;
    if (walk == 0 && can_walk) {
        const long long nt = (slots + walkers - 1) / walkers;      // tiles of the busiest walker
        if (p.nbk == 1) {
            walking = 2 * slots >= 3 * walkers;
        } else {
            const double walk_cost = (double)nt * p.nbk + 0.5 + (((nt & 1) && p.NG > 1) ? 0.07 * p.nbk : 0.0);
            walking = nt >= 2 && walk_cost < 0.99 * best_tile;
        }
    }
    if (walking) {
        p.KS = 1;
        p.div_KS = make_fastdiv(1u);
        p.walkers = (int)walkers;
        p.slots = (int)slots;
        p.out_img_bytes = (unsigned)out_img;
        p.y_bytes = (unsigned long long)p.N * out_img;
        p.nblocks = p.NG * p.walkers;
        const int wgrid = (p.nblocks + 7) / 8 * 8;
        if (p.nbk == 1) {          // the entries stay in LDS
            if (NF == 1) {
                PCONV_HIP(allow_big_lds((const void*)quad_walk_kernel_nf1<T>, lds));
                hipLaunchKernelGGL((quad_walk_kernel_nf1<T>), dim3(wgrid), dim3(1024), lds, stream, p);
            } else if constexpr (sizeof(T) == 2) {
                PCONV_HIP(allow_big_lds((const void*)quad_walk_kernel_nf2<T>, lds));
                hipLaunchKernelGGL((quad_walk_kernel_nf2<T>), dim3(wgrid), dim3(1024), lds, stream, p);
            } else {
                return PCONV_EUNSUPPORTED;
            }
        } else {
            if (NF == 1) {
                PCONV_HIP(allow_big_lds((const void*)quad_stream_kernel_nf1<T>, lds));
                hipLaunchKernelGGL((quad_stream_kernel_nf1<T>), dim3(wgrid), dim3(1024), lds, stream, p);
            } else if constexpr (sizeof(T) == 2) {
                PCONV_HIP(allow_big_lds((const void*)quad_stream_kernel_nf2<T>, lds));
                hipLaunchKernelGGL((quad_stream_kernel_nf2<T>), dim3(wgrid), dim3(1024), lds, stream, p);
            } else {
                return PCONV_EUNSUPPORTED;
            }
        }
        PCONV_HIP(hipGetLastError());
        return PCONV_OK;
    }
    const long long nb = slots * p.NG * KS;
    if (nb > 0x7FFFFFF0) return PCONV_ESHAPE;
    p.nblocks = (int)nb;
    p.KS = KS;
    p.div_KS = make_fastdiv((unsigned)KS);
    if (KS > 1) {
        // 16 words per lane, filter slot and wave of every tile; one split's part is addressed with 32-bit offsets
        const size_t split_bytes = (size_t)slots * p.NG * FW * NF * 64 * 16 * sizeof(float);
        if (split_bytes >= kInvalidOffset) return PCONV_EUNSUPPORTED;
        if (int rc = get_workspace(wp, arena, (size_t)KS * split_bytes / sizeof(float), (size_t)slots * p.NG, &p.ws,
                                   &p.counters, stream))
            return rc;
        p.ws_split_bytes = (unsigned)split_bytes;
    }
    const int grid = (p.nblocks + 7) / 8 * 8;
#define PCONV_QCASE(NFv, FWv)                                                                           \
    if (NF == NFv && FW == FWv) {                                                                       \
        PCONV_HIP(allow_big_lds((const void*)quad_kernel_nf##NFv<FWv, T>, lds));                        \
        hipLaunchKernelGGL((quad_kernel_nf##NFv<FWv, T>), dim3(grid), dim3(FWv * 64), lds, stream, p);  \
    } else
    PCONV_QCASE(1, 16) PCONV_QCASE(2, 16) { return PCONV_EUNSUPPORTED; }
#undef PCONV_QCASE
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

// Whether the kernel with four columns per lane can run the layer, and with how many workgroups at two filters per
// wave (same conditions as launch_quad checks).
static bool quad_applicable(int N, int C, int F, int H, int W, int Ho, int stride, size_t esize, long long* workgroups) {
    if (stride != 1 || W % 4 != 0 || W / 4 > 64) return false;
    const unsigned long long img = (unsigned long long)C * H * W * esize;
    const int BL = 64 / (W / 4), NRB = (Ho + PCONV_QUAD_ROWS - 1) / PCONV_QUAD_ROWS;
    if (img * (unsigned long long)((BL + NRB - 1) / NRB + 1) >= 0x7FFFFFFFull) return false;
    const long long nblk = (long long)N * NRB;
    if (nblk > 0x7FFFFFFF) return false;
    *workgroups = (nblk + BL - 1) / BL * ((F + 31) / 32);
    return *workgroups <= 0x7FFFFFF0;
}

// The dense baseline's weights in matrix-core order: one buffer per device, grown on demand, kept until the process
// ends.  Calls of pconv_dense_conv3x3 with fp16 storage that overlap in time on one device share it and race.
static int dense_weight_buffer(size_t bytes, void** out) {
    static std::mutex mu;
    static void* buf[kMaxDevices] = {};
    static size_t cap[kMaxDevices] = {};
    int dev = -1;
    PCONV_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return PCONV_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (bytes > cap[dev]) {
        if (buf[dev]) PCONV_HIP(hipFree(buf[dev]));
        buf[dev] = nullptr;
        cap[dev] = 0;
        PCONV_HIP(hipMalloc(&buf[dev], bytes));
        cap[dev] = bytes;
    }
    *out = buf[dev];
    return PCONV_OK;
}

static bool tiled_applicable(int N, int C, int H, int W, int stride, size_t esize) {
    if (stride != 1) return false;
    // 32-bit byte offsets inside the buffer descriptor: one image, times the few images one slot can span
    const unsigned long long img = (unsigned long long)C * H * W * esize;
    const int lw = std::min(W, 62) + 2;
    const int s = std::max(1, 64 / lw);
    (void)N;
    return img * (unsigned long long)(s + 1) < 0x7FFFFFFFull;
}

}  // namespace pconv

// ---------------------------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------------------------

using namespace pconv;

extern "C" const char* pconv_last_hip_error(void) { return g_hip_error; }

static int check_conv_args(const void* x, const void* y, int N, int C, int F, int H, int W, int stride, int pad,
                           unsigned flags, int* Ho, int* Wo) {
    if (!x || !y) return PCONV_EINVAL;
    if (flags & ~(unsigned)(PCONV_FLAG_RELU | PCONV_FLAG_NHWC)) return PCONV_EINVAL;
    if (stride != 1 && stride != 2) return PCONV_EUNSUPPORTED;
    if (pad != 0 && pad != 1) return PCONV_EUNSUPPORTED;
    if (N < 0 || C <= 0 || F <= 0 || H <= 0 || W <= 0) return PCONV_ESHAPE;
    if (H + 2 * pad < 3 || W + 2 * pad < 3) return PCONV_ESHAPE;
    *Ho = (H + 2 * pad - 3) / stride + 1;
    *Wo = (W + 2 * pad - 3) / stride + 1;
    if ((long long)*Ho * *Wo > 0x7FFFFFFF || N > 65535 || F > 65535) return PCONV_ESHAPE;
    if ((unsigned long long)N * C * H * W >= (1ull << 40) || (unsigned long long)N * F * *Ho * *Wo >= (1ull << 40))
        return PCONV_ESHAPE;
    return PCONV_OK;
}

// `arena` null: the handle's own workspace, allocated and grown on demand.  Otherwise the call allocates nothing:
// split launches take their workspace from the arena, and a form of the layer that is not there yet is an error.
// `plan` not null: nothing is launched or allocated; the kernel family that the call would take (and for the
// matrix-core kernel its tile shape) is written there.
struct PlanOut {
    int kernel, mfma_shape;
};
static int conv3x3_impl(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H, int W,
                        int stride, int pad, unsigned flags, void* stream, const pconv_tuning* tuning,
                        const WsArena* arena, PlanOut* plan = nullptr) {
    if (!wp) return PCONV_EINVAL;
    int Ho = 0, Wo = 0;
    if (int rc = check_conv_args(x, y, N, wp->C, wp->F, H, W, stride, pad, flags, &Ho, &Wo)) return rc;
    if (!wp->d_ent) return PCONV_ESTATE;
    int dev = -1;
    PCONV_HIP(hipGetDevice(&dev));
    if (dev != wp->device) return PCONV_ESTATE;
    if (N == 0) return PCONV_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t esize = wp->dtype == PCONV_F16 ? 2 : 4;
    const int relu = (flags & PCONV_FLAG_RELU) ? 1 : 0;

    int kernel = tuning ? tuning->kernel : PCONV_KERNEL_AUTO;
    // Channel-minor activations and outputs: the matrix-core kernel only (fp16 storage, C and F multiples of 8,
    // buffers aligned to 16 bytes, a layer without channel lists).
    const bool nhwc = (flags & PCONV_FLAG_NHWC) != 0;
    if (nhwc) {
        if (wp->dtype != PCONV_F16 || wp->C % 8 || wp->F % 8 || wp->mfma.empty()) return PCONV_EUNSUPPORTED;
        if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) % 16) return PCONV_EUNSUPPORTED;
        if (kernel != PCONV_KERNEL_AUTO && kernel != PCONV_KERNEL_MFMA) return PCONV_EUNSUPPORTED;
        kernel = PCONV_KERNEL_MFMA;
    }
    int R = tuning ? tuning->rows : 0, NF = tuning ? tuning->filters_per_wave : 0, waves = tuning ? tuning->waves : 0;
    int CPW = tuning ? tuning->channels_per_wave : 0;
    int KS = tuning ? tuning->channel_splits : 0;
    int buffers = tuning ? tuning->buffers : 0;
    // The matrix-core kernel (fp16 storage): the layer as a dense contraction over its masked weights.  Automatic
    // choice: the tile shape with the smallest estimated time, if that is below an estimate for the vector kernels
    // (effective multiply-adds at the rate they reach on such a layer plus a fixed part: measured 20 TMAC/s at unit
    // stride, half of that on maps narrower than 14 columns, 5 TMAC/s at stride 2).  Layers with few output tiles
    // (batch 1, small maps with many channels) stay with the vector kernels, whose channel split fills the GPU.
    const bool all_auto = !tuning || (tuning->rows == 0 && tuning->filters_per_wave == 0 && tuning->waves == 0 &&
                                      tuning->channels_per_wave == 0 && tuning->channel_order == 0 &&
                                      tuning->channel_splits == 0 && tuning->buffers == 0 && tuning->split_reduce == 0);
    if (kernel == PCONV_KERNEL_MFMA || (kernel == PCONV_KERNEL_AUTO && wp->dtype == PCONV_F16 && all_auto)) {
        const bool forced = kernel == PCONV_KERNEL_MFMA;
        if (wp->dtype != PCONV_F16) return PCONV_EUNSUPPORTED;
        MfmaConv a{};
        a.x = x; a.y = y; a.bias = bias;
        a.N = N; a.C = wp->C; a.F = wp->F; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo;
        a.stride = stride; a.pad = pad; a.relu = relu;
        a.nhwc = nhwc ? 1 : 0;
        a.shape = tuning ? tuning->mfma_shape : 0;
        a.rows = tuning ? tuning->rows : 0;
        a.walk = tuning ? tuning->slot_walk : 0;
        if (a.shape < 0 || a.shape > kMfmaShapes) return PCONV_EINVAL;
        // (a layer of 1x1 kernels: its one tap is the centre of a 3x3 kernel at padding 1, which is tap 0 of a kernel
        // of extent 1 at padding 0 -- the same outputs, and no halo rows and columns to stage; and the copy of its
        // weights with channel ranges in the place of taps, if the layer has one: a quarter of the blocks, each four
        // times as deep.  Both for maps of at most 1024 pixels (and for channel-minor tensors): the 56 x 56 layers of
        // ResNet-50, channel-major, whose 8-pixel loads and four-row tiles are fine as they are, lost a tenth)
        a.groups = 1;
        a.kext = 3;
        if (wp->is_1x1 && pad == 1 && ((long long)H * W <= 1024 || nhwc)) {
            a.kext = 1;
            a.pad = 0;
            // (at stride 1 a 1x1 layer does not know rows from columns: an image's H*W pixels, contiguous in either
            // layout, are cut into rows of whatever length suits the kernel -- a multiple of 8 pixels for the widest
            // loads where H*W has such a divisor, and rows that fill a tile of 224 pixels)
            if (stride == 1) {
                const long long hw = (long long)H * W;
                long long best_w = W;
                int best_lw = 0, best_fill = 0;
                for (int w2 = 1; w2 <= 224 && w2 <= hw; ++w2) {
                    if (hw % w2) continue;
                    const int lw2 = w2 % 8 == 0 ? 8 : w2 % 4 == 0 ? 4 : w2 % 2 == 0 ? 2 : 1;
                    const int fill = (224 / w2) * w2;
                    if (lw2 > best_lw || (lw2 == best_lw && fill >= best_fill)) {
                        best_lw = lw2; best_fill = fill; best_w = w2;
                    }
                }
                // (rows that are as good as they are stay: 56 x 56 maps measured a tenth slower as 14 rows of 224)
                const int lw0 = W % 8 == 0 ? 8 : W % 4 == 0 ? 4 : W % 2 == 0 ? 2 : 1;
                if (W <= 224 && lw0 == best_lw && (224 / W) * W == best_fill) best_w = W;
                a.W = a.Wo = (int)best_w;
                a.H = a.Ho = (int)(hw / best_w);
            }
        }
        if (wp->is_1x1 && a.kext == 1 && (long long)H * W <= 1024)
            for (const MfmaWeights& m : wp->mfma)
                if (m.groups > 1) a.groups = m.groups;
        for (const MfmaWeights& m : wp->mfma)
            if (m.groups == a.groups) {
                a.n_taps = m.n_taps;
                break;
            }
        // tile shape and number of workgroups per tile (each with a part of the channel blocks), where not given
        double best_us = -1.0;
        const int want_shape = a.shape, want_splits = tuning ? tuning->channel_splits : 0;
        const int want_reduce = tuning ? tuning->split_reduce : 0;
        int best_sp = 0;
        if (want_splits < 0 || want_reduce < 0 || want_reduce > 2) return PCONV_EINVAL;
        for (int sh = 1; sh <= kMfmaShapes; ++sh) {
            if (want_shape && sh != want_shape) continue;
            // (A split pays where a layer has fewer tiles than compute units and many channel blocks in sequence --
            // ResNet-50's 512 -> 512 layers at batch 32: 83 -> 55 us in two parts at 14x14 stride 2, 69 -> 40 us in
            // four at 7x7 -- and costs the round trip of MT x NT floats per part otherwise: the 64 -> 64 layer at
            // 56x56 goes from 17 to 53 us in two parts.  The estimate carries both.  Not asked for, the choice is
            // between 1, 2 and, at stride 1, 4 parts: more lost on every shape measured.)
            for (int ks = 1; ks <= 16; ks *= 2)
                for (int sp = 0; sp <= (ks > 1 ? 1 : 0); ++sp) {
                    // sp = 1: the parts are added by a second kernel, which lets more of them pay: up to 8 (layers
                    // of one or two taps, whose blocks are too short to hide their loads: 16); added by the last
                    // arriver: 2 or, at stride 1, 4
                    if (want_reduce && ks > 1 && sp != want_reduce - 1) continue;
                    const int most = a.n_taps <= 2 ? 16 : sp ? 8 : stride == 2 ? 2 : 4;
                    if (want_splits ? ks != want_splits : ks > most) continue;
                    // (the weights kept for this shape's tile height say whether its tiles have channel lists)
                    for (const MfmaWeights& m : wp->mfma)
                        if (m.mt == mfma_shape_height(sh) && m.groups == a.groups) {
                            a.d_clist = m.d_clist; a.d_tinfo = m.d_tinfo;
                            a.min_blocks = m.min_blocks; a.total_blocks = m.total_blocks;
                        }
                    a.second_pass = sp;
                    const double t = mfma_estimate_us(a, sh, ks);
                    if (t >= 0.0 && (best_us < 0.0 || t < best_us)) {
                        best_us = t; a.shape = sh; a.splits = ks; best_sp = sp;
                    }
                }
        }
        a.second_pass = best_sp;
        if (best_us < 0.0) {
            a.shape = want_shape;                // (nothing fits: launch_mfma_conv says so)
            a.splits = want_splits ? want_splits : 1;
            a.second_pass = want_reduce == 2 ? 1 : 0;
        }
        bool take = best_us >= 0.0 || forced;
        if (take && !forced) {
            // (an entry of a 1x1 layer is one tap with the loop overhead of four: measured 3.1 entries per nanosecond
            // against 5 for the 3x3 layers the rate below is quoted for)
            const double macs = (double)N * Ho * Wo * (wp->is_1x1 ? 6.4 : 4.0) * (double)wp->n_kept;
            const double rate = stride == 2 ? 5e6 : Wo < 14 ? 10e6 : 20e6;      // multiply-adds per microsecond
            take = best_us < macs / rate + 8.0;
        }
        if (take && plan && best_us >= 0.0) {
            plan->kernel = PCONV_KERNEL_MFMA;
            plan->mfma_shape = a.shape;
            return PCONV_OK;
        }
        int rc = PCONV_EUNSUPPORTED;
        if (take)
            for (const MfmaWeights& m : wp->mfma) {
                if (!m.d_w || m.mt != mfma_shape_height(a.shape) || m.groups != a.groups) continue;
                a.d_w = m.d_w; a.mt = m.mt; a.n_taps = m.n_taps;
                a.d_clist = m.d_clist; a.d_tinfo = m.d_tinfo;
                a.min_blocks = m.min_blocks; a.total_blocks = m.total_blocks; a.w_bytes = m.bytes();
                std::memcpy(a.taps, m.taps, sizeof(a.taps));
                if (a.kext == 1) std::memset(a.taps, 0, sizeof(a.taps));
                if (a.splits > 1) {
                    size_t floats = 0, counters = 0;
                    rc = mfma_workspace(a, &floats, &counters);
                    if (rc == PCONV_OK) rc = get_workspace(wp, arena, floats, counters, &a.ws, &a.counters, st);
                    // (a split that the library chose itself and whose partial sums do not fit the fixed array of
                    // the entry point that allocates nothing: the same tile shape, unsplit)
                    if (rc == PCONV_ESCRATCH && !want_splits) {
                        a.splits = 1;
                        a.second_pass = 0;
                        a.ws = nullptr;
                        a.counters = nullptr;
                        rc = PCONV_OK;
                    }
                    if (rc != PCONV_OK) break;
                }
                rc = launch_mfma_conv(a, stream);
            }
        if (rc != PCONV_EUNSUPPORTED || forced) return rc;
        // (no tile shape takes the layer, or the vector kernels are expected to be faster: go on below)
    }
    // What the tiled kernel sees: the layer itself at stride 1; at stride 2 the layer re-packed over the four
    // row/column parity planes of the input (a stride-1 problem with 4*C channels of half the height and width).
    const int tH = stride == 1 ? H : (H + 1) / 2, tW = stride == 1 ? W : (W + 1) / 2;
    const int tC = stride == 1 ? wp->C : 4 * wp->C;
    const bool can_tile = tC < 65536 && tiled_applicable(N, tC, tH, tW, 1, esize);
    const bool automatic = waves == 0 && NF == 0 && CPW == 0;
    if (kernel == PCONV_KERNEL_AUTO && automatic && KS == 0 && buffers == 0) {
        // The kernel with four columns per lane has no channel split: it is the faster one (measured on the VGG-16
        // and ResNet-50 layer shapes at batch 32 and 64) once its own workgroups nearly fill the 256 CUs.
        long long wgs = 0;
        if (reinterpret_cast<uintptr_t>(x) % 4 == 0 && quad_applicable(N, wp->C, wp->F, H, W, Ho, stride, esize, &wgs)) {
            // tiles (slots) of the layer, and the workgroups that would walk over them (two filters per wave with
            // fp16 storage, one with fp32: see launch_quad)
            const int walk_nf = wp->dtype == PCONV_F16 ? 2 : 1;
            const long long slots = wgs / ((wp->F + 31) / 32);
            const int cus = compute_units();
            const long long nearly_full = (long long)cus * 25 / 32;       // 200 of 256: measured break-even
            const long long walkers = std::max(1, cus / ((wp->F + 16 * walk_nf - 1) / (16 * walk_nf)));
            if (wp->n_buckets == 1 && pad == 1 && reinterpret_cast<uintptr_t>(y) % 16 == 0 && 2 * slots >= 3 * walkers) {
                // one chunk of channels (a network's first layer) and more tiles than CUs: workgroups that keep their
                // filters and walk over the tiles (launch_quad turns to them under the same condition); measured
                // 13 to 32 % faster than one workgroup per tile at batch 4 to 64
                kernel = PCONV_KERNEL_QUAD;
                NF = walk_nf;
            } else if (wgs >= nearly_full) {
                kernel = PCONV_KERNEL_QUAD;
                NF = 2;
            } else if (wp->C <= 16 && wgs * ((wp->F + 15) / 16) / ((wp->F + 31) / 32) >= nearly_full) {
                // a single chunk of channels (a network's first layer): nothing to amortise over two filters per
                // wave, and one filter per wave gives twice the workgroups
                kernel = PCONV_KERNEL_QUAD;
                NF = 1;
            }
        }
    }
    if (kernel == PCONV_KERNEL_AUTO) kernel = can_tile ? PCONV_KERNEL_TILED : PCONV_KERNEL_GENERIC;
    if (kernel == PCONV_KERNEL_TILED && !can_tile) return PCONV_EUNSUPPORTED;
    if (plan) {
        plan->kernel = kernel;
        plan->mfma_shape = 0;
        return PCONV_OK;
    }
    const pconv_packed* lay = wp;
    const void* tx = x;
    // Stride 2 with even H and W: the kernels with paired staging read the parity planes straight from x (16 waves,
    // two channels per wave, channels in their own order).  Otherwise the input is split into planes by a pass of
    // its own first.
    const int order = tuning ? tuning->channel_order : PCONV_ORDER_AUTO;
    // (two-element loads: x must be aligned to two elements)
    const bool pair = kernel == PCONV_KERNEL_TILED && stride == 2 && H % 2 == 0 && W % 2 == 0 &&
                      reinterpret_cast<uintptr_t>(x) % (2 * esize) == 0 &&
                      order != PCONV_ORDER_BALANCED && buffers <= 1 &&
                      (automatic || (waves == 16 && (CPW == 0 || CPW == 2)));
    if (kernel == PCONV_KERNEL_TILED && stride == 2) {
        if (!wp->by_parity[pad]) {
            if (arena) return PCONV_ESTATE;   // re-packing the layer over parity planes allocates and uploads
            pconv_packed* child = nullptr;
            if (int rc = derive_for_stride2(wp, pad, true, &child)) return rc;
            wp->by_parity[pad] = child;
        }
        lay = wp->by_parity[pad];
    }
    if (kernel == PCONV_KERNEL_TILED && stride == 2 && !pair) {
        const size_t need = (size_t)N * tC * tH * tW * esize;
        if (need > wp->planes_bytes && arena) return PCONV_ESCRATCH;
        if (need > wp->planes_bytes) {
            if (wp->d_planes) PCONV_HIP(hipFree(wp->d_planes));   // hipFree waits for work that may still use it
            wp->d_planes = nullptr;
            wp->planes_bytes = 0;
            PCONV_HIP(hipMalloc(&wp->d_planes, need));
            wp->planes_bytes = need;
        }
        const dim3 grid((unsigned)((long long)N * wp->C), (unsigned)((tH + 3) / 4));
        if (wp->dtype == PCONV_F16)
            hipLaunchKernelGGL(parity_planes_kernel<__half>, grid, dim3(256), 0, st, (const __half*)x,
                               (__half*)wp->d_planes, H, W, tH, tW);
        else
            hipLaunchKernelGGL(parity_planes_kernel<float>, grid, dim3(256), 0, st, (const float*)x,
                               (float*)wp->d_planes, H, W, tH, tW);
        PCONV_HIP(hipGetLastError());
        tx = wp->d_planes;
    }

    if (kernel == PCONV_KERNEL_TILED) {
        if (R == 0) R = kR;
        if (R != kR) return PCONV_EUNSUPPORTED;
        if (automatic) {
            // Automatic tiling: the candidate with the smallest estimated time.  The estimate is a count of clocks
            // per workgroup from measured phase costs of this kernel on MI355X (one workgroup per CU at a time):
            // a fixed start-up, per chunk the larger of multiply-add issue and the global-load rate of the staging
            // plus the LDS write and barriers, and the cost of combining partial sums when channels are split.
            const int ncs = (Wo + 61) / 62, ows = (Wo + ncs - 1) / ncs;
            const int segs_per_wave = 64 / (ows + 2);
            const long long nseg = (long long)N * ((Ho + kR - 1) / kR) * ((Wo + ows - 1) / ows);
            const long long slots = (nseg + segs_per_wave - 1) / segs_per_wave;
            static const int cand[4][3] = {{2, 16, 2}, {1, 16, 2}, {1, 8, 4}, {2, 16, 1}};   // NF, waves, CPW
            double best = 0.0;
            for (int i = 0; i < 4; ++i) {
                const int nf = cand[i][0], w = cand[i][1], cpw = cand[i][2], cc = w * cpw;
                if (pair && (w != 16 || cpw != 2)) continue;   // the paired staging is built for this tiling
                if (cc == 16 && lay->C > 16) continue;   // half-size chunks only pay for layers with few channels
                const long long tiles = slots * ((lay->F + nf * w - 1) / (nf * w));
                const int nch = (lay->C + cc - 1) / cc;
                const double per_filter_chunk = (double)lay->n_kept / ((double)lay->F * nch);
                for (int ks = 1; ks <= std::min(nch, 16); ks *= 2) {
                    // (the workspace of one split is addressed with 32-bit byte offsets)
                    if (ks > 1 && (unsigned long long)tiles * w * nf * 2048 >= kInvalidOffset) break;
                    const double issue = (w / 4) * nf * per_filter_chunk * 128.0 + 750.0;
                    const double staging = std::min(lay->C, cc) * 9.0 * 18.0 * (pair ? 0.5 : 1.0);
                    const double chunk = std::max(issue, staging) + 3400.0;
                    const double combine = ks == 1 ? 1500.0 * nf : nf == 1 ? 1200.0 * ks : 4500.0 + 2400.0 * ks;
                    const double wg = 9000.0 + (double)((nch + ks - 1) / ks) * chunk + combine;
                    const double rounds = (double)((tiles * ks + compute_units() - 1) / compute_units());
                    const double t = rounds * wg;
                    if (best == 0.0 || t < best) { best = t; NF = nf; waves = w; CPW = cpw; KS = ks; }
                }
            }
        }
        if (KS < 0 || buffers < 0 || buffers > 2) return PCONV_EINVAL;
        if (buffers == 0) buffers = 1;
        if (waves == 0) waves = 8;
        if (NF == 0) NF = 1;
        if (CPW == 0) CPW = waves >= 16 ? 2 : 32 / waves;
        if (waves < 1 || waves > 16) return PCONV_EUNSUPPORTED;
        TiledParams p{};
        p.x = tx;
        p.y = y;
        p.ent = lay->d_ent;
        p.eptr = lay->d_eptr;
        p.forder = lay->d_forder;
        p.bias = bias;
        p.N = N;
        p.C = lay->C;
        p.F = lay->F;
        p.H = tH;
        p.W = tW;
        p.Ho = Ho;
        p.Wo = Wo;
        p.pad = pad;
        p.relu = relu;
        p.nbk = lay->n_buckets;
        p.bpc = (CPW * waves) / kBucket;
        p.perm = nullptr;
        p.perm_stride = 0;
        p.pair = pair ? 1 : 0;
        // a balanced layout exists for the tilings of the automatic choice
        if (order != PCONV_ORDER_PLAIN && !pair) {
            for (const BalancedLayout& b : lay->balanced)
                if (b.fw == waves && b.nf == NF && b.cc == CPW * waves && b.d_ent) {
                    p.ent = b.d_ent;
                    p.eptr = b.d_eptr;
                    p.perm = b.d_perm;
                    p.perm_stride = b.n_chunks * b.cc;
                    p.nbk = b.n_chunks;
                    p.bpc = 1;
                }
            if (order == PCONV_ORDER_BALANCED && !p.perm) return PCONV_EUNSUPPORTED;
        }
        p.x_bytes = (unsigned long long)N * lay->C * tH * tW * esize;
        p.img_bytes = (unsigned)((size_t)lay->C * tH * tW * esize);
        p.plane_bytes = (unsigned)((size_t)tH * tW * esize);
        return lay->dtype == PCONV_F16 ? launch_tiled<__half>(p, lay, NF, waves, CPW, KS, buffers, st, arena)
                                      : launch_tiled<float>(p, lay, NF, waves, CPW, KS, buffers, st, arena);
    }
    if (kernel == PCONV_KERNEL_QUAD) {
        if (stride != 1) return PCONV_EUNSUPPORTED;
        if (reinterpret_cast<uintptr_t>(x) % 4 != 0) return PCONV_EUNSUPPORTED;   // four-element loads, dword-aligned
        if ((unsigned long long)wp->C * H * W * esize >= 0x7FFFFFFFull) return PCONV_EUNSUPPORTED;
        QuadParams p{};
        p.x = x;
        p.y = y;
        p.ent = wp->d_ent;
        p.eptr = wp->d_eptr;
        p.forder = wp->d_forder;
        p.bias = bias;
        p.N = N;
        p.C = wp->C;
        p.F = wp->F;
        p.H = H;
        p.W = W;
        p.Ho = Ho;
        p.Wo = Wo;
        p.pad = pad;
        p.relu = relu;
        p.nbk = wp->n_buckets;
        p.perm = nullptr;
        p.perm_stride = 0;
        const int nf = NF == 0 ? 2 : NF;
        const int fw = waves == 0 ? 16 : waves;
        if (nf != 1 && nf != 2) return PCONV_EUNSUPPORTED;
        if (KS < 0) return PCONV_EINVAL;       // (0: launch_quad decides)
        if (order != PCONV_ORDER_PLAIN) {
            for (const BalancedLayout& b : wp->balanced)
                if (b.fw == fw && b.nf == nf && b.cc == fw && b.d_ent) {
                    p.ent = b.d_ent;
                    p.eptr = b.d_eptr;
                    p.perm = b.d_perm;
                    p.perm_stride = b.n_chunks * b.cc;
                    p.nbk = b.n_chunks;
                }
            if (order == PCONV_ORDER_BALANCED && !p.perm) return PCONV_EUNSUPPORTED;
        }
        if (fw != 16 && !p.perm) return PCONV_EUNSUPPORTED;   // the canonical entries come in chunks of 16 channels
        if ((unsigned long long)wp->n_kept * sizeof(DevEntry) >= kInvalidOffset) return PCONV_EUNSUPPORTED;
        p.ent_bytes = (unsigned)((size_t)wp->n_kept * sizeof(DevEntry));
        p.x_bytes = (unsigned long long)N * wp->C * H * W * esize;
        p.img_bytes = (unsigned)((size_t)wp->C * H * W * esize);
        p.plane_bytes = (unsigned)((size_t)H * W * esize);
        const int walk = tuning ? tuning->slot_walk : 0;
        return wp->dtype == PCONV_F16 ? launch_quad<__half>(p, wp, nf, fw, KS, walk, st, arena)
                                      : launch_quad<float>(p, wp, nf, fw, KS, walk, st, arena);
    }
    if (kernel != PCONV_KERNEL_GENERIC) return PCONV_EINVAL;
    const dim3 grid((unsigned)(((long long)Ho * Wo + 255) / 256), (unsigned)wp->F, (unsigned)N);
    if (wp->dtype == PCONV_F16)
        hipLaunchKernelGGL(generic_kernel<__half>, grid, dim3(256), 0, st, (const __half*)x, (__half*)y, wp->d_ent,
                           wp->d_eptr, wp->d_forder, bias, wp->C, wp->F, H, W, Ho, Wo, stride, pad, wp->n_buckets, relu);
    else
        hipLaunchKernelGGL(generic_kernel<float>, grid, dim3(256), 0, st, (const float*)x, (float*)y, wp->d_ent,
                           wp->d_eptr, wp->d_forder, bias, wp->C, wp->F, H, W, Ho, Wo, stride, pad, wp->n_buckets, relu);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

extern "C" int pconv_conv3x3_tuned(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H,
                                   int W, int stride, int pad, unsigned flags, void* stream,
                                   const pconv_tuning* tuning) {
    return conv3x3_impl(x, y, wp, bias, N, H, W, stride, pad, flags, stream, tuning, nullptr);
}

extern "C" int pconv_conv3x3(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H, int W,
                             int stride, int pad, unsigned flags, void* stream) {
    return conv3x3_impl(x, y, wp, bias, N, H, W, stride, pad, flags, stream, nullptr, nullptr);
}

// A 1x1 layer packed by pconv_pack_1x1 is a 3x3 layer of centre taps: at padding 1 its output is the 1x1 layer's.
extern "C" int pconv_conv1x1(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H, int W,
                             int stride, unsigned flags, void* stream) {
    if (!wp) return PCONV_EINVAL;
    if (!wp->is_1x1) return PCONV_ESTATE;
    return conv3x3_impl(x, y, wp, bias, N, H, W, stride, 1, flags, stream, nullptr, nullptr);
}

// The input gradient of a layer at stride 1 and padding 1 is the forward pass of its transposed layer over dy.
extern "C" int pconv_conv3x3_grad_input(const void* dy, void* dx, const pconv_packed* wpt, int N, int H, int W,
                                        void* stream) {
    return conv3x3_impl(dy, dx, wpt, nullptr, N, H, W, 1, 1, 0, stream, nullptr, nullptr);
}

extern "C" int pconv_conv3x3_noalloc(const void* x, void* y, const pconv_packed* wp, const float* bias, int N, int H,
                                     int W, int stride, int pad, unsigned flags, void* stream) {
    WsArena arena{};
    if (int rc = current_arena(&arena)) return rc;
    return conv3x3_impl(x, y, wp, bias, N, H, W, stride, pad, flags, stream, nullptr, &arena);
}

extern "C" size_t pconv_noalloc_scratch_bytes(void) { return kArenaBytes; }

extern "C" int pconv_conv3x3_choice(const pconv_packed* wp, int N, int H, int W, int stride, int pad, int* kernel,
                                    int* mfma_shape) {
    PlanOut out{0, 0};
    // (pointers that are aligned as device allocations are; nothing is read through them)
    void* const aligned = reinterpret_cast<void*>(static_cast<uintptr_t>(4096));
    const int rc = conv3x3_impl(aligned, aligned, wp, nullptr, N, H, W, stride, pad, 0, nullptr, nullptr, nullptr, &out);
    if (rc != PCONV_OK) return rc;
    if (kernel) *kernel = out.kernel;
    if (mfma_shape) *mfma_shape = out.mfma_shape;
    return PCONV_OK;
}

extern "C" int pconv_dense_conv3x3(const void* x, void* y, const void* w, const float* bias, int dtype, int N, int C,
                                   int F, int H, int W, int stride, int pad, unsigned flags, void* stream) {
    if (!w) return PCONV_EINVAL;
    if (dtype != PCONV_F32 && dtype != PCONV_F16) return PCONV_EINVAL;
    int Ho = 0, Wo = 0;
    if (int rc = check_conv_args(x, y, N, C, F, H, W, stride, pad, flags & ~(unsigned)PCONV_FLAG_DENSE_DIRECT, &Ho, &Wo))
        return rc;
    if (N == 0) return PCONV_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int relu = (flags & PCONV_FLAG_RELU) ? 1 : 0;
    if (dtype == PCONV_F16 && !(flags & PCONV_FLAG_DENSE_DIRECT)) {
        // the matrix-core kernel on all nine taps of all kernels; the weights are brought into its order by a small
        // kernel first (part of the call), in a buffer that the library keeps per device and grows on demand
        MfmaConv a{};
        a.x = x; a.y = y; a.bias = bias; a.n_taps = 9;
        for (int t = 0; t < 9; ++t) a.taps[t] = (uint8_t)t;
        a.N = N; a.C = C; a.F = F; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo;
        a.stride = stride; a.pad = pad; a.relu = relu;
        double best_us = -1.0;
        for (int sh = 1; sh <= kMfmaShapes; ++sh) {
            const double t = mfma_estimate_us(a, sh, 1);
            if (t >= 0.0 && (best_us < 0.0 || t < best_us)) { best_us = t; a.shape = sh; }
        }
        a.splits = 1;
        const int mt = a.shape ? mfma_shape_height(a.shape) : 128;
        const size_t need = mfma_weight_bytes(F, C, mt, 9);
        void* buf = nullptr;
        if (int rc = dense_weight_buffer(need, &buf)) return rc;
        if (int rc = launch_mfma_arrange(w, buf, F, C, mt, stream)) return rc;
        a.d_w = buf; a.mt = mt;
        const int rc = a.shape ? launch_mfma_conv(a, stream) : PCONV_EUNSUPPORTED;
        if (rc != PCONV_EUNSUPPORTED) return rc;
    }
    const dim3 grid((unsigned)(((long long)Ho * Wo + 255) / 256), (unsigned)F, (unsigned)N);
    if (dtype == PCONV_F16)
        hipLaunchKernelGGL(dense_kernel<__half>, grid, dim3(256), 0, st, (const __half*)x, (__half*)y, (const __half*)w,
                           bias, C, F, H, W, Ho, Wo, stride, pad, relu);
    else
        hipLaunchKernelGGL(dense_kernel<float>, grid, dim3(256), 0, st, (const float*)x, (float*)y, (const float*)w,
                           bias, C, F, H, W, Ho, Wo, stride, pad, relu);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

extern "C" int pconv_maxpool2x2(const void* x, void* y, int dtype, int N, int C, int H, int W, void* stream) {
    if (!x || !y) return PCONV_EINVAL;
    if (dtype != PCONV_F32 && dtype != PCONV_F16) return PCONV_EINVAL;
    if (N < 0 || C <= 0 || H < 2 || W < 2) return PCONV_ESHAPE;
    if (N == 0) return PCONV_OK;
    const long long planes = (long long)N * C;
    const long long total = planes * (H / 2) * (W / 2);
    const unsigned grid = (unsigned)std::min<long long>((total + 255) / 256, 1 << 20);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == PCONV_F16)
        hipLaunchKernelGGL(maxpool_kernel<__half>, dim3(grid), dim3(256), 0, st, (const __half*)x, (__half*)y, planes, H, W);
    else
        hipLaunchKernelGGL(maxpool_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)x, (float*)y, planes, H, W);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}
