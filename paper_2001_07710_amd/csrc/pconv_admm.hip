// The selection-variable steps of the pruning framework (paper, section 5.1) and the pattern assignment (sections
// 4.1, 5.1) as device kernels: one thread per 3x3 kernel, everything in registers, bound by HBM.  Declared in
// include/pconv_admm.h.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <hipcub/device/device_radix_sort.hpp>

#include <cmath>
#include <cstdint>

#include "pconv_admm.h"
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

constexpr int kThreads = 256;

int grid_for(long long n) {
    return (int)((n + kThreads - 1) / kThreads);
}

// One thread, one kernel's vectors.  KMAX is K rounded up to 4, 8, 16 or 32: the vector lives in registers, entries
// from K on are minus infinity, which sorts behind everything and adds nothing to any sum that is used.
// WHOLE: K == KMAX and all four buffers are 16-byte aligned, so a vector is KMAX/4 128-bit accesses.
typedef float float4v __attribute__((ext_vector_type(4)));
template <int KMAX, bool WHOLE>
__global__ __launch_bounds__(kThreads) void proximal_kernel(const float* __restrict__ z, const float* __restrict__ mu,
                                                            double rho, long long n, int K, float* __restrict__ u,
                                                            float* mu_out) {
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const float* zi = z + i * K;
    float zf[KMAX], mf[KMAX];
    if constexpr (WHOLE) {
#pragma unroll
        for (int q = 0; q < KMAX / 4; ++q) {
            const float4v a = reinterpret_cast<const float4v*>(zi)[q];
            const float4v b = mu ? reinterpret_cast<const float4v*>(mu + i * K)[q] : float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                zf[4 * q + e] = a[e];
                mf[4 * q + e] = b[e];
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
            zf[j] = j < K ? zi[j] : 0.f;
            mf[j] = (j < K && mu) ? mu[i * K + j] : 0.f;
        }
    }
    double zv[KMAX], mv[KMAX], d[KMAX], s[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        zv[j] = (double)zf[j];
        mv[j] = (double)mf[j];
        d[j] = j < K ? zv[j] + mv[j] / rho : -INFINITY;
        s[j] = d[j];
    }
    // breakpoints, largest first (an odd-even transposition network: KMAX rounds of compare-exchanges on registers)
#pragma unroll
    for (int round = 0; round < KMAX; ++round)
#pragma unroll
        for (int j = round & 1; j + 1 < KMAX; j += 2) {
            const double a = s[j], b = s[j + 1];
            const bool swap = b > a;
            s[j] = swap ? b : a;
            s[j + 1] = swap ? a : b;
        }
    // the root of 1^T [d - nu 1]_+ = 1: with exactly the m largest entries above it, nu = (their sum - 1) / m, and it
    // is the root if it lies in [s[m], s[m-1])
    double nu = 0.0, total = 0.0;
    bool found = false;
#pragma unroll
    for (int m = 1; m <= KMAX; ++m) {
        total += s[m - 1];
        const double cand = (total - 1.0) / (double)m;
        const double lower = (m < KMAX && m < K) ? s[m] : -INFINITY;
        if (!found && m <= K && cand < s[m - 1] && cand >= lower) {
            nu = cand;
            found = true;
        }
    }
    float uf[KMAX], nf[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        const double uj = fmax(d[j] - nu, 0.0);
        uf[j] = (float)uj;
        nf[j] = (float)(mv[j] + rho * (zv[j] - uj));
    }
    if constexpr (WHOLE) {
#pragma unroll
        for (int q = 0; q < KMAX / 4; ++q) {
            if (u) reinterpret_cast<float4v*>(u + i * K)[q] = float4v{uf[4 * q], uf[4 * q + 1], uf[4 * q + 2], uf[4 * q + 3]};
            if (mu_out)
                reinterpret_cast<float4v*>(mu_out + i * K)[q] = float4v{nf[4 * q], nf[4 * q + 1], nf[4 * q + 2], nf[4 * q + 3]};
        }
    } else {
#pragma unroll
        for (int j = 0; j < KMAX; ++j)
            if (j < K) {
                if (u) u[i * K + j] = uf[j];
                if (mu_out) mu_out[i * K + j] = nf[j];
            }
    }
}

__global__ __launch_bounds__(kThreads) void binarize_kernel(const float* __restrict__ z, long long n, int K,
                                                            int32_t* __restrict__ pid) {
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const float* zi = z + i * K;
    float best = zi[0];
    int arg = 0;
    for (int j = 1; j < K; ++j) {
        const float v = zi[j];
        if (v > best) {          // (strictly: ties stay with the lowest index)
            best = v;
            arg = j;
        }
    }
    pid[i] = arg;
}

// K a multiple of 4 up to 32 and z 16-byte aligned: the vector in KQ 128-bit loads, all issued before the first use
template <int KQ>
__global__ __launch_bounds__(kThreads) void binarize_vec_kernel(const float4v* __restrict__ z, long long n,
                                                                int32_t* __restrict__ pid) {
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    float4v v[KQ];
#pragma unroll
    for (int q = 0; q < KQ; ++q) v[q] = z[i * KQ + q];
    float best = v[0][0];
    int arg = 0;
#pragma unroll
    for (int q = 0; q < KQ; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (v[q][e] > best) {
                best = v[q][e];
                arg = 4 * q + e;
            }
    pid[i] = arg;
}

struct Library {
    uint16_t mask[126];
};

// The 256 kernels of a block are 256 x 9 consecutive weights: loaded as one coalesced run (16 bytes per lane and
// load, whatever the storage type), parked in LDS, and read back 9 per thread (a stride of 9 words or 4.5 words
// touches every bank once per 64 lanes' worth of accesses).  Loading 9 weights per thread straight from memory makes
// every wave-wide load touch 36 cache lines.
template <typename T>
__global__ __launch_bounds__(kThreads) void assign_kernel(const T* __restrict__ w, long long n, Library lib, int K,
                                                          int32_t* __restrict__ pid) {
    __shared__ __attribute__((aligned(16))) T tile[kThreads * 9];
    // (the masks once into LDS: indexed by the loop counter straight from the kernel arguments they come as one
    // memory load per pattern, each waited for)
    __shared__ uint32_t masks[126];
    if ((int)threadIdx.x < K) masks[threadIdx.x] = lib.mask[threadIdx.x];
    const long long first = (long long)blockIdx.x * kThreads;             // first kernel of the block
    const int count = (int)(n - first < kThreads ? n - first : kThreads);  // kernels of the block
    const T* src = w + first * 9;
    constexpr int PER = 16 / (int)sizeof(T);                               // elements per 16-byte piece
    const bool aligned = (reinterpret_cast<uintptr_t>(src) & 15u) == 0;
    const int pieces = aligned ? count * 9 / PER : 0;
    for (int k = threadIdx.x; k < pieces; k += kThreads)
        reinterpret_cast<float4v*>(tile)[k] = reinterpret_cast<const float4v*>(src)[k];
    for (int k = pieces * PER + threadIdx.x; k < count * 9; k += kThreads) tile[k] = src[k];   // (tail, or all of it)
    __syncthreads();
    if ((int)threadIdx.x >= count) return;
    double sq[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const double v = (double)(float)tile[threadIdx.x * 9 + t];
        sq[t] = v * v;
    }
    double best = -1.0;
    int arg = 0;
    for (int j = 0; j < K; ++j) {
        // (the mask is the same for the whole wave: its bits become the factors 1.0 and 0.0 on the scalar unit, and a
        // tap is one fused multiply-add -- fma(sq, 1, e) is the rounded sum e + sq, fma(sq, 0, e) is e, so this is
        // the sum of the kept taps in ascending order, one rounding per kept tap, as the host entry computes it;
        // with a select per tap the kernel was bound by its own instructions at a third of the memory rate)
        const unsigned m = __builtin_amdgcn_readfirstlane(masks[j]);
        double e = 0.0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const double bit = __builtin_bit_cast(double, (m >> t & 1u) ? 0x3FF0000000000000ull : 0ull);
            e = __builtin_fma(sq[t], bit, e);
        }
        if (e > best) {
            best = e;
            arg = j;
        }
    }
    pid[first + threadIdx.x] = arg;
}

// squared norm of the pattern-pruned kernel as a sort key: a non-negative double's bit pattern orders like its value
template <typename T>
__global__ __launch_bounds__(kThreads) void norm_key_kernel(const T* __restrict__ w, long long n, Library lib, int K,
                                                            const int32_t* __restrict__ pid, uint64_t* __restrict__ key,
                                                            uint32_t* __restrict__ idx) {
    __shared__ uint32_t masks[126];
    if ((int)threadIdx.x < K) masks[threadIdx.x] = lib.mask[threadIdx.x];
    __syncthreads();
    const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    const int32_t j = pid[i];
    const unsigned m = masks[(j >= 0 && j < K) ? j : 0];
    double e = 0.0;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const double v = (double)(float)w[i * 9 + t];
        if (m >> t & 1u) e = e + v * v;                       // (taps ascending, product and sum rounded separately)
    }
    key[i] = __builtin_bit_cast(uint64_t, e);
    idx[i] = (uint32_t)i;
}

__global__ __launch_bounds__(kThreads) void mark_kept_kernel(const uint32_t* __restrict__ order, long long n, long long k,
                                                             uint8_t* __restrict__ mask) {
    const long long r = (long long)blockIdx.x * kThreads + threadIdx.x;
    if (r < n) mask[order[r]] = r < k ? 1 : 0;
}

size_t round256(size_t b) {
    return (b + 255) / 256 * 256;
}

}  // namespace
}  // namespace pconv

using namespace pconv;

extern "C" int pconv_select_connectivity_device(const void* w, int dtype, long long n, const uint16_t* lib, int K,
                                                const int32_t* pid, double keep, uint8_t* mask, void* workspace,
                                                size_t* workspace_bytes, void* stream) {
    if (!workspace_bytes || n < 0 || (dtype != PCONV_F32 && dtype != PCONV_F16)) return PCONV_EINVAL;
    if (n > 0x7FFFFFFFll) return PCONV_ESHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // workspace: keys in, keys out (8 bytes each), indices in, indices out (4 bytes each), the sort's own scratch
    size_t sort_bytes = 0;
    PCONV_HIP(hipcub::DeviceRadixSort::SortPairsDescending(nullptr, sort_bytes, (const uint64_t*)nullptr, (uint64_t*)nullptr,
                                                          (const uint32_t*)nullptr, (uint32_t*)nullptr, (int)n, 0, 64, st));
    const size_t kb = round256((size_t)n * 8), ib = round256((size_t)n * 4);
    const size_t need = 2 * kb + 2 * ib + round256(sort_bytes) + 256;
    if (!workspace) {
        *workspace_bytes = need;
        return PCONV_OK;
    }
    if (!w || !lib || !pid || !mask || !(keep >= 0.0 && keep <= 1.0)) return PCONV_EINVAL;
    if (K < 1 || K > 126) return PCONV_EPATTERN;
    Library l{};
    for (int j = 0; j < K; ++j) {
        if (lib[j] >= 512 || __builtin_popcount(lib[j]) != 4) return PCONV_EPATTERN;
        l.mask[j] = lib[j];
    }
    if (*workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return PCONV_ESCRATCH;
    if (n == 0) return PCONV_OK;
    long long k = (long long)std::floor(keep * (double)n + 0.5);
    k = k < 0 ? 0 : (k > n ? n : k);
    char* base = static_cast<char*>(workspace);
    uint64_t* key_in = reinterpret_cast<uint64_t*>(base);
    uint64_t* key_out = reinterpret_cast<uint64_t*>(base + kb);
    uint32_t* idx_in = reinterpret_cast<uint32_t*>(base + 2 * kb);
    uint32_t* idx_out = reinterpret_cast<uint32_t*>(base + 2 * kb + ib);
    void* sort_tmp = base + 2 * kb + 2 * ib;
    const dim3 grid(grid_for(n)), block(kThreads);
    if (dtype == PCONV_F32)
        hipLaunchKernelGGL(norm_key_kernel<float>, grid, block, 0, st, static_cast<const float*>(w), n, l, K, pid, key_in,
                           idx_in);
    else
        hipLaunchKernelGGL(norm_key_kernel<_Float16>, grid, block, 0, st, static_cast<const _Float16*>(w), n, l, K, pid,
                           key_in, idx_in);
    PCONV_HIP(hipGetLastError());
    // a stable sort, largest key first: equal norms stay in ascending index order
    PCONV_HIP(hipcub::DeviceRadixSort::SortPairsDescending(sort_tmp, sort_bytes, key_in, key_out, idx_in, idx_out, (int)n, 0,
                                                          64, st));
    hipLaunchKernelGGL(mark_kept_kernel, grid, block, 0, st, idx_out, n, k, mask);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

extern "C" int pconv_admm_proximal(const float* z, const float* mu, float rho, long long n, int K, float* u,
                                   float* mu_out, void* stream) {
    if (!z || K < 1 || K > 32 || n < 0 || !(rho > 0.0f) || std::isinf(rho)) return PCONV_EINVAL;
    if (n == 0 || (!u && !mu_out)) return PCONV_OK;
    if (n > 0x7FFFFFFFll * kThreads) return PCONV_ESHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(grid_for(n)), block(kThreads);
    const uintptr_t bits = reinterpret_cast<uintptr_t>(z) | reinterpret_cast<uintptr_t>(mu) | reinterpret_cast<uintptr_t>(u) |
                           reinterpret_cast<uintptr_t>(mu_out);
    const bool whole = (K == 4 || K == 8 || K == 16 || K == 32) && bits % 16 == 0;
#define PCONV_PROX(KM)                                                                                              \
    do {                                                                                                            \
        if (whole)                                                                                                  \
            hipLaunchKernelGGL((proximal_kernel<KM, true>), grid, block, 0, st, z, mu, (double)rho, n, K, u, mu_out);   \
        else                                                                                                        \
            hipLaunchKernelGGL((proximal_kernel<KM, false>), grid, block, 0, st, z, mu, (double)rho, n, K, u, mu_out);  \
    } while (0)
    if (K <= 4)
        PCONV_PROX(4);
    else if (K <= 8)
        PCONV_PROX(8);
    else if (K <= 16)
        PCONV_PROX(16);
    else
        PCONV_PROX(32);
#undef PCONV_PROX
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

extern "C" int pconv_admm_binarize(const float* z, long long n, int K, int32_t* pid, void* stream) {
    if (!z || !pid || K < 1 || K > 126 || n < 0) return PCONV_EINVAL;
    if (n == 0) return PCONV_OK;
    if (n > 0x7FFFFFFFll * kThreads) return PCONV_ESHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(grid_for(n)), block(kThreads);
    const float4v* zq = reinterpret_cast<const float4v*>(z);
    const bool vec = K % 4 == 0 && K <= 32 && reinterpret_cast<uintptr_t>(z) % 16 == 0;
    switch (vec ? K / 4 : 0) {
        case 1: hipLaunchKernelGGL(binarize_vec_kernel<1>, grid, block, 0, st, zq, n, pid); break;
        case 2: hipLaunchKernelGGL(binarize_vec_kernel<2>, grid, block, 0, st, zq, n, pid); break;
        case 3: hipLaunchKernelGGL(binarize_vec_kernel<3>, grid, block, 0, st, zq, n, pid); break;
        case 4: hipLaunchKernelGGL(binarize_vec_kernel<4>, grid, block, 0, st, zq, n, pid); break;
        case 5: hipLaunchKernelGGL(binarize_vec_kernel<5>, grid, block, 0, st, zq, n, pid); break;
        case 6: hipLaunchKernelGGL(binarize_vec_kernel<6>, grid, block, 0, st, zq, n, pid); break;
        case 7: hipLaunchKernelGGL(binarize_vec_kernel<7>, grid, block, 0, st, zq, n, pid); break;
        case 8: hipLaunchKernelGGL(binarize_vec_kernel<8>, grid, block, 0, st, zq, n, pid); break;
        default: hipLaunchKernelGGL(binarize_kernel, grid, block, 0, st, z, n, K, pid);
    }
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}

extern "C" int pconv_assign_patterns_device(const void* w, int dtype, long long n, const uint16_t* lib, int K,
                                            int32_t* pid, void* stream) {
    if (!w || !lib || !pid || n < 0 || (dtype != PCONV_F32 && dtype != PCONV_F16)) return PCONV_EINVAL;
    if (K < 1 || K > 126) return PCONV_EPATTERN;
    Library l{};
    for (int j = 0; j < K; ++j) {
        if (lib[j] >= 512 || __builtin_popcount(lib[j]) != 4) return PCONV_EPATTERN;
        l.mask[j] = lib[j];
    }
    if (n == 0) return PCONV_OK;
    if (n > 0x7FFFFFFFll * kThreads) return PCONV_ESHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == PCONV_F32)
        hipLaunchKernelGGL(assign_kernel<float>, dim3(grid_for(n)), dim3(kThreads), 0, st, static_cast<const float*>(w), n,
                           l, K, pid);
    else
        hipLaunchKernelGGL(assign_kernel<_Float16>, dim3(grid_for(n)), dim3(kThreads), 0, st,
                           static_cast<const _Float16*>(w), n, l, K, pid);
    PCONV_HIP(hipGetLastError());
    return PCONV_OK;
}
