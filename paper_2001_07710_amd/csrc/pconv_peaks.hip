// Measured peaks of the chip the library runs on (gfx950): small register-, LDS- and memory-only kernels that say
// what a resource delivers when nothing else is in the way.  Built into libpconv_peaks.so, apart from libpconv.so:
// nothing on the convolution path calls into this file.  `bench.py --peaks` prints the numbers; the design notes
// quote them as "measured on this chip".
//
// Every entry point runs its kernel on the current device's default stream between two HIP events and returns the
// figure it is named for, or a negative HIP error code.  Rates that are "per clock" use the engine clock the
// runtime reports (hipDeviceAttributeClockRate), i.e. the nominal peak clock, not the clock the chip happened to
// hold during the run.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef float float4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

#define PEAK_HIP(call)                       \
    do {                                     \
        hipError_t e_ = (call);              \
        if (e_ != hipSuccess) return -(double)(int)e_; \
    } while (0)

struct DeviceShape {
    int cus;
    double clock_hz;
};
int device_shape(DeviceShape* d) {
    int dev = 0, cus = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return -1;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess) return -1;
    d->cus = cus;
    d->clock_hz = khz * 1e3;
    return 0;
}

template <typename F>
double timed_ms(F launch) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.0;
    launch();                                     // warm-up
    (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0, 0);
    launch();
    (void)hipEventRecord(e1, 0);
    (void)hipEventSynchronize(e1);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return hipGetLastError() == hipSuccess ? (double)ms : -1.0;
}

// ---- device-to-device copy, 16 bytes per lane
__global__ __launch_bounds__(256) void copy_kernel(const float4v* __restrict__ src, float4v* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// ---- fp32 multiply-adds on registers only: 16 independent accumulators per lane
__global__ __launch_bounds__(1024) void fma_kernel(float* out, int iters) {
    float a[16];
    // (both operands per lane, in vector registers: a multiply-add with an operand in a scalar register or a literal
    // runs at half the rate on this chip)
    const float x = 1.0f + threadIdx.x * 1e-7f, y = 0.999f + threadIdx.x * 1e-8f;
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = (float)i;
    // (v_fmac_f32 spelled out: the three-address v_fma_f32 that the compiler picks for a[i] = fma(a[i], x, y)
    // reads three vector registers per lane and reaches two thirds of this rate)
    for (int it = 0; it < iters; ++it) {
        asm volatile(
            "v_fmac_f32 %0, %16, %17\n v_fmac_f32 %1, %16, %17\n v_fmac_f32 %2, %16, %17\n v_fmac_f32 %3, %16, %17\n"
            "v_fmac_f32 %4, %16, %17\n v_fmac_f32 %5, %16, %17\n v_fmac_f32 %6, %16, %17\n v_fmac_f32 %7, %16, %17\n"
            "v_fmac_f32 %8, %16, %17\n v_fmac_f32 %9, %16, %17\n v_fmac_f32 %10, %16, %17\n v_fmac_f32 %11, %16, %17\n"
            "v_fmac_f32 %12, %16, %17\n v_fmac_f32 %13, %16, %17\n v_fmac_f32 %14, %16, %17\n v_fmac_f32 %15, %16, %17"
            : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]), "+v"(a[8]),
              "+v"(a[9]), "+v"(a[10]), "+v"(a[11]), "+v"(a[12]), "+v"(a[13]), "+v"(a[14]), "+v"(a[15])
            : "v"(x), "v"(y));
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += a[i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- 128-bit LDS reads, neighbouring lanes read neighbouring 16-byte pieces (no bank conflicts)
__global__ __launch_bounds__(1024) void lds_kernel(float* out, int iters) {
    extern __shared__ __align__(16) float tile[];
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) tile[i] = (float)i;
    __syncthreads();
    const unsigned base = (threadIdx.x & 63) * 16;
    float s = 0.f;
    for (int it = 0; it < iters; ++it) {
        const unsigned a = base + (unsigned)(it & 7) * 6144u;
        float4v q0, q1, q2, q3, q4, q5, q6, q7;
        asm volatile(
            "ds_read_b128 %0, %8\n ds_read_b128 %1, %8 offset:1024\n ds_read_b128 %2, %8 offset:2048\n"
            "ds_read_b128 %3, %8 offset:3072\n ds_read_b128 %4, %8 offset:4096\n ds_read_b128 %5, %8 offset:5120\n"
            "ds_read_b128 %6, %8 offset:6144\n ds_read_b128 %7, %8 offset:7168\n s_waitcnt lgkmcnt(0)"
            : "=&v"(q0), "=&v"(q1), "=&v"(q2), "=&v"(q3), "=&v"(q4), "=&v"(q5), "=&v"(q6), "=&v"(q7)
            : "v"(a));
        s += q0.x + q7.y;
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- global loads that hit the same few cache lines over and over: what is left is the rate at which a compute
// unit takes load instructions (BYTES per lane: 4 or 16)
template <int BYTES>
__global__ __launch_bounds__(1024) void vmem_issue_kernel(const float* __restrict__ src, float* out, int iters) {
    const float* p = src + (threadIdx.x & 63) * (BYTES / 4);
    float s = 0.f;
    for (int it = 0; it < iters; ++it) {
        if (BYTES == 4) {
            float q0, q1, q2, q3;
            asm volatile(
                "global_load_dword %0, %4, off\n global_load_dword %1, %4, off offset:1024\n"
                "global_load_dword %2, %4, off offset:2048\n global_load_dword %3, %4, off offset:3072\n s_waitcnt vmcnt(0)"
                : "=&v"(q0), "=&v"(q1), "=&v"(q2), "=&v"(q3)
                : "v"(p)
                : "memory");
            s += q0 + q3;
        } else {
            float4v q0, q1, q2, q3;
            asm volatile(
                "global_load_dwordx4 %0, %4, off\n global_load_dwordx4 %1, %4, off offset:1024\n"
                "global_load_dwordx4 %2, %4, off offset:2048\n global_load_dwordx4 %3, %4, off offset:3072\n s_waitcnt vmcnt(0)"
                : "=&v"(q0), "=&v"(q1), "=&v"(q2), "=&v"(q3)
                : "v"(p)
                : "memory");
            s += q0.x + q3.y;
        }
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- global stores of 16 bytes per lane that hit the same few cache lines of the L2 over and over (every wave its
// own 4 KB): the rate at which a compute unit's store path takes wave-wide store instructions
__global__ __launch_bounds__(1024) void vmem_store_kernel(float* dst, int iters) {
    float* p = dst + ((size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * 1024 + (threadIdx.x & 63) * 4;
    const float4v v = {1.f, 2.f, 3.f, (float)threadIdx.x};
    for (int it = 0; it < iters; ++it)
        asm volatile(
            "global_store_dwordx4 %0, %1, off nt\n global_store_dwordx4 %0, %1, off offset:1024 nt\n"
            "global_store_dwordx4 %0, %1, off offset:2048 nt\n global_store_dwordx4 %0, %1, off offset:3072 nt"
            :
            : "v"(p), "v"(v)
            : "memory");
}

// ---- fp16 MFMA on registers only: four independent 32x32x16 accumulator tiles per wave
__global__ __launch_bounds__(512) void mfma_kernel(float* out, int iters) {
    half8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(threadIdx.x * 0.001f + e);
        b[e] = (_Float16)(e * 0.5f);
    }
    float16v c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

struct Scratch {
    float* p = nullptr;
    size_t bytes = 0;
    ~Scratch() {
        if (p) (void)hipFree(p);
    }
    bool get(size_t n) {
        if (hipMalloc((void**)&p, n) != hipSuccess) return false;
        bytes = n;
        return hipMemset(p, 0, n) == hipSuccess;
    }
};

}  // namespace

// Device copy bandwidth in GB/s, read + written bytes counted, `mib` MiB each way.
extern "C" double pconv_peak_copy_gbs(int mib) {
    if (mib < 1 || mib > 8192) return -1.0;
    DeviceShape d;
    if (device_shape(&d)) return -1.0;
    const size_t bytes = (size_t)mib << 20, n = bytes / 16;
    Scratch a, b;
    if (!a.get(bytes) || !b.get(bytes)) return -2.0;
    const double ms = timed_ms([&] {
        hipLaunchKernelGGL(copy_kernel, dim3(d.cus * 8), dim3(256), 0, 0, (const float4v*)a.p, (float4v*)b.p, n);
    });
    return ms <= 0.0 ? -3.0 : 2.0 * (double)bytes / (ms * 1e-3) / 1e9;
}

// fp32 vector multiply-add rate in TFLOP/s with `waves_per_simd` waves on every SIMD (1, 2 or 4).
extern "C" double pconv_peak_fma_tflops(int waves_per_simd) {
    if (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4) return -1.0;
    DeviceShape d;
    if (device_shape(&d)) return -1.0;
    const int threads = waves_per_simd * 4 * 64, iters = 20000;
    Scratch o;
    if (!o.get((size_t)d.cus * threads * 4)) return -2.0;
    const double ms = timed_ms([&] { hipLaunchKernelGGL(fma_kernel, dim3(d.cus), dim3(threads), 0, 0, o.p, iters); });
    return ms <= 0.0 ? -3.0 : 2.0 * 16.0 * iters * threads * (double)d.cus / (ms * 1e-3) / 1e12;
}

// 128-bit LDS reads: bytes per nominal clock and compute unit, `waves` waves per compute unit (4..16).
extern "C" double pconv_peak_lds_read_bytes_per_clk(int waves) {
    if (waves < 1 || waves > 16) return -1.0;
    DeviceShape d;
    if (device_shape(&d)) return -1.0;
    const int iters = 4000;
    Scratch o;
    if (!o.get((size_t)d.cus * waves * 64 * 4)) return -2.0;
    if (hipFuncSetAttribute((const void*)lds_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess) return -2.0;
    const double ms = timed_ms([&] { hipLaunchKernelGGL(lds_kernel, dim3(d.cus), dim3(waves * 64), 65536, 0, o.p, iters); });
    return ms <= 0.0 ? -3.0 : 8.0 * iters * waves * 1024.0 / (ms * 1e-3 * d.clock_hz);
}

// Nominal clocks a compute unit spends per wave-wide global load instruction that hits the cache, for loads of
// `bytes_per_lane` (4 or 16) bytes per lane, 16 waves per compute unit.
extern "C" double pconv_peak_vmem_clk_per_load(int bytes_per_lane) {
    if (bytes_per_lane != 4 && bytes_per_lane != 16) return -1.0;
    DeviceShape d;
    if (device_shape(&d)) return -1.0;
    const int iters = 4000, waves = 16;
    Scratch src, o;
    if (!src.get(1 << 16) || !o.get((size_t)d.cus * waves * 64 * 4)) return -2.0;
    const double ms = timed_ms([&] {
        if (bytes_per_lane == 4)
            hipLaunchKernelGGL(vmem_issue_kernel<4>, dim3(d.cus), dim3(waves * 64), 0, 0, src.p, o.p, iters);
        else
            hipLaunchKernelGGL(vmem_issue_kernel<16>, dim3(d.cus), dim3(waves * 64), 0, 0, src.p, o.p, iters);
    });
    return ms <= 0.0 ? -3.0 : ms * 1e-3 * d.clock_hz / (4.0 * iters * waves);
}

// Nominal clocks a compute unit spends per wave-wide 16-byte-per-lane streaming store instruction, `waves` (1..16)
// waves per compute unit storing to cache lines that stay in the L2.
extern "C" double pconv_peak_vmem_clk_per_store(int waves) {
    if (waves < 1 || waves > 16) return -1.0;
    DeviceShape d;
    if (device_shape(&d)) return -1.0;
    const int iters = 4000;
    Scratch o;
    if (!o.get((size_t)d.cus * waves * 4096)) return -2.0;
    const double ms = timed_ms([&] { hipLaunchKernelGGL(vmem_store_kernel, dim3(d.cus), dim3(waves * 64), 0, 0, o.p, iters); });
    return ms <= 0.0 ? -3.0 : ms * 1e-3 * d.clock_hz / (4.0 * iters * waves);
}

// Dense fp16 MFMA rate (v_mfma_f32_32x32x16_f16) in TFLOP/s with `waves_per_simd` waves on every SIMD (1 or 2).
extern "C" double pconv_peak_mfma_f16_tflops(int waves_per_simd) {
    if (waves_per_simd != 1 && waves_per_simd != 2) return -1.0;
    DeviceShape d;
    if (device_shape(&d)) return -1.0;
    const int threads = waves_per_simd * 4 * 64, iters = 20000;
    Scratch o;
    if (!o.get((size_t)d.cus * threads * 4)) return -2.0;
    const double ms = timed_ms([&] { hipLaunchKernelGGL(mfma_kernel, dim3(d.cus), dim3(threads), 0, 0, o.p, iters); });
    return ms <= 0.0 ? -3.0 : 4.0 * 2.0 * 32 * 32 * 16 * iters * (threads / 64) * (double)d.cus / (ms * 1e-3) / 1e12;
}

// Compute units and nominal engine clock (MHz) of the current device.
extern "C" int pconv_peak_device(int* compute_units, double* clock_mhz) {
    DeviceShape d;
    if (device_shape(&d)) return -1;
    if (compute_units) *compute_units = d.cus;
    if (clock_mhz) *clock_mhz = d.clock_hz / 1e6;
    return 0;
}
