/*
 * pconv_peaks — measured peaks of the GPU that libpconv runs on.  C ABI of libpconv_peaks.so, a library of its own:
 * nothing on the convolution path uses it.  The roofline figures of the benchmark are quoted against the published
 * peaks of MI355X; these small register-, LDS- and memory-only kernels say what the same resources deliver on the
 * chip at hand, which is what the design notes mean by "measured on this chip".
 *
 * Every function runs its kernel on the current device's default stream, synchronises, and returns the figure, or a
 * negative value on error.  "Per clock" figures use the engine clock that the runtime reports for the device (the
 * nominal peak clock), not the clock held during the run.
 */
#ifndef PCONV_PEAKS_H
#define PCONV_PEAKS_H

#ifdef __cplusplus
extern "C" {
#endif

/* Compute units and nominal engine clock (MHz) of the current device; 0 on success. */
int pconv_peak_device(int* compute_units, double* clock_mhz);

/* Device-to-device copy with 16-byte accesses, `mib` MiB each way: GB/s, bytes read plus bytes written. */
double pconv_peak_copy_gbs(int mib);

/* fp32 vector multiply-adds on registers only (16 independent accumulators per lane), `waves_per_simd` = 1, 2 or 4
 * waves on every SIMD: TFLOP/s. */
double pconv_peak_fma_tflops(int waves_per_simd);

/* 128-bit LDS reads without bank conflicts, `waves` (1..16) waves per compute unit: bytes per clock and compute unit. */
double pconv_peak_lds_read_bytes_per_clk(int waves);

/* Global loads that hit the cache, 16 waves per compute unit, `bytes_per_lane` = 4 or 16: clocks a compute unit
 * spends per wave-wide load instruction (the issue rate of its address unit). */
double pconv_peak_vmem_clk_per_load(int bytes_per_lane);

/* Streaming global stores of 16 bytes per lane to lines that stay in the L2, `waves` (1..16) waves per compute unit:
 * clocks a compute unit spends per wave-wide store instruction (1 KB). */
double pconv_peak_vmem_clk_per_store(int waves);

/* Dense fp16 matrix-core multiply-adds (v_mfma_f32_32x32x16_f16) on registers only, `waves_per_simd` = 1 or 2:
 * TFLOP/s. */
double pconv_peak_mfma_f16_tflops(int waves_per_simd);

#ifdef __cplusplus
}
#endif
#endif /* PCONV_PEAKS_H */
