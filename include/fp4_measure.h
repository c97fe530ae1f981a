/*
 * fp4_measure.h -- measurement and self-check helpers of libfp4mi.so, kept apart from the
 * product ABI (fp4_linear.h): the library's own rounding routine exposed for exhaustive
 * checks, ceilings of the part the rooflines are read against, and a per-launch timer of the
 * GEMM kernel.  Nothing here is on the hot path.  Status codes are fp4_status.
 */
#ifndef FP4_MEASURE_H
#define FP4_MEASURE_H

#include "fp4_linear.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Host-side evaluation of the library's own rounding routine: codes[i] = Q(x[i]) for
 * n fp32 values in HOST memory (the same inline function the kernels use, compiled for
 * the CPU; lets the rounding be checked exhaustively without a GPU). */
int fp4_host_round_codes(const float* x_host, int64_t n, uint8_t* codes_host);
/* The same for the E4M3 rounding of the mixed-format path. */
int fp8_host_round_codes(const float* x_host, int64_t n, uint8_t* codes_host);

/* The rounding as the quantization kernels perform it on the device (App. A's rule carried out
 * by the FP4 convert instruction, eight values per packed word): codes[i] = Q(x[i]), one code per
 * byte, x and codes in DEVICE memory, n a multiple of 8.
 * fp4_device_round_sweep: runs every one of the 2^32 fp32 bit patterns, in each of the eight
 * positions of a packed word, through that routine and through the comparison chain that
 * fp4_host_round_codes exposes, and ADDS the number of disagreements to *mismatches (device
 * memory, 8 bytes, set it to 0 first).  About a second of GPU time. */
int fp4_device_round_codes(const float* x, int64_t n, uint8_t* codes, void* stream);
int fp4_device_round_sweep(unsigned long long* mismatches, void* stream);

/* ---- ceilings measured on the part (for reading the rooflines; not part of the method) ----
 * fp4_probe_mfma: `workgroups` workgroups of 8 waves each run `iters` iterations of 8 FP4
 *   32x32x64 MFMAs per wave with operands taken from operand_bytes (device, >= 16 bytes): an
 *   issue loop without memory traffic.  FLOP = workgroups * 8 * iters * 8 * 131072.  The rate
 *   depends on the operand data (random codes draw more power than constant ones).
 *   sink: device, workgroups * 512 floats.
 * fp4_probe_copy: dst[0..nbytes) = src[0..nbytes), 16 bytes per lane (streaming copy). */
int fp4_probe_mfma(const void* operand_bytes, int64_t nbytes, int workgroups, int iters, float* sink,
                   void* stream);
int fp4_probe_copy(const void* src, void* dst, int64_t nbytes, void* stream);

/* ---- measurement helper (host-side state, off by default; not thread-safe) ----
 * Between fp4_trace_begin(n) and fp4_trace_end() every launch of the FP4 GEMM kernel and of the
 * tiled sparse-product kernel, from any entry point, is bracketed by a pair of HIP events recorded
 * on the launch's own stream (at most n launches; later ones are not recorded).
 * fp4_trace_end waits for the recorded launches, writes their durations in milliseconds and their
 * kinds, in launch order, to ms_host / kind_host [0..capacity) (HOST memory) and returns the number
 * of launches recorded (>= 0) or a negative fp4_status. */
enum { FP4_TRACE_GEMM = 0, FP4_TRACE_SPMM = 1 };
int fp4_trace_begin(int max_launches);
int fp4_trace_end(float* ms_host, int* kind_host, int capacity);

#ifdef __cplusplus
}
#endif
#endif /* FP4_MEASURE_H */
