/*
 * Measurement helpers of libvispec_verify: three trivial kernels whose achieved rates show
 * what the machine delivers (streaming read, copy, bf16 matrix-core loop). They are not part
 * of the verification method; bench.py times them and prints the rates beside the data-sheet
 * peaks its roofline fractions are quoted against. Same conventions as vispec_verify.h: C ABI,
 * device pointers owned by the caller, kernels enqueued on `stream`, no allocation, int32
 * vs_error results (VS_ERR_NULL, VS_ERR_SHAPE for sizes or alignment, VS_ERR_NO_DEVICE,
 * VS_ERR_HIP).
 */
#ifndef VISPEC_PEAKS_H
#define VISPEC_PEAKS_H

#include <stddef.h>
#include <stdint.h>

#include "vispec_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

#define VS_PEAK_MAX_WORKGROUPS 65536

/* Reads `bytes` (rounded down to 16) of `src` (16-byte aligned) once with `workgroups` x 256
 * threads; `sink` receives one uint32 per workgroup (xor of what it read; sink must hold
 * `workgroups` words, zeroed or not). Algorithmic bytes = bytes. */
int32_t vs_peak_hbm_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream);

/* dst[0..bytes) = src[0..bytes) in 16-byte pieces (both 16-byte aligned, not overlapping).
 * Algorithmic bytes = 2 x bytes (read + write). */
int32_t vs_peak_hbm_copy(void* dst, const void* src, size_t bytes, int32_t workgroups, void* stream);

/* `workgroups` x 8 waves each issue iters x 16 v_mfma_f32_32x32x16_bf16 on four independent
 * accumulators. `operands`: 8 x 128 x 16 bytes (per wave of a workgroup: 64 lanes x 8 bf16 for the
 * A operand, then the same for B; every workgroup reads the same 16 KB); their bit patterns set the
 * power the loop draws. `sink`: workgroups x 512 floats. vs_peak_mfma_flops gives the flops of one
 * such launch. */
int32_t vs_peak_mfma_bf16(const void* operands, int32_t iters, void* sink, int32_t workgroups, void* stream);
double vs_peak_mfma_flops(int32_t iters, int32_t workgroups);

#ifdef __cplusplus
}
#endif
#endif /* VISPEC_PEAKS_H */
