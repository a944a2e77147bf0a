/*
 * mttkrp_calibrate.h -- what this GPU sustains on its own, measured with the
 * same ingredients the streaming kernel uses: a read-only pass over a buffer
 * (non-temporal 16-byte loads, nothing else) and back-to-back 16x16x4 MFMAs on
 * register operands (no memory traffic).  The paper's performance model (Sec.
 * IV-B) takes a machine's bandwidth and flop rate as given; these two calls
 * measure them, so that a result can be quoted against the ceiling the box
 * reaches as well as against the data-sheet peak.
 *
 * Both calls time `launches` launches (after two untimed ones) with HIP events
 * on `stream`, wait for them, and return the mean milliseconds per launch.
 * They allocate nothing and keep no state.  Errors: MTTKRP_ERR_INVALID_ARG
 * for null or misaligned arguments or launches < 1, MTTKRP_ERR_DEVICE when a
 * HIP call fails.
 */
#ifndef MTTKRP_CALIBRATE_H
#define MTTKRP_CALIBRATE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Read-only stream over buf[0 .. bytes): every 16-byte piece is loaded once.
 *   buf     device, 16-byte aligned; bytes a multiple of 16, at least 16
 *   ms_mean host, written: mean milliseconds per pass (GB/s = bytes / ms / 1e6)
 */
int mttkrp_calibrate_stream(const void* buf, size_t bytes, int launches, float* ms_mean,
                            void* stream);

/*
 * Back-to-back MFMAs: every SIMD of the chip issues independent
 * v_mfma_f64_16x16x4_f64 (dtype_bytes = 8) or v_mfma_f32_16x16x4_f32
 * (dtype_bytes = 4) on non-trivial register operands for about `gflop_per_launch`
 * GFLOP per launch (rounded up to whole loop iterations; 2048 flop per MFMA).
 *   ms_mean  host, written: mean milliseconds per launch
 *   flop     host, written: flop actually executed per launch
 * The sustained rate depends on how long the chip has been under load (the
 * clock drops under sustained matrix-core load), so use launches of the length
 * of the kernel that is being compared.
 */
int mttkrp_calibrate_mfma(int dtype_bytes, double gflop_per_launch, int launches, float* ms_mean,
                          double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MTTKRP_CALIBRATE_H */
