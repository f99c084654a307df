/*
 * dppo_probe.h -- measurement utilities of the DPPO loss library (not part of the loss).
 *
 * Plain streaming kernels and a matrix-core loop that benchmarks use to state what the device
 * itself sustains next to what the loss kernels reach, and that calibrate the HBM byte counters
 * (a copy of known size).  Conventions as in dppo.h: device pointers owned by the caller, work
 * enqueued on `stream`, nothing allocated, no synchronisation, host-side checks only.
 */
#ifndef DPPO_PROBE_H
#define DPPO_PROBE_H

#include "dppo.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Plain device-to-device copy of `bytes` bytes with 16-byte vector loads/stores (dst, src and
 * bytes multiples of 16; buffers must not overlap), a write-only fill of `bytes` bytes with a
 * 32-bit pattern, and a read-only pass over `bytes` bytes (`sink` is a 4-byte device location
 * that is practically never written).  bench.py and the
 * counter-calibration probe use them: a copy of known size scales the HBM byte counters, and
 * their bandwidth is the device's streaming ceiling the loss kernels are compared with. */
dppo_status_t dppo_probe_copy(void* dst, const void* src, size_t bytes, void* stream);
/* The same copy with the loss kernels' address pattern: one workgroup per row of `row_bytes` bytes
 * (rows `pitch_bytes` apart; both multiples of 16), as many workgroups as compute units. */
dppo_status_t dppo_probe_copy_rows(void* dst, const void* src, int64_t rows, size_t row_bytes, size_t pitch_bytes, void* stream);
/* The same row-by-row copy with the memory pattern of the register-resident loss kernel and none
 * of its arithmetic: one persistent workgroup per compute unit holds a whole row in its registers,
 * writes it in one run of non-temporal stores and then requests its next row in one run of loads.
 * row_bytes <= 311296 (512 threads x 38 chunks of 16 bytes), else DPPO_ERR_SHAPE. */
dppo_status_t dppo_probe_copy_resident(void* dst, const void* src, int64_t rows, size_t row_bytes, size_t pitch_bytes, void* stream);
dppo_status_t dppo_probe_fill(void* dst, size_t bytes, uint32_t value, void* stream);
dppo_status_t dppo_probe_read(const void* src, size_t bytes, void* sink, void* stream);
/* Matrix-core ceiling under the board's power limit: one workgroup of 4 waves per compute unit,
 * each wave `iters` rounds of independent bf16 products on register operands with 256 fp32
 * accumulators: `shape` 16 = 64 x v_mfma_f32_16x16x32_bf16 per round, 32 = 16 x
 * v_mfma_f32_32x32x16_bf16.  `out` (device, at least 1024 bytes per compute unit, `out_bytes`
 * says how many) receives one float per lane; `*flop` (host, may be NULL) the floating-point
 * operations of the launch, for the caller to divide by the time it measures.
 * DPPO_ERR_SHAPE for another shape or negative iters, DPPO_ERR_WORKSPACE if `out` is too small. */
dppo_status_t dppo_probe_mfma(int shape, int iters, void* out, size_t out_bytes, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DPPO_PROBE_H */
