/* Measured-peak probes for the roofline of the sub-bit convolution library (gfx950 / MI355X).
 *
 * Not part of the method: these are the yardsticks that bench.py prints as `roofline.peaks_measured`
 * next to the vendor peaks, so that every roofline fraction can be recomputed from tracked code.
 * Each probe launches ONE kernel on `stream` (a hipStream_t passed as void*), asynchronously; the
 * caller times it with HIP events on that stream and divides the stated work by the duration.
 *
 * All pointers are caller-owned DEVICE pointers; nothing is allocated, freed or retained.  Return
 * value: 0 on success, -1 invalid argument (null pointer, size not a multiple of 4096, counts < 1),
 * -4 if the launch failed.  Built into libsnn_peaks.so (separate from the product library).
 */
#ifndef SNN_PEAKS_H
#define SNN_PEAKS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Device-to-device copy, 16 bytes per lane and access.  Work: `bytes` read + `bytes` written.
 * `bytes` must be a multiple of 4096. */
int snn_peak_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Write-only stream of 16-byte stores (non-temporal when `nontemporal` != 0): the pattern of a
 * kernel that writes its output once.  Work: `bytes` written. */
int snn_peak_fill(void *dst, size_t bytes, int nontemporal, void *stream);

/* Read-only stream of 16-byte loads (non-temporal when `nontemporal` != 0), four in flight per lane, every block
 * reading one contiguous piece: the pattern of a kernel that reads its input once (sign + pack).  Work: `bytes` read.  A buffer larger than the 256 MB
 * memory-side cache measures HBM, a smaller one read again measures that cache.
 * out: SNN_PEAK_READ_BLOCKS * 256 words (one folded word per lane). */
#define SNN_PEAK_READ_BLOCKS 16384
int snn_peak_read(const void *src, size_t bytes, int nontemporal, uint32_t *out, void *stream);

/* Plain integer VALU: a loop of v_xor_b32 + v_bcnt_u32_b32 (the 1-bit kernel's pair).
 * `blocks` workgroups of 256 lanes; work: blocks * 256 * iters * 32 lane-operations.
 * out: blocks * 256 words (a checksum that keeps the loop alive). */
int snn_peak_valu_xor_bcnt(uint32_t *out, int iters, int blocks, void *stream);

/* Matrix cores, FP4 (e2m1) x FP6 (e2m3) operands, fp32 accumulators, 8 independent accumulator
 * sets per wave.  shape 0: v_mfma_f32_32x32x64_f8f6f4 (131072 flop per instruction);
 * shape 1: v_mfma_f32_16x16x128_f8f6f4 (65536 flop).  pattern 0: every operand slot holds a
 * random code; 1: the operands of the sub-bit kernel (A: a one-hot row per 32 slots, B: small
 * integers -4 .. 5); 2: zeros.  `blocks` workgroups of 4 waves; work: blocks * 4 * iters * 8
 * instructions.  out: blocks * 256 floats, then (at out + blocks * 256) per workgroup two 64-bit
 * counters: shader clocks and constant-rate (100 MHz) ticks spent in the loop by wave 0, from
 * which the clock the loop ran at follows. */
int snn_peak_mfma_f4f6(float *out, int shape, int pattern, int iters, int blocks, void *stream);

/* Bytes of `out` that snn_peak_mfma_f4f6 writes. */
size_t snn_peak_mfma_out_bytes(int blocks);

/* Candidate form of stage 2 (Sec. 4.5: gather the responses by index, sum over c_in) WITHOUT the
 * matrix cores: a lane holds the K = 32 responses of 4 pixels as bytes of 32 registers, the
 * accumulators of 64 output channels as bytes of 64 registers (widened to 16 bits every 28 input
 * channels), and adds `response[idx[ci][co]]` with the wave-uniform index supplied through the
 * vector-register index mode: one v_add_u32 = 4 gather-adds.  Stage 1 is NOT part of the probe (the
 * responses are constants), so the rate is an upper bound of that form.
 *   idx: uint32 [n_ci][64] followed by 48 readable words (the loop requests its indices three chunks of
 *        16 ahead and does not stop at the end), every value < 32;  n_ci a multiple of 28, at most 7168
 *   out: blocks * 256 words; each receives sum over (ci, co) of 4 * value(idx[ci][co]) with
 *        value(k) = (7 k + 3) mod 10  (the four bytes of a lane hold the same value)
 * `blocks` workgroups of 4 waves.  Work: blocks * 256 * 4 * 64 * n_ci gather-adds. */
int snn_peak_swar_gather(uint32_t *out, const uint32_t *idx, int n_ci, int blocks, void *stream);

#ifdef __cplusplus
}
#endif

#endif
