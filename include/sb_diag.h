/*
 * sb_diag.h -- measurement aids of the stick-breaking attention library (libsbattn.so).
 *
 * Nothing here is part of the method (Eq. 1 / Algorithms 1 and 2): these calls exist so that
 * the benchmark can put the attention kernels' rates beside what the chip sustains with the
 * same instruction mix and nothing else in flight.  Same conventions as sb_attn.h: device
 * pointers owned by the caller, 16-byte aligned, `stream` a hipStream_t (NULL = default
 * stream), calls only enqueue, the return value is an sb_status.
 */
#ifndef SB_DIAG_H
#define SB_DIAG_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Matrix pipe alone: runs `iters` x 16 independent 32x32x16 bf16 MFMAs per wavefront, two
 * wavefronts per SIMD on the whole chip, on operands taken from `operands` (device, bf16,
 * at least 1 MiB) and nothing else.  The rate it reaches is what the matrix cores sustain
 * on that data under the chip's power limit.  ticks (device, 3 x u64) receives [0] shader
 * clocks and [1] 100 MHz reference ticks of one wavefront's loop; *flop (host) receives the
 * FLOP the launch executes.
 */
int sb_diag_mfma_rate(const void* operands, size_t operand_bytes, int iters, unsigned long long* ticks,
                      double* flop, void* stream);

/*
 * Memory pipe alone: one kernel that loads every 16-byte word of [data, data + bytes) once
 * and does nothing else (bytes a multiple of 16, at least 1 MiB).  bytes / duration is the
 * read bandwidth a kernel without arithmetic reaches on this chip: the practical ceiling
 * beside the published 8 TB/s for the bandwidth-bound decode kernel.  sink: device, one u32,
 * written only if the xor of all words has one particular value (it keeps the loads alive).
 */
int sb_diag_stream_read(const void* data, size_t bytes, unsigned int* sink, void* stream);

/*
 * sb_attn_fwd_train (same arguments, same kernel, same results) that also samples the clock:
 * clocks (device, 4 x u64) receives the shader-clock counter and the 100 MHz reference
 * counter read by the launch's first workgroup when it starts ([0], [1]) and when it ends
 * ([2], [3]); ([2]-[0]) / ([3]-[1]) * 100 MHz is the shader clock the chip sustained
 * under this kernel's load.
 */
int sb_diag_fwd_clock(const void* q, const void* k, const void* v, void* o, float* m,
                      int B, int H, int T, int d, unsigned long long* clocks, void* stream);

/*
 * The training forward (sb_attn_fwd_train: same arguments, same outputs to the same tolerance)
 * with the other of the two ways the in-tile reverse cumulative sum of Algorithm 1 can be
 * taken on this chip: on the matrix pipe, as a product with a triangular matrix of ones, in
 * the log form of Eq. 2 (softplus per element, the sum by MFMA with the summands split into
 * two bf16 parts, one more exponential per weight).  The product path uses an in-lane chain
 * instead; this entry point exists so that the choice is a measured one.  d = 128 only
 * (SB_ERR_UNSUPPORTED otherwise).  Logits beyond the range of the base-2 softplus are fine
 * (it is overflow-proof).
 */
int sb_diag_fwd_tri(const void* q, const void* k, const void* v, void* o, float* m,
                    int B, int H, int T, int d, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SB_DIAG_H */
