/*
 * she_diag.h - hardware diagnostics of the MI355X library.  NOT part of the problem statement of
 * "SHE: A Fast and Accurate Deep Neural Network for Encrypted Data" (arXiv 1906.00148) and not needed
 * to evaluate anything: a micro-benchmark that the benchmark program prints beside its roofline figures
 * so that a reader can see what the FP64 pipes and the LDS of the device at hand deliver.  Same conventions as she.h.
 */
#ifndef SHE_DIAG_H
#define SHE_DIAG_H

#include "she.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Issue rate of one FP64 vector instruction form on this device, measured with 2 wavefronts per SIMD like the
 * blind rotation (form 0: fma with scalar multiplier and addend, 1: fma with three vector-register operands, 2: add
 * of two vector registers, 3: the additions of form 2 with the blind rotation's memory instructions beside them:
 * per 64 additions 6 LDS reads, 3 LDS writes and 2 global loads of 16 bytes per lane, the loads streaming the
 * context's spectral bootstrapping key).  ns_per_instruction is per FP64 instruction and SIMD; tflops_as_fma
 * prices every FP64 instruction as an FMA over the whole chip, the figure to hold against the published FP64
 * vector peak.  Either pointer may be NULL. */
int she_probe_fp64_rate(she_ctx *ctx, int form, double *ns_per_instruction, double *tflops_as_fma);

/* Throughput of the LDS pipe of one compute unit on this device, in bytes per nanosecond, for 16-byte-per-lane
 * operations of 8 wavefronts (2 per SIMD, like the blind rotation) in the layout of the transforms' exchange buffer
 * (eight rows of 64 slots plus padding).  form 0: loads of consecutive slots; 1: stores of consecutive slots (what an
 * exchange writes); 2: the read-back after the first pass (lane 8a + b reads slots a*row + b + 8m) with the row length
 * the 512-point plan uses for that exchange; 3: the same with a row of 65 slots; 4: the read-back after the second
 * pass (b*row + 8a + m) with its row length of 65.  The row lengths of the plans were chosen from these figures. */
int she_probe_lds_rate(she_ctx *ctx, int form, double *bytes_per_ns_per_cu);

#ifdef __cplusplus
}
#endif
#endif /* SHE_DIAG_H */
