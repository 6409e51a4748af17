/*
 * she_diag.h - hardware diagnostics of the MI355X library.  NOT part of the problem statement of
 * "SHE: A Fast and Accurate Deep Neural Network for Encrypted Data" (arXiv 1906.00148) and not needed
 * to evaluate anything: a micro-benchmark that the benchmark program prints beside its roofline figures
 * so that a reader can see what the FP64 pipes of the device at hand issue at.  Same conventions as she.h.
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

#ifdef __cplusplus
}
#endif
#endif /* SHE_DIAG_H */
