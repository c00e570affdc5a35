/*
 * libpsa measurement aids.  NOT part of the method and not needed to use it: two trivial kernels the
 * benchmark runs to state what this GPU sustains, next to the published peaks that its roofline
 * fractions are quoted against.  Status codes are those of psa.h.
 */
#ifndef PSA_PROBE_H
#define PSA_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * psa_probe_copy: plain streaming copy of `bytes` (a multiple of 16) from src to dst, both device
 *   pointers of at least that size; moves 2 * bytes through HBM.
 * psa_probe_mfma: `workgroups` workgroups of 4 wavefronts, each wavefront issuing iters * 16
 *   bfloat16 32x32x16 MFMAs on register operands.  random_operands = 0: a few small values (the
 *   least power the matrix pipe can draw); != 0: random signs and mantissas, magnitudes in [0.5, 2),
 *   as real activations have (the sustained rate is markedly lower: the clock follows the power).
 *   sink: device, workgroups * 256 floats (written once).  flops (host pointer, nullable) receives
 *   the floating-point operations of the launch.
 * Both are asynchronous on `stream`; PSA_EINVAL for null pointers or sizes out of range.
 */
int psa_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
int psa_probe_mfma(float* sink, int workgroups, int iters, int random_operands, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PSA_PROBE_H */
