/*
 * libsv measurement aids -- not part of the method's boundary (include/sv.h): what this chip sustains, as opposed
 * to what its data sheet says, for setting kernel roofline fractions beside achievable ceilings.  Same library,
 * same conventions (plain pointers, status codes of sv.h).
 */
#ifndef SV_PROBE_H_
#define SV_PROBE_H_

#include "sv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * sv_probe_rates -- measurement aid, SYNCHRONOUS; implements no passage of the
 * paper.  Measures what the device sustains, for setting the attention
 * kernels' roofline fractions (taken against the published peaks) beside the
 * achievable ceilings: *mfma_tflops_out = dense bf16 rate of a register-only
 * v_mfma_f32_32x32x16_bf16 loop on every SIMD with constant small-integer
 * operands, *mfma_tflops_random_out = the same loop on pseudo-random operands
 * (the clock under a full-chip matrix load is well below the boost clock, and
 * lower still when the multipliers see real data); *hbm_read_gbs_out = rate of a
 * streaming read of dev_buf[0, bytes) (use a buffer several times the 256 MB
 * memory-side cache).  Any output may be NULL (that probe is skipped).
 * dev_buf: device memory, 16-byte aligned, >= 1 MiB, read only (its first
 * word is written only if a data-dependent condition that cannot occur holds).
 */
SV_API int sv_probe_rates(void* dev_buf, size_t bytes, double* mfma_tflops_out, double* mfma_tflops_random_out,
                          double* hbm_read_gbs_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SV_PROBE_H_ */
