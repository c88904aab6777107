/*
 * Device characterisation for the benchmark: NOT part of the product path and not bound by the rules
 * of ozimmu.h (this call allocates a few KiB of device and pinned host memory for its duration and
 * synchronises the device).
 */
#ifndef OZIMMU_PROBE_H
#define OZIMMU_PROBE_H

#include "ozimmu.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Sustained rate of a register-only INT8 MFMA issue loop on all compute units, in 10^12 INT8
 * operations per second, and the shader clock it ran at (the ceiling against which the slice-product
 * kernel of Section 3.1 is judged: the reachable matrix-core clock depends on the operand data).
 *   pattern 0: all-zero operands; 1: random bytes; 2: random signed 7-bit magnitudes (the value
 *     distribution of the slices); 3: random signed 3-bit magnitudes; 4: random 7-bit magnitudes
 *     without sign; 5: A as 2, every byte of B equal to 1; 6: A as 2, B zero.
 *   shape 0: v_mfma_i32_32x32x32_i8 (the instruction the product kernel uses);
 *         1: v_mfma_i32_16x16x64_i8 (the kernel for a gate on a state vector uses it);
 *         2: v_mfma_i32_16x16x32_i8, the older form with half the inner dimension.
 * Errors: OZIMMU_ERR_BAD_DIM for an unknown pattern or shape or iters < 1, OZIMMU_ERR_NULL,
 * OZIMMU_ERR_HIP.
 */
ozimmu_status_t ozimmu_probe_int8_mfma(int pattern, int shape, int iters, double* tera_ops_per_s,
                                       double* shader_mhz);

#ifdef __cplusplus
}
#endif
#endif /* OZIMMU_PROBE_H */
