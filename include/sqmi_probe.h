/*
 * sqmi -- measurement aids of the library, NOT part of the method's boundary (that is sqmi.h).
 * bench.py uses them to report kernels against what the hardware sustains.
 */
#ifndef SQMI_PROBE_H
#define SQMI_PROBE_H

#include "sqmi.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Runs `iters` rounds of 16 register-fed INT8 MFMAs (16x16x64, the shape of the compute-bound GEMM tiles) on each of
 * the 8 waves of `workgroups` workgroups, i.e. workgroups * 8 * iters * 16 * 32768 integer operations, with no
 * memory traffic inside the loop.  The operand registers are filled once from `data` (device int8, at least
 * workgroups * 49152 bytes: the bit patterns matter, the sustained clock depends on them); sink: device int32
 * [workgroups * 512], overwritten.  bench.py times it to report the GEMM against what the matrix pipes sustain. */
sq_status sq_probe_mfma_i8(const int8_t* data, size_t data_bytes, int workgroups, int iters, int32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SQMI_PROBE_H */
