/* Instruction-rate probe for gfx950 (MI355X), C ABI: a measurement aid beside the allocation search
 * library (libloki_probe.so, built from csrc/loki_valu_rate.hip; not part of libloki_alloc.so).  It tells what
 * the GPU at hand sustains for the vector-ALU instruction classes the search's kernels are made of, for
 * callers that report a fraction of peak. */
#ifndef LOKI_PROBE_H
#define LOKI_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Sustained issue rate, in wavefront instructions per second over the whole GPU, of a dependency-free
 * stream of one vector-ALU instruction class, 8 wavefronts per SIMD.
 *   kind  0 v_mul_f64, 1 v_add_f64, 2 v_max_f64, 3 the search's multiply/add/max mix, 4 v_add_u32,
 *         5 v_fma_f64, 6 v_rcp_f64, 7 v_mul_lo_u32, 8 v_mul_hi_u32, 9 v_min_u32,
 *         10 ds_read_b64 (LDS reads of 8 bytes per lane, 16 in flight per wavefront)
 *   d_workspace  device, >= 4 MiB, 8-byte aligned (a sink for the kernels; the caller owns it)
 *   hip_stream   a hipStream_t (null: the default stream)
 *   wave_instructions_per_second  host, written on success
 * Blocks until the measurement (tens of ms) is done.  Returns 0, -1 (a null pointer), -4 (workspace too
 * small or misaligned), -6 (no such kind), or -5 with *hip_error (host, may be null) set to the HIP runtime's
 * code.  The nominal figure is compute_units * 4 SIMDs * clock / 4 cycles. */
int loki_measure_valu_rate(int kind, void *d_workspace, size_t workspace_bytes, void *hip_stream,
                           double *wave_instructions_per_second, int *hip_error);

#ifdef __cplusplus
}
#endif

#endif
