/*
 * msgemm_measure.h -- measurement aids of the msGeMM library for AMD MI355X
 * (gfx950).  Nothing here is msGeMM: a dense comparison kernel on the same
 * inputs (Section 6 of arxiv 2310.06178 names the matrix units as what a
 * table-add has to compete with) and kernels that only read memory, only read
 * LDS, or run the look-up + add instruction mix alone -- the yardsticks that
 * the benchmark times beside msgemm_run.  Same conventions as msgemm.h: device
 * pointers, a hipStream_t passed as void*, MSGEMM_OK or a negative
 * msgemm_status_t, nothing thrown across the boundary.
 */
#ifndef MSGEMM_MEASURE_H
#define MSGEMM_MEASURE_H

#include "msgemm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Comparison point only, not msGeMM: the same Y computed as a dense
 * contraction on the matrix cores (codes dequantised to bf16/fp16 in
 * registers, MFMA per scale block, fp32 accumulate).  Floating-point dtypes
 * only.  Exists so the LUT path can be timed against it on equal inputs
 * (Section 6 argues the matrix units are what a table-add has to compete with).
 * Reads rows like msgemm_consume_lut: the same first-call allocation applies.
 */
int msgemm_dequant_mfma_run(const msgemm_plan_t* plan, const void* X, int64_t ldx,
                            void* Y, int64_t ldy, void* stream);

/*
 * Measurement aid, not msGeMM: reads `bytes` bytes at `src` (device, 16-byte
 * aligned, bytes a multiple of 128 KiB) once, with the load shape of the fused
 * kernel's code stream (128 bits per lane, one workgroup per compute unit) and
 * nothing else.  Timed like msgemm_run it gives the rate at which this device
 * delivers a cold stream of that size to a single launch: the practical
 * ceiling beside the nominal HBM peak.  `sink` (device, >= 4 bytes) is only
 * written if the data sums to a magic value.
 */
int msgemm_calib_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/*
 * The same read with its launch shape as parameters, for the sweep that shows
 * what a launch that only reads can reach on this device: `workgroups_per_cu`
 * (1..16) workgroups per compute unit of `waves_per_workgroup` (1..16)
 * wavefronts, `depth` (1, 2, 4, 8 or 16) 16-byte loads per lane in flight per
 * wavefront, `non_temporal` != 0 marks the loads as streaming.  bytes: below
 * 2 GiB and such that every wavefront gets a multiple of `depth` loads of 1 KiB
 * (else MSGEMM_ERR_INVALID_ARG).
 */
int msgemm_calib_stream_read_shape(const void* src, size_t bytes, void* sink, int waves_per_workgroup,
                                   int workgroups_per_cu, int depth, int non_temporal, void* stream);

/*
 * Measurement aid, not msGeMM: one workgroup of 16 wavefronts per compute unit
 * reads LDS and nothing else -- every lane `reads` times (a multiple of 8, at
 * most 2^20) `width_bytes` (4, 8 or 16) bytes, consecutive lanes consecutive
 * slots, i.e. free of bank conflicts, eight reads in flight per lane.  Timed
 * like msgemm_run it gives the LDS read bandwidth of the device, the
 * denominator for the gather of the batched kernels (Section 6 of the paper
 * expects phase 2 to be bound by such look-ups).  *bytes_out (host, may be NULL)
 * receives the bytes one launch reads; `sink` (device, >= 4 bytes) is only
 * written if the data sums to a magic value.
 */
int msgemm_calib_lds_read(int width_bytes, int reads, void* sink, size_t* bytes_out, void* stream);

/*
 * Measurement aid, not msGeMM: the inner loop of the batched kernels and
 * nothing else.  One workgroup of 8 wavefronts per compute unit; every lane
 * makes 128 * tiles look-ups (tiles in 1 .. 65536) of 16 bytes in a 128 KiB
 * table at addresses formed from code bytes as the kernels form them, and adds
 * each entry's eight fp16 columns to fp32 sums with two matrix-core
 * instructions against the identity, the look-ups eight ahead of the adds.
 * Timed like msgemm_run it gives the rate at which the device sustains that
 * instruction mix: the practical ceiling of phase 2 for batches (Section 6
 * expects phase 2 to be bound by the look-ups; here the adds cost as much).
 * *lookups_out (host, may be NULL) receives the lane look-ups of one launch;
 * `sink` (device, >= 4 bytes) is never written in practice.
 */
int msgemm_calib_lookup_add(int tiles, void* sink, size_t* lookups_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MSGEMM_MEASURE_H */
