/* ovggt_measure.h -- measurement helper of the MI355X OVGGT build; NOT part of the hot path and
 * built as a library of its own (libovggt_measure.so), so the product library exports nothing
 * that only a benchmark needs.
 */
#ifndef OVGGT_MEASURE_H
#define OVGGT_MEASURE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The rate (TFLOP/s, host double) that the matrix cores sustain when every wave issues nothing
 * but the attention kernel's MFMA (v_mfma_f32_32x32x16_f16, fp32 accumulation) on register
 * operands: the denominator that is reachable in practice for the temporal attention of Sec. 3.1,
 * beside the published dense peak.  `workgroups` workgroups of four waves (512 on a 256-CU chip
 * gives two waves per SIMD, as the attention kernel has), `iters` rounds of four MFMAs per wave
 * (20000 makes a launch of about a millisecond), twenty launches timed after one of warm-up.
 * random_operands != 0: unit-variance random operands, under which the chip lowers its clock;
 * 0: constant operands.  sink_dev: device memory, at least 4 bytes, never written.  Synchronises
 * hip_stream (a hipStream_t as void*).  Returns 0, -1 (bad argument) or -4 (a HIP call failed). */
int ovggt_measure_mfma_loop(void* sink_dev, int32_t workgroups, int32_t random_operands, int32_t iters,
                            double* tflops, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* OVGGT_MEASURE_H */
