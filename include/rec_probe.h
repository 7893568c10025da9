/*
 * rec_probe.h - measurement helper: what the matrix cores of this device sustain.
 *
 * The published bf16 matrix rate of the chip (the MLP roofline of this build)
 * assumes every compute unit issuing matrix instructions at the top clock.
 * Whether a device sustains that depends on the operand values: with all compute
 * units busy the chip is power-limited, and bit patterns that toggle more of the
 * multiplier array lower the rate it settles at.  rec_probe_mfma() runs nothing
 * but v_mfma_f32_32x32x16_bf16 on register operands, so that a benchmark can
 * put the rate the hardware reaches on constant and on random operands beside
 * the published peak and beside its own GEMMs.  Not part of the forward pass.
 */
#ifndef REC_PROBE_H
#define REC_PROBE_H

#include <stdint.h>
#include "rec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Enqueues on `stream` one launch of `blocks` workgroups of 8 wavefronts; every
 * wavefront issues iters * 32 matrix instructions (32 x 32 x 16, bf16 in, fp32
 * accumulate, 8 independent accumulator tiles): 2 * 32 * 32 * 16 flops each,
 * blocks * 8 * iters * 32 * 32768 flops per launch.  random_operands = 0: every
 * operand element is 1.0; otherwise pseudo-random values in [-1, 1), different
 * per lane and changed every iteration by a sign flip of one operand.
 * dev_sink (device float[1]) receives a checksum.
 * REC_ERR_ARG on null sink or non-positive counts (blocks <= 65536, iters <= 2^20). */
REC_API rec_status rec_probe_mfma(int32_t random_operands, int32_t blocks, int32_t iters,
                          float *dev_sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* REC_PROBE_H */
