/*
 * quest_probe.h - measurement aid for the benchmark, not part of the method: what the matrix
 * pipes of this machine sustain when nothing else is asked of the chip.  A kernel whose waves hold
 * their operands in registers and issue independent matrix instructions back to back, with no LDS
 * or memory traffic in the loop.  bench.py times it on operand data shaped like the method's
 * (signed bytes 8 u of Gaussian-fitted 4-bit codes; bf16 values s u), because the rate the chip
 * sustains depends on the data (it is power-limited), and reports every matmul kernel also as a
 * fraction of this rate.
 */
#ifndef QUEST_PROBE_H
#define QUEST_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueues one launch of the register-only loop on `stream` (hipStream_t as void*).
 *   kind        0: v_mfma_i32_32x32x32_i8 (32768 multiply-adds each)
 *               1: v_mfma_f32_32x32x16_bf16 (16384 multiply-adds each)
 *   operands    device memory, workgroups * 256 * 32 bytes: per thread two 16-byte operands
 *   sink        device memory, workgroups * 256 * 4 bytes: one word per thread (keeps the loop alive)
 *   workgroups  workgroups of 256 threads (four waves); iterations: loop trips of 8 instructions per wave
 * Total multiply-adds of a launch: workgroups * 4 * iterations * 8 * (32768 or 16384).
 * Returns 0, or 1 for a null pointer / non-positive count / unknown kind, 2 if the launch was refused.
 */
int32_t quest_probe_mfma_loop(int32_t kind, const void *operands, void *sink, int32_t workgroups,
                              int32_t iterations, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QUEST_PROBE_H */
