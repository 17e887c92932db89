/*
 * aeris_probe.h -- measurement aid shipped with the shifted-window attention library; not part
 * of the attention path and not needed by its callers.  bench.py uses it to report, next to the
 * fraction of the published MFMA peak, the fraction of the MFMA rate this machine sustains under
 * its power limit.
 */
#ifndef AERIS_PROBE_H
#define AERIS_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launches `blocks` workgroups of 256 threads, each wave issuing
 * 8 * iters v_mfma_f32_32x32x16_bf16 on register operands (32768 FLOP each) and nothing else.
 * random_operands != 0 fills the operands with pseudo-random bf16 values of unit scale, else
 * with small integers.  sink: device buffer of blocks * 256 floats, overwritten.
 * 1 <= blocks <= 65536, 1 <= iters.  FLOPs of a launch: blocks * 4 * iters * 8 * 32768.
 */
int aeris_mfma_loop_probe(int32_t blocks, int32_t iters, int32_t random_operands, float* sink,
                          void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* AERIS_PROBE_H */
