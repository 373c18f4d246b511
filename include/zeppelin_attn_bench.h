/*
 * zeppelin_attn_bench.h -- measurement aids of the attention engine. Not part of the product ABI: a caller of the
 * engine needs none of this. bench.py and the tests use them.
 *  - zp_profile_*: exported by libzeppelin_attn.so (they bracket the launches that library makes).
 *  - zp_mfma_probe: exported by libzeppelin_bench.so, a separate small library that holds only the probe kernel.
 */
#ifndef ZEPPELIN_ATTN_BENCH_H
#define ZEPPELIN_ATTN_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid: enqueues a register-only loop of bf16 MFMAs (256 workgroups x 4 waves, iters * 32 instructions of
 * 32x32x16 per wave = 256 * 4 * iters * 32 * 32768 flop in total) with all-zero (random_operands = 0) or random
 * operand values, so a caller that times the launch learns the MFMA rate the chip sustains on such data: the clock
 * held under random operands is lower than under zeros. out: device, ZP_MFMA_PROBE_OUT_BYTES bytes, overwritten.
 * iters in [1, 2^22]. Returns -1 on a null or misaligned pointer or iters out of range,
 * else the hipError_t of the launch (0 = success). */
#define ZP_MFMA_PROBE_OUT_BYTES 262144
#define ZP_MFMA_PROBE_FLOP_PER_ITER 1073741824.0 /* 256 * 4 * 32 * 32768 */
int zp_mfma_probe(float *out, int32_t iters, int32_t random_operands, void *stream);

/* Measurement aid: per-kernel durations from hipEvents recorded on the launch stream.
 * zp_profile_enable(1) clears the records and starts recording every kernel the library launches (one
 * record per launch, in launch order); zp_profile_enable(0) stops and clears. zp_profile_get() waits for
 * record i to finish and returns its kernel label (truncated to name_cap-1 chars) and duration in ms.
 * Event creation is a host-side allocation: keep it off in production loops. */
int zp_profile_enable(int on);
int zp_profile_count(void);
int zp_profile_get(int i, char *name, int name_cap, float *ms);

#ifdef __cplusplus
}
#endif
#endif
