/*
 * hexgen_bench.h -- measurement-only entry points of libhexgen.so (used by bench.py, the profiles and the tests
 * that exercise every kernel instantiation).  None of them is part of the paper's statement of the problem
 * (include/hexgen.h holds those calls); they exist so that per-kernel durations, byte-counter scale factors and
 * the machine's practical HBM / MFMA ceilings can be measured through the same library the product runs.
 * Conventions (status codes, device vs host pointers, streams) as in hexgen.h.
 */
#ifndef HEXGEN_BENCH_H
#define HEXGEN_BENCH_H

#include "hexgen.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-slot timing.  While enabled, prefill / decode record HIP events on the caller's stream
 * around each projection launch, so per-kernel time can be read without an external profiler
 * (this costs a few microseconds per timed launch: enable it for measurement passes only).
 * Slots: 0 QKV projection, 1 W_O, 2 W1/W3 (+SwiGLU), 3 W2, 4 attention, 5 the whole call, 6 (decode calls of at most
 * 32 rows only) the first kernel of the W1/W3 projection alone: with 3 or more rows that projection is a split kernel
 * followed by a finishing kernel, and slot 2 brackets the pair.
 * enable(slot_mask): bit i selects slot i (0 = off, 127 = all); synchronises and clears earlier records.
 * read() synchronises and returns the summed time in milliseconds and the number of timed launches.
 */
hexgen_status_t hexgen_stage_profile_enable(hexgen_stage_t *st, int slot_mask);
hexgen_status_t hexgen_stage_profile_read(hexgen_stage_t *st, int slot, double *total_ms, int64_t *count);
/* The W1/W3 (+SwiGLU) decode projection of every layer, back to back, `reps` times over, between two HIP events on
 * `stream`: total_ms / launches is that kernel's duration without the per-launch event overhead of the slots above
 * (every launch streams a different layer's weights, as in a decode step).  Runs on the operands the last decode call
 * left in the workspace and overwrites only the workspace's FFN operand; HEXGEN_ERR_STATE before the first decode
 * call of at most 32 rows or on an fp32 stage.  Synchronises the stream.
 */
hexgen_status_t hexgen_stage_time_w13_decode(hexgen_stage_t *st, int reps, double *total_ms, int64_t *launches,
                                             void *stream);

/* HBM calibration kernels of known size (used by the benchmark and to scale profiler byte counters):
 * copy moves `bytes` (multiple of 16) from src to dst; read streams `bytes` from src and writes at most one
 * float per block to `sink` (device, >= blocks floats).  `blocks` = grid size (256-thread blocks).
 */
hexgen_status_t hexgen_stream_copy(void *dst, const void *src, int64_t bytes, int blocks, void *stream);
hexgen_status_t hexgen_stream_read(const void *src, void *sink, int64_t bytes, int blocks, void *stream);

/* Matrix-core calibration: `blocks` 4-wave blocks each run `iters` k-steps of a 128 x 128 x 32 wave tile out of
 * registers (2^20 flop per wave and iteration).  variant 0: 16x16x32 bf16 MFMA, 1: 32x32x16 bf16 MFMA, 2 / 3: the
 * same plus the LDS fragment reads a GEMM issues; 4 .. 7: variants 0 .. 3 on operands with random signs and
 * mantissas instead of 1.0 (the power the matrix cores draw, and with it the clock the chip holds, depends on the
 * operand bits; run tens of milliseconds for a steady figure).  8 .. 11: 16x16x32 on random bits with 128 result
 * registers per wave (a 64 x 128 wave tile, as the two-phase GEMM loop holds): results in accumulation registers (8, 10)
 * or in ordinary vector registers (9, 11), issued row by row (8, 9) or in a serpentine that changes one operand per
 * instruction (10, 11).  `sink`: device, >= 256 floats.  Time it with events.
 */
hexgen_status_t hexgen_mfma_probe(int variant, void *sink, int iters, int blocks, void *stream);

/* Measurement and test hook, process-wide: force one tile configuration of the prefill projection GEMM instead of
 * the choice by shape.  code names the block tile: 88 = 256 x 256 on 4 waves, 98 = 256 x 256 on 8 waves, 198 = the same
 * with the two waves of each SIMD half a k-step out of phase (the default for large launches), 194 / 184 = 128 x 256 /
 * 256 x 128 on the same two-phase loop (the defaults for launches that do not fill the chip with 198), 84 = 256 x 128,
 * 48 = 128 x 256, 94 / 49 = 128 x 256 on 8 waves (2 x 4 / 4 x 2 wave grid), 44 = 128 x 128, 72 = 448 features x 128
 * tokens on 4 waves; 0 restores the default.  (Residual-epilogue launches need 128 features per wave and fall back to
 * 84, from 194 to 184, from 72 to 198.)  HEXGEN_ERR_INVALID_ARG for any other code.
 * Codes 1198 / 2198 / 3198 are ABLATIONS of 198 for power measurements -- the same kernel without its direct-to-LDS loads
 * inside the k-loop / with loads that only re-read the first k-step (cache hits) / without its LDS operand reads.  They
 * compute garbage (all accesses in bounds): never leave one of them set.
 */
hexgen_status_t hexgen_set_gemm_tile(int code);

/* Measurement and test hook, process-wide: force the number of blocks one (sequence, kv head) pair's context is split
 * over in the decode attention (1 = one block per pair, 2..8 = split with the last block merging) instead of the
 * choice by batch and context lengths; 0 restores the default.  HEXGEN_ERR_INVALID_ARG outside 0..8. */
hexgen_status_t hexgen_set_attn_split(int nsplit);

#ifdef __cplusplus
}
#endif
#endif /* HEXGEN_BENCH_H */
