/*
 * plora_bench.h - benchmark-only hooks of libplora (not part of the layer's interface).
 *
 * Per-kernel timing for bench.py: while enabled (non-zero), every kernel class of every
 * plora_linear_* / plora_lora_* call is bracketed by a pair of HIP events recorded on the
 * call's own stream.  Enabling clears earlier records; at most 16384 brackets are kept.
 * plora_kernel_time sums the recorded durations of one class (milliseconds) and counts them; the
 * caller must have synchronised the streams first.
 * Classes: 0 base GEMM forward (with the fused expand), 1 dX GEMM (with the fused low-rank term),
 * 2 shrink, 3 dH, 4 dB, 5 dA, 6 the preparation launch (metadata, packing of A_k, conversion of a
 * saved activation), 7 the optimizer step (all launches of one plora_adamw_step call), 8 the stand-alone
 * low-rank update of plora_lora_fwd / plora_lora_bwd, 9 the expansion of an NF4 base weight.
 * Returns 0, or -1 on a bad argument or event error.  Process-global state, NOT thread-safe: one
 * benchmarking thread only, and no timed call may run concurrently with these two functions.
 */
#ifndef PLORA_BENCH_H
#define PLORA_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

void plora_set_kernel_timing(int enabled);
int plora_kernel_time(int kernel_class, float *total_ms, int *count);

#ifdef __cplusplus
}
#endif
#endif /* PLORA_BENCH_H */
