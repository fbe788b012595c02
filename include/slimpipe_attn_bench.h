/*
 * slimpipe_attn_bench.h - measurement aids of libslimpipe_attn (not part of the paper's method, not needed to
 * use the library): per-kernel event timing and the sustained rate of the matrix instruction on this GPU.
 * Used by bench.py only.  Same conventions as slimpipe_attn.h (status codes, device pointers, streams).
 */
#ifndef SLIMPIPE_ATTN_BENCH_H
#define SLIMPIPE_ATTN_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing.  While enabled, every kernel the library enqueues is bracketed by HIP events recorded on
 * the caller's stream.  slimpipe_attn_profile_read waits for the recorded events, adds up the elapsed time per
 * kernel kind since the last read and clears the records.  The records are process-wide and guarded by a mutex:
 * enabling the switch serialises the launches of concurrent host threads. */
enum {
  SLIMPIPE_KERNEL_FWD = 0, SLIMPIPE_KERNEL_DELTA = 1, SLIMPIPE_KERNEL_DQ = 2, SLIMPIPE_KERNEL_DKDV = 3,
  SLIMPIPE_KERNEL_MERGE = 4, SLIMPIPE_KERNEL_FINALIZE = 5, SLIMPIPE_KERNEL_DKDV_REDUCE = 6,
  SLIMPIPE_KERNEL_DQ_REDUCE = 7, SLIMPIPE_KERNEL_KINDS = 8
};
int slimpipe_attn_profile_enable(int enable);
int slimpipe_attn_profile_read(double total_ms[SLIMPIPE_KERNEL_KINDS], int64_t launches[SLIMPIPE_KERNEL_KINDS]);

/* The rate, in TFLOP/s, at which this GPU sustains a pure stream of the bf16 MFMA instruction the attention
 * kernels use, with constant operands (random_operands == 0) or with random ones (!= 0), under which the chip
 * is power limited and clocks lower.  Runs two short kernels (about 20 ms each) on the stream and waits for them.
 * sink: device pointer to at least one float (never written in practice). */
int slimpipe_attn_mfma_rate(int random_operands, float* sink, double* tflops, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIMPIPE_ATTN_BENCH_H */
