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

/* How evenly the XCDs of the GPU run the same work.  Launches `workgroups` workgroups of 8 waves that each issue 4 * iters
 * bf16 matrix instructions on random operands and writes, per workgroup, its start and end time (ticks of the constant
 * 100 MHz wall clock) and the XCD it ran on into the three DEVICE arrays (workgroups entries each).  Waits for the kernel.
 * The hardware hands workgroups to the XCDs round-robin whatever their speed, so a launch of equal workgroups ends when
 * the slowest XCD ends; bench.py reports the per-XCD times as `xcd_spread`. */
int slimpipe_attn_xcd_rate(int32_t iters, int32_t workgroups, int64_t* t_start, int64_t* t_end, uint32_t* xcc, void* hip_stream);

/* What float32 atomic adds into dq would cost a backward kernel that computes the scores once (key-stationary, dK/dV
 * in registers, dQ added into memory).  Launches key_tiles * heads workgroups of 8 waves; each walks the s_q /
 * rows_per_step query tiles of one head and per tile adds 1.0f to a rows_per_step x 128 block of dq
 * ([s_q, heads, 128] float32, device, zero before the call) as eight 32 x 32 MFMA C tiles with head_dim along the
 * lanes (rows_per_step = 32: two waves per tile add to the same 32 rows; 64: each wave its own 32 rows), with
 * filler_mfma (multiple of 4) matrix instructions per wave and step in between, and with_atomics = 0 leaving the
 * adds out.  placement 0: consecutive workgroups share a head; 1: workgroup w takes head w % heads and counts in
 * *xcc_mismatch (device, zero before the call) the workgroups whose XCD differs from w % 8.  rotate != 0 shifts the
 * start tile by the workgroup's key tile.  Afterwards every element of dq holds key_tiles * (64 / rows_per_step).
 * Waits for the kernel; *ms = its duration. */
int slimpipe_attn_dq_atomic_probe(float* dq, int32_t s_q, int32_t heads, int32_t key_tiles, int32_t rows_per_step,
                                  int32_t placement, int32_t rotate, int32_t filler_mfma, int32_t with_atomics,
                                  uint32_t* xcc_mismatch, double* ms, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIMPIPE_ATTN_BENCH_H */
