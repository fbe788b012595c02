/*
 * slimpipe_attn.h - C ABI of the slice-wise causal attention hot path for AMD MI355X (gfx950).
 *
 * The operation is the attention step of SlimPipe's slice-wise pipeline schedule
 * (paper Sec. 4.1.2): the queries of slice i of a sequence attend causally to the cached
 * keys/values of slices 0..i, forward and backward, the backward passes of the slices running
 * in reverse order.  Any call may be restricted to a key range [kv_begin, kv_end); it then
 * returns the partial output together with the softmax normaliser of that range, which is what
 * the paper's attention context exchange (Sec. 4.2.2) and commutated context parallelism
 * (Sec. 5) ship between devices and fold together with the online-softmax merge rule.
 *
 * Conventions
 *   - All data pointers are DEVICE pointers owned by the caller.  The library allocates nothing on
 *     the device, enqueues its kernels on the caller's HIP stream (a hipStream_t passed as void*,
 *     NULL = default stream) and returns without synchronising.
 *   - State.  Per device the library remembers two facts that depend on the device alone: that its
 *     kernels have been allowed their dynamic LDS (done once, see slimpipe_attn_init) and the number of
 *     compute units.  Both are set under a once-flag / atomically, so the entry points may be called from
 *     several host threads at once (each with its own stream and buffers).  Nothing else persists
 *     between calls; the measurement aids of slimpipe_attn_bench.h keep their own records.
 *   - q, out, d_out, dq:  [batch, s_q, n_q_heads, head_dim], element strides given, head_dim contiguous.
 *   - k, v, dk_acc, dv_acc: [batch, kv_capacity, n_kv_heads, head_dim]; row j of the prefix IS global
 *     key position j (the base pointer is position 0).
 *   - lse: [batch, n_q_heads, s_q] float32, contiguous; lse = ln sum_j exp(scale * q.k_j) over the
 *     visible keys of the call (natural log, scale inside).
 *   - Key j is visible to query row r iff kv_begin <= j < kv_end and (causal == 0 or
 *     j <= q_offset + r).  A row that sees no key gets out = 0, lse = -inf and contributes no
 *     gradient.  An empty range is legal.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *   - q, k, v, d_out are bf16.  All strides are in elements, must be multiples of 8 and the base
 *     pointers 16-byte aligned.
 *   - Every function returns SLIMPIPE_OK (0) or a negative slimpipe_status; nothing is printed,
 *     nothing aborts.  Argument validation is pure host code.
 */
#ifndef SLIMPIPE_ATTN_H
#define SLIMPIPE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum slimpipe_status {
  SLIMPIPE_OK = 0,
  SLIMPIPE_EINVAL_NULL = -1,      /* a required pointer is NULL                                   */
  SLIMPIPE_EINVAL_SHAPE = -2,     /* batch/s_q/heads <= 0, Hq % Hkv != 0, head_dim not 64 or 128,  */
                                  /* scale not finite or <= 0, bad dtype code, n_parts out of range,*/
                                  /* batch or n_q_heads > 65535, more than 2^30 work items a launch */
                                  /* (ceil(s_q / 256) * n_q_heads * batch * key ranges)             */
  SLIMPIPE_EINVAL_RANGE = -3,     /* kv_begin > kv_end, kv_end > kv_capacity, negative offsets     */
  SLIMPIPE_EINVAL_STRIDE = -4,    /* a stride is not a positive multiple of 8 elements             */
  SLIMPIPE_EINVAL_ALIGN = -5,     /* a pointer is not 16-byte aligned                              */
  SLIMPIPE_EWORKSPACE = -6,       /* workspace missing or smaller than slimpipe_attn_workspace_bytes */
  SLIMPIPE_ELAUNCH = -7,          /* the HIP runtime refused a launch                              */
  SLIMPIPE_ETOOLARGE = -8         /* slimpipe_attn_bwd_noalloc: the call needs more than its fixed scratch */
} slimpipe_status;

enum { SLIMPIPE_BF16 = 0, SLIMPIPE_F32 = 1 };

typedef struct slimpipe_attn_params {
  int32_t batch;
  int32_t s_q;          /* rows of the query slice                                        */
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;     /* 64 or 128                                                      */
  int32_t causal;       /* 0 or 1                                                         */
  int64_t kv_capacity;  /* rows addressable behind k/v (and dk_acc/dv_acc)                */
  int64_t q_offset;     /* global position of query row 0                                 */
  int64_t kv_begin;     /* half-open range of global key positions this call attends to   */
  int64_t kv_end;
  float   scale;        /* softmax scale, > 0 (1/sqrt(head_dim) in every workload)        */
  int32_t out_dtype;    /* forward: dtype of `out` (SLIMPIPE_BF16, or SLIMPIPE_F32 for    */
                        /* partials that will be merged).  Ignored by backward.           */
  int64_t q_stride_b, q_stride_s, q_stride_h;     /* q and dq                              */
  int64_t kv_stride_b, kv_stride_s, kv_stride_h;  /* k, v, dk_acc, dv_acc                  */
  int64_t o_stride_b, o_stride_s, o_stride_h;     /* out                                   */
  int64_t do_stride_b, do_stride_s, do_stride_h;  /* d_out (backward only)                 */
} slimpipe_attn_params;

/* Prepares the CURRENT device (hipSetDevice) for launches: allows every kernel of the library the dynamic LDS
 * it uses (more than the 64 KB a kernel gets by default).  Thread-safe, idempotent, a few microseconds after
 * the first call.  Every launching entry point does the same on its first call on a device, so calling this is
 * optional - except before HIP graph capture: the attribute call is not a stream operation and must have happened
 * before a capture begins, so call slimpipe_attn_init() once per device first; after it a capture needs no
 * eager warm-up launch.  Returns SLIMPIPE_OK or SLIMPIPE_ELAUNCH. */
int slimpipe_attn_init(void);

/* Host-only argument check shared by every entry point (is_bwd != 0 also checks what only the
 * backward needs).  No device access. */
int slimpipe_attn_validate(const slimpipe_attn_params* p, int is_bwd);

/* Bytes of device workspace the call would like.  Forward: 256 bytes for a counter through which the workgroups take
 * their work items (see the backward below), plus, when the call is a short slice over a long cache whose query
 * blocks leave compute units idle, room for the float32 partial (out, lse) of the 2 to 16
 * key ranges of equal work the call is cut into (see slimpipe_attn_fwd).  Backward needs two floats per
 * (batch, q head, row): delta = rowsum(d_out * out) (kept negated) and lse in log2 units, each array rounded up to
 * 256 bytes; slimpipe_attn_bwd refuses less.  On top of that it can use, in this order: 256 bytes for the counters
 * through which the workgroups of the dq and dk/dv kernels take their work items (the hardware hands workgroups to the
 * chip's eight XCDs in turn whatever their speed; with counters a faster XCD takes more items; the results do
 * not depend on who computes what), and room for partial dk/dv sums: when the key tiles of a call do not fill the
 * GPU's compute units evenly, or when the counters are there and more items make for a more even finish, the query
 * rows of each key tile are cut into 2, 4 or 8 chunks that run as work items of their own, each writing float32
 * partial sums [chunk][dk, dv][batch][kv head][keys rounded up to 256][head_dim] that a second kernel adds up
 * in chunk order.  The figure returned here includes that room for the split this call would pick;
 * given less, slimpipe_attn_bwd uses the largest split that fits (down to none).  In the same way the dq
 * kernel of a short slice over a long cache is cut into 2 to 16 key ranges of equal work, as the forward is,
 * with float32 partial dq [range][batch, s_q, n_q_heads, head_dim] behind the partial dk/dv that a reduce kernel
 * adds up in range order; that room is included too and used as far as it is there. */
int slimpipe_attn_workspace_bytes(const slimpipe_attn_params* p, int is_bwd, size_t* bytes);

/* Forward of one query slice against keys [kv_begin, kv_end) of the cached prefix
 * (Sec. 4.1.2; partial ranges: Sec. 4.2.2).  Writes out (dtype p->out_dtype, strides o_*) and
 * lse [batch, n_q_heads, s_q].  Scores are never stored.
 *   workspace : may be NULL (16-byte aligned otherwise).  Its first 256 bytes, when it has them, hold the counter
 *               through which the workgroups take their work items (set to zero by a one-thread kernel ahead of
 *               the forward kernel; the results do not depend on it).  Given slimpipe_attn_workspace_bytes(p, 0)
 *               bytes, a call whose query blocks would not fill the GPU cuts [kv_begin, kv_end) into ranges of
 *               equal work (cut points on multiples of 256 keys), computes them in one launch into float32
 *               partials behind the counter and merges them (the rule of slimpipe_attn_merge) into (out, lse)
 *               in the same call; given less room it uses as many ranges as fit, down to the undivided
 *               computation. */
int slimpipe_attn_fwd(const slimpipe_attn_params* p,
                      const void* q_slice, const void* k_prefix, const void* v_prefix,
                      void* out, float* lse,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward of the same call (Sec. 4.1.2: backward per slice in reverse order, K/V kept for it).
 *   out, lse : the rows' FINAL values (for a split computation: the merged ones), out is bf16.
 *   dq       : dq_dtype SLIMPIPE_BF16 (overwritten) or SLIMPIPE_F32 (overwritten, or += when
 *              dq_accumulate != 0, which is how the partial dq of several ranges are summed).
 *              Uses the q strides.
 *   dk_acc, dv_acc : float32 with the kv strides; rows [kv_begin, kv_end) are overwritten
 *              (dkv_accumulate == 0) or incremented (!= 0); other rows are untouched.  Each row is
 *              owned by one workgroup (or a fixed number of them whose partial sums are added in a
 *              fixed order) that sums queries and the heads of a GQA group in a fixed order, so
 *              results are bit-reproducible from run to run for the same workspace size.
 * Enqueues: delta pre-pass, dq kernel, dk/dv kernel, and the reduce kernel when the stream is split. */
int slimpipe_attn_bwd(const slimpipe_attn_params* p,
                      const void* q_slice, const void* k_prefix, const void* v_prefix,
                      const void* out, const void* d_out, const float* lse,
                      void* dq, int32_t dq_dtype, int32_t dq_accumulate,
                      float* dk_acc, float* dv_acc, int32_t dkv_accumulate,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* slimpipe_attn_bwd for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and kernels as slimpipe_attn_bwd,
 * and bit for bit the results it gives with a workspace of the minimum size (the dk/dv query stream is not split,
 * dq is not cut into key ranges), but what the kernels exchange - the two row-statistic arrays (delta and lse in
 * log2 units, one float each per (batch, q head, row)) and the 256-byte counter through which workgroups take their
 * work items - lives in a fixed array of 4 MiB + 256 bytes in device memory that belongs to the library, one copy per
 * GPU, held until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no events) and does not
 * synchronise.
 *   limit : batch * n_q_heads * s_q <= slimpipe_attn_noalloc_max_rows() = 524288, each array rounded up to 256
 *           bytes; beyond that SLIMPIPE_ETOOLARGE is returned and nothing is launched.
 *   The array keeps the last call's contents; every call overwrites the entries it reads and sets the counter to
 *   zero itself (nothing has to start at zero).  All calls on one GPU share it: two calls whose kernels may overlap
 *   on one GPU (different streams, or host threads) race - serialise them, or use slimpipe_attn_bwd with a
 *   workspace each.  Graph capture: call slimpipe_attn_init() before the capture begins. */
int slimpipe_attn_bwd_noalloc(const slimpipe_attn_params* p,
                              const void* q_slice, const void* k_prefix, const void* v_prefix,
                              const void* out, const void* d_out, const float* lse,
                              void* dq, int32_t dq_dtype, int32_t dq_accumulate,
                              float* dk_acc, float* dv_acc, int32_t dkv_accumulate, void* hip_stream);
int slimpipe_attn_noalloc_max_rows(void);

/* Online-softmax merge of n_parts (1..16) partial results over disjoint key sets (Sec. 4.2.2):
 *   lse = ln sum_r exp(lse_r),  out = sum_r exp(lse_r - lse) * out_r   (weight 0 when lse_r = -inf).
 * outs / lses are HOST arrays of n_parts DEVICE pointers.  Every partial out is contiguous
 * [rows, n_q_heads, head_dim] of part_dtype, every partial lse [batch, n_q_heads, s_q] with
 * rows = batch * s_q; the merged out has dtype out_dtype and the same contiguous layout. */
int slimpipe_attn_merge(int32_t n_parts, const void* const* outs, const float* const* lses,
                        int32_t part_dtype, int32_t batch, int32_t s_q, int32_t n_q_heads,
                        int32_t head_dim, void* out, int32_t out_dtype, float* lse,
                        void* hip_stream);

/* Round float32 accumulators (dk_acc/dv_acc after the last slice's backward) to bf16, RNE.
 * Contiguous, n_elems elements.  The paper trains in bf16 and says nothing of the precision in which the
 * key/value gradients of the slices of a sequence are added up (Sec. 4.1.2 only fixes that the backward passes
 * run slice by slice); the reading taken here: float32 accumulators across the calls, in call order, and ONE
 * rounding to bf16 at the end, which is this call. */
int slimpipe_attn_finalize_bf16(const float* acc, void* dst_bf16, int64_t n_elems, void* hip_stream);

/* The same two calls with the cached keys / values given the way the paper stores them (Sec. 5): a list
 * of slice-sized chunks instead of one buffer, so that the cache grows in the forward passes and shrinks
 * in the backward passes without copies.
 *   k_chunks, v_chunks (and dk_chunks, dv_chunks) : HOST arrays of n_chunks device pointers; row j of the
 *              prefix is row j % chunk_len of chunk j / chunk_len, laid out inside the chunk with the kv
 *              strides of `p` (kv_stride_s between rows).  The arrays are read during the call only.
 *   n_chunks : 1 .. 64;  n_chunks * chunk_len >= p->kv_capacity;  with more than one chunk, chunk_len is a
 *              multiple of 256 (SLIMPIPE_EINVAL_SHAPE otherwise).  Chunks of slices the range does not
 *              touch are never dereferenced but must be non-NULL.
 * Everything else (ranges, masks, outputs, workspace, accumulation, error codes) is as in the calls above;
 * with one chunk the result is bit-identical to them. */
int slimpipe_attn_fwd_chunked(const slimpipe_attn_params* p, const void* q_slice,
                              const void* const* k_chunks, const void* const* v_chunks,
                              int32_t n_chunks, int64_t chunk_len, void* out, float* lse,
                              void* workspace, size_t workspace_bytes, void* hip_stream);
int slimpipe_attn_bwd_chunked(const slimpipe_attn_params* p, const void* q_slice,
                              const void* const* k_chunks, const void* const* v_chunks,
                              int32_t n_chunks, int64_t chunk_len,
                              const void* out, const void* d_out, const float* lse,
                              void* dq, int32_t dq_dtype, int32_t dq_accumulate,
                              float* const* dk_chunks, float* const* dv_chunks, int32_t dkv_accumulate,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* Forward of one query slice over SEVERAL key ranges in one launch (Sec. 4.2.2: the pieces a context exchange
 * cuts a slice's keys into; also how a short slice over a long cache fills the GPU).  Keys / values as a chunk
 * list as above (n_chunks = 1: one buffer).
 *   n_ranges         : 1 .. 16;  kv_begin[r] <= kv_end[r] <= p->kv_capacity (HOST arrays; p->kv_begin / kv_end
 *                      are not used).  Ranges may be empty, overlap or leave gaps: each is computed on its own.
 *   part_out, part_lse : device, float32, [n_ranges][batch, s_q, n_q_heads, head_dim] and
 *                      [n_ranges][batch, n_q_heads, s_q], contiguous: what slimpipe_attn_fwd would return for
 *                      each range with out_dtype SLIMPIPE_F32.
 *   out, lse         : both NULL (parts only), or the merged result of all ranges (out: p->out_dtype, strides
 *                      o_*), written by the merge kernel in the same call. */
int slimpipe_attn_fwd_ranges(const slimpipe_attn_params* p, const void* q_slice,
                             const void* const* k_chunks, const void* const* v_chunks,
                             int32_t n_chunks, int64_t chunk_len,
                             int32_t n_ranges, const int64_t* kv_begin, const int64_t* kv_end,
                             float* part_out, float* part_lse, void* out, float* lse, void* hip_stream);

const char* slimpipe_attn_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SLIMPIPE_ATTN_H */
