// Host-visible argument blocks and launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slimpipe {

// The cached keys / values as the paper stores them (Sec. 5): a list of slice-sized chunks rather than
// one buffer.  Row j of the prefix is row j % len of chunk j / len; inside a chunk rows follow the kv
// strides.  A contiguous prefix is the list of one chunk (any length).  With more than one chunk `len`
// is a multiple of 256 and the kernels walk key tiles on an absolute grid, so that no tile straddles two
// chunks.
constexpr int kMaxChunks = 64;
struct KvChunks {
  const __bf16* k[kMaxChunks];
  const __bf16* v[kMaxChunks];
  int64_t len;
  int32_t n;
};
// keys one workgroup of the dk/dv kernel owns
inline __host__ __device__ constexpr int dkdv_keys_per_workgroup() { return 8 * 32; }
// first key of the tile grid for tiles of `tile` keys
inline __host__ __device__ int64_t kv_grid_origin(int64_t kv_begin, int32_t n_chunks, int tile) {
  return n_chunks > 1 ? kv_begin / tile * tile : kv_begin;
}

// Key ranges one forward launch covers (paper Sec. 4.2.2: the pieces of a context exchange).  Range r
// of a launch writes its (out, lse) at out + r * out_range_stride, lse + r * lse_range_stride.
constexpr int kMaxRanges = 16;

struct FwdArgs {
  const __bf16* q;
  KvChunks kv;
  void* out;
  float* lse;
  int32_t s_q, n_q_heads, group, causal, out_f32;
  int32_t n_ranges;                                   // >= 1; third item coordinate = batch index * n_ranges + range
  int64_t range_begin[kMaxRanges], range_end[kMaxRanges];
  int64_t out_range_stride, lse_range_stride;         // in elements of the output type / floats
  // work items = (query block, q head, batch index x range), items[0] * [1] * [2] of them; with `ticket` (a counter
  // set to zero before the launch) the grid holds more workgroups than items and each takes the next item from the
  // counter (see BwdArgs::ticket); nullptr: workgroup index = item
  unsigned* ticket;
  int32_t items[3];
  int64_t q_offset, kv_capacity;
  float scale_log2e;
  int64_t q_stride_b, q_stride_s, q_stride_h;
  int64_t kv_stride_b, kv_stride_s, kv_stride_h;
  int64_t o_stride_b, o_stride_s, o_stride_h;
};

struct BwdArgs {
  const __bf16* q;
  KvChunks kv;
  const __bf16* out;
  const __bf16* d_out;
  const float* lse;
  float* delta;            // workspace [batch, n_q_heads, s_q]: -rowsum(dO * O) (negated: initial accumulator of dP in dk/dv)
  float* lse2;             // workspace [batch, n_q_heads, s_q]: lse * log2(e), +inf where lse = -inf
  void* dq;
  float* dk_acc[kMaxChunks];   // float32 accumulators, chunked like the keys / values
  float* dv_acc[kMaxChunks];
  float* part;             // workspace [n_split][2][batch][n_kv_heads][nkeys_pad][head_dim]: partial dk, dv (n_split > 1)
  // dq kernel: key ranges of one launch (third item coordinate = batch index * n_dq_ranges + range).  With one range dq is the
  // caller's buffer; with several it is the float32 workspace [range][batch, s_q, heads, head_dim] that
  // dq_reduce_kernel adds up into dq_final.
  int32_t n_dq_ranges;
  int64_t dq_range_begin[kMaxRanges], dq_range_end[kMaxRanges];
  int64_t dq_range_stride;                       // elements between the partial dq of two ranges
  int64_t dq_stride_b, dq_stride_s, dq_stride_h; // of `dq` as the dq kernel writes it
  void* dq_final;                                // the caller's dq (q strides) when n_dq_ranges > 1
  int32_t dq_final_f32, dq_final_accumulate;
  int32_t n_split;         // chunks the query stream of a key tile is cut into (one workgroup each)
  int64_t nkeys_pad;       // key rows per (batch, kv head) plane of `part`
  // dk/dv work items = (key tile x chunk, kv head, batch index), dkdv_items[0] * [1] * [2] of them.  With `ticket`
  // (a counter in the workspace that the delta kernel sets to zero) workgroups take the next item from the counter
  // instead of deriving it from their index: the hardware hands workgroups to the eight XCDs round-robin whatever
  // their speed, and this lets a faster XCD take more items.  The dk/dv launch then has dkdv_wgs workgroups (one per
  // compute unit) that loop over items, with ticket_dkdv[0..7] one counter per XCD; the dq launch has a quarter more
  // workgroups than items, one item each, and one counter.
  // nullptr: workgroup index = item (no room for the counter in the workspace, or no more items than compute units:
  // then every workgroup starts at once and there is nothing to even out).
  unsigned* ticket_dkdv;
  unsigned* ticket_dq;
  int32_t dkdv_wgs;
  int32_t dkdv_items[3];
  int32_t dq_items[3];      // dq work items = (query block, q head, batch index x key range), handed out the same way
  int32_t s_q, n_q_heads, n_kv_heads, group, causal;
  int32_t dq_f32, dq_accumulate, dkv_accumulate;
  int64_t q_offset, kv_begin, kv_end, kv_capacity;
  float scale, scale_log2e;
  int64_t q_stride_b, q_stride_s, q_stride_h;
  int64_t kv_stride_b, kv_stride_s, kv_stride_h;
  int64_t o_stride_b, o_stride_s, o_stride_h;
  int64_t do_stride_b, do_stride_s, do_stride_h;
};

struct MergeArgs {
  const void* outs[16];
  const float* lses[16];
  int32_t n_parts, part_f32, out_f32, head_dim, n_q_heads, s_q;
  int64_t rows;            // batch * s_q
  void* out;               // strides o_* (parts are contiguous [batch, s_q, heads, head_dim])
  float* lse;
  int64_t o_stride_b, o_stride_s, o_stride_h;
};

// The attention kernels use more than 64 KB of dynamic LDS, which a kernel has to be allowed once per device
// (hipFuncSetAttribute; the attribute belongs to the function on the CURRENT device).  These two set it for
// every instantiation of the forward / backward kernels; api.hip calls them once per device.
hipError_t opt_in_fwd_kernels();
hipError_t opt_in_bwd_kernels();

hipError_t launch_fwd(const FwdArgs& a, int batch, int head_dim, hipStream_t st);
hipError_t launch_zero_counter(unsigned* counter, hipStream_t st);
hipError_t launch_delta(const BwdArgs& a, int batch, int head_dim, hipStream_t st);
hipError_t launch_bwd_dq(const BwdArgs& a, int batch, int head_dim, hipStream_t st);
hipError_t launch_bwd_dkdv(const BwdArgs& a, int batch, int head_dim, hipStream_t st);
hipError_t launch_dkdv_reduce(const BwdArgs& a, int batch, int head_dim, hipStream_t st);
hipError_t launch_dq_reduce(const BwdArgs& a, int batch, int head_dim, hipStream_t st);
hipError_t launch_merge(const MergeArgs& a, hipStream_t st);
hipError_t launch_finalize(const float* acc, __bf16* dst, int64_t n, hipStream_t st);
hipError_t launch_dq_atomic_probe(float* dq, int s_q, int heads, int key_tiles, int rows_per_step, int placement, int rotate,
                                  int filler_mfma, int with_atomics, unsigned* xcc_mismatch, hipStream_t st);
hipError_t launch_xcd_rate(int iters, int workgroups, long long* t_start, long long* t_end, unsigned* xcc, hipStream_t st);
hipError_t launch_mfma_rate(int random, int iters, int workgroups, float* sink, hipStream_t st);

}  // namespace slimpipe
