// C ABI of the library: host-only validation, launch planning, error mapping.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/slimpipe_attn.h"
#include "../../include/slimpipe_attn_bench.h"
#include "kernels.hpp"

using namespace slimpipe;

// Fixed device memory of the entry point that allocates nothing (slimpipe_attn_bwd_noalloc): the backward's row
// statistics live here instead of in a caller's workspace.  Every GPU the library runs on holds its own copy
// until the process ends.  Host code never uses this name as an address: it asks the runtime for the device
// address once per device (ensure_device_ready) and passes that pointer to the kernels.
constexpr size_t kScratchBytes = (size_t)4 << 20;          // the two statistics arrays
constexpr size_t kScratchTicketBytes = 256;                // + the counter the workgroups take their work items from
static __device__ __align__(256) unsigned char scratch[kScratchBytes + kScratchTicketBytes];

namespace {

bool stride_ok(int64_t s) { return s > 0 && (s % 8) == 0; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// one float array per row statistic (delta, lse in log2 units), each rounded up to 256 bytes
size_t stat_bytes(const slimpipe_attn_params* p) {
  size_t n = (size_t)p->batch * (size_t)p->n_q_heads * (size_t)p->s_q * sizeof(float);
  return (n + 255) & ~(size_t)255;
}
size_t delta_bytes(const slimpipe_attn_params* p) { return 2 * stat_bytes(p); }

// ---- per-device state: the only state the library keeps besides the benchmark's profiling switch ----
// For each device the dynamic-LDS opt-in of the kernels (done once, under std::call_once) and the number of
// compute units.  Both are functions of the device alone, so concurrent callers agree on them.
constexpr int kMaxDevices = 64;
struct DeviceState {
  std::once_flag once;
  hipError_t status = hipSuccess;
  void* scratch = nullptr;       // this device's copy of `scratch` below (its address differs from device to device)
};
DeviceState g_device[kMaxDevices];
std::atomic<int> g_compute_units[kMaxDevices];

// Makes the current device ready for launches: SLIMPIPE_OK, or SLIMPIPE_ELAUNCH when the runtime refuses.
int ensure_device_ready(void** scratch_ptr = nullptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SLIMPIPE_ELAUNCH;
  DeviceState& d = g_device[dev];
  std::call_once(d.once, [&d] {
    d.status = opt_in_fwd_kernels();
    if (d.status == hipSuccess) d.status = opt_in_bwd_kernels();
    if (d.status == hipSuccess) d.status = hipGetSymbolAddress(&d.scratch, HIP_SYMBOL(scratch));
    if (d.status == hipSuccess && d.scratch == nullptr) d.status = hipErrorInvalidSymbol;
  });
  if (scratch_ptr) *scratch_ptr = d.scratch;
  return d.status == hipSuccess ? SLIMPIPE_OK : SLIMPIPE_ELAUNCH;
}

// Compute units of the current device (256 on MI355X, also assumed when no device can be asked, so that the
// workspace query stays a pure host function).
int compute_units() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  int cus = g_compute_units[dev].load(std::memory_order_relaxed);
  if (cus > 0) return cus;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
  g_compute_units[dev].store(cus, std::memory_order_relaxed);
  return cus;
}

// The dk/dv kernel runs one workgroup per compute unit; a call with W key tiles takes ceil(W / CUs)
// rounds of one tile's query stream each.  Cutting every stream into S chunks makes W*S workgroups of
// 1/S the length: S is the smallest of 1, 2, 4, 8 that comes within 3% of the best rounds/S, as long
// as a chunk keeps at least 64 query tiles (the prologue and epilogue of a workgroup cost a few tiles).
int64_t dkdv_key_tiles(const slimpipe_attn_params* p, int n_chunks) {
  if (p->kv_end <= p->kv_begin) return 0;
  const int64_t per = dkdv_keys_per_workgroup();
  return (p->kv_end - kv_grid_origin(p->kv_begin, n_chunks, (int)per) + per - 1) / per;
}
int preferred_split(const slimpipe_attn_params* p, int n_chunks, bool ticket) {
  const int64_t tiles = dkdv_key_tiles(p, n_chunks);
  const int64_t w = tiles * p->n_kv_heads * p->batch;
  if (w <= 0) return 1;
  const int64_t stream = ((int64_t)p->s_q + 31) / 32 * (p->n_q_heads / p->n_kv_heads);
  const int cus = compute_units();
  double best = 1e30;
  double cost[4];
  for (int i = 0; i < 4; ++i) {
    const int s = 1 << i;
    cost[i] = (s > 1 && stream / s < 64) ? 1e30 : (double)((w * s + cus - 1) / cus) / s;
    if (cost[i] < best) best = cost[i];
  }
  int split = 1;
  for (int i = 3; i >= 0; --i)
    if (cost[i] <= best * 1.03) split = 1 << i;
  // Items handed out through a counter: a compute unit that finishes early takes another one, so more items even out
  // compute units (and XCDs) of unequal speed and key tiles of unequal streams (the causal diagonal).  Up to about 8
  // items per compute unit, as long as a chunk keeps at least 512 query tiles (a workgroup's prologue and epilogue
  // cost about 8 tiles' time, and every chunk adds a plane of partial sums to the reduce kernel's work).
  // And no split for the sake of whole rounds once there are two items per compute unit anyway: the counter evens out
  // most of what the rounding would cost, and the partial sums with their reduce kernel cost more than the rest.
  if (ticket) {
    if (w >= 2 * (int64_t)cus) split = 1;
    while (split < 8 && w * split < 8 * (int64_t)cus && stream / (2 * split) >= 512) split *= 2;
  }
  return split;
}
// room for the ticket counter of the dk/dv kernel behind the two statistics arrays
constexpr size_t kTicketBytes = 256;
size_t split_bytes(const slimpipe_attn_params* p, int n_chunks, int split) {
  if (split <= 1) return 0;
  return (size_t)split * 2 * (size_t)p->batch * (size_t)p->n_kv_heads *
         (size_t)(dkdv_key_tiles(p, n_chunks) * dkdv_keys_per_workgroup()) * (size_t)p->head_dim * sizeof(float);
}

// ---- key ranges of one forward launch --------------------------------------------------------------
// Visible (query, key) pairs of the call with keys in [p->kv_begin, e).
double visible_pairs_upto(const slimpipe_attn_params* p, int64_t e) {
  if (e > p->kv_end) e = p->kv_end;
  if (e <= p->kv_begin) return 0.0;
  const int64_t s = p->s_q;
  if (!p->causal) return (double)s * (double)(e - p->kv_begin);
  // row i sees keys below q_offset + i + 1: rows from i0 on see all of [kv_begin, e), rows i1 .. i0-1 a part
  int64_t i0 = e - p->q_offset - 1;
  i0 = i0 < 0 ? 0 : (i0 > s ? s : i0);
  int64_t i1 = p->kv_begin - p->q_offset;
  i1 = i1 < 0 ? 0 : (i1 > i0 ? i0 : i1);
  const double full = (double)(s - i0) * (double)(e - p->kv_begin);
  const double cnt = (double)(i0 - i1);
  const double first = (double)(p->q_offset + i1 + 1 - p->kv_begin), last = (double)(p->q_offset + i0 - p->kv_begin);
  return full + (cnt > 0 ? 0.5 * cnt * (first + last) : 0.0);
}

// One forward workgroup owns 256 query rows of one head and walks the whole key range; a short slice over a
// long cache leaves compute units idle.  Cutting the key range into R ranges of equal work (one launch,
// partial (out, lse) per range, then the online-softmax merge) makes R times the workgroups: R is the
// smallest count that comes within 3% of the best rounds/R, as long as a range keeps at least 1024 keys.
int fwd_preferred_ranges(const slimpipe_attn_params* p) {
  const int64_t w = (((int64_t)p->s_q + 255) / 256) * p->n_q_heads * p->batch;
  const int64_t keys = p->kv_end - p->kv_begin;
  if (w <= 0 || keys <= 0) return 1;
  const int cus = compute_units();
  double best = 1e30, cost[kMaxRanges + 1];
  for (int r = 1; r <= kMaxRanges; ++r) {
    // (a range keeps at least 1024 keys; batch * ranges is the grid's z dimension)
    cost[r] = (r > 1 && (keys / r < 1024 || (int64_t)p->batch * r > 65535)) ? 1e30 : (double)((w * r + cus - 1) / cus) / r;
    if (cost[r] < best) best = cost[r];
  }
  for (int r = 1; r <= kMaxRanges; ++r)
    if (cost[r] <= best * 1.03) return r;
  return 1;
}
size_t fwd_part_out_bytes(const slimpipe_attn_params* p) {
  size_t n = (size_t)p->batch * (size_t)p->s_q * (size_t)p->n_q_heads * (size_t)p->head_dim * sizeof(float);
  return (n + 255) & ~(size_t)255;
}
size_t fwd_parts_bytes(const slimpipe_attn_params* p, int ranges) {
  return ranges <= 1 ? 0 : (size_t)ranges * (fwd_part_out_bytes(p) + stat_bytes(p));
}
// The dq kernel has the forward's launch shape and is cut into key ranges the same way; its partial results are
// float32 [range][batch, s_q, heads, head_dim].
size_t dq_parts_bytes(const slimpipe_attn_params* p, int ranges) {
  return ranges <= 1 ? 0 : (size_t)ranges * fwd_part_out_bytes(p);
}
// Cut points of equal work on multiples of 256 keys (no range boundary inside a chunk-grid tile).
void equal_work_ranges(const slimpipe_attn_params* p, int ranges, int64_t* begin, int64_t* end) {
  const double total = visible_pairs_upto(p, p->kv_end);
  int64_t prev = p->kv_begin;
  for (int r = 0; r < ranges; ++r) {
    int64_t cut = p->kv_end;
    if (r + 1 < ranges) {
      const double want = total * (double)(r + 1) / (double)ranges;
      int64_t lo = prev / 256, hi = (p->kv_end + 255) / 256;        // smallest multiple of 256 with enough pairs below it
      while (lo < hi) {
        const int64_t mid = (lo + hi) / 2;
        if (visible_pairs_upto(p, mid * 256) >= want) hi = mid; else lo = mid + 1;
      }
      cut = lo * 256;
      if (cut < prev) cut = prev;
      if (cut > p->kv_end) cut = p->kv_end;
    }
    begin[r] = prev;
    end[r] = cut;
    prev = cut;
  }
}

// A chunk list is legal when it covers kv_capacity rows; with more than one chunk the chunk length is a
// multiple of the dk/dv key tile (256), so that no key tile of any kernel straddles two chunks.
int check_chunks(const slimpipe_attn_params* p, int32_t n_chunks, int64_t chunk_len) {
  if (n_chunks < 1 || n_chunks > kMaxChunks || chunk_len < 1) return SLIMPIPE_EINVAL_SHAPE;
  if (n_chunks * chunk_len < p->kv_capacity) return SLIMPIPE_EINVAL_RANGE;
  if (n_chunks > 1 && chunk_len % dkdv_keys_per_workgroup() != 0) return SLIMPIPE_EINVAL_SHAPE;
  return SLIMPIPE_OK;
}



// ---- optional per-kernel event timing (benchmark aid) ----------------------------------------------
struct ProfRecord { int kind; hipEvent_t start, stop; };
std::atomic<bool> g_prof_on{false};
std::mutex g_prof_mutex;                     // guards the two vectors
std::vector<ProfRecord> g_prof_records;
std::vector<hipEvent_t> g_prof_free;

hipEvent_t prof_event() {                    // (caller holds g_prof_mutex)
  if (!g_prof_free.empty()) { hipEvent_t e = g_prof_free.back(); g_prof_free.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

template <class F>
hipError_t timed(int kind, hipStream_t st, F&& launch, bool allow = true) {
  if (!allow || !g_prof_on.load(std::memory_order_relaxed)) return launch();
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  ProfRecord r{kind, prof_event(), prof_event()};
  if (!r.start || !r.stop) return launch();
  (void)hipEventRecord(r.start, st);
  hipError_t e = launch();
  (void)hipEventRecord(r.stop, st);
  g_prof_records.push_back(r);
  return e;
}

}  // namespace

extern "C" {

int slimpipe_attn_init(void) { return ensure_device_ready(); }

int slimpipe_attn_profile_enable(int enable) {
  g_prof_on.store(enable != 0, std::memory_order_relaxed);
  return SLIMPIPE_OK;
}

int slimpipe_attn_profile_read(double total_ms[SLIMPIPE_KERNEL_KINDS], int64_t launches[SLIMPIPE_KERNEL_KINDS]) {
  if (!total_ms || !launches) return SLIMPIPE_EINVAL_NULL;
  for (int i = 0; i < SLIMPIPE_KERNEL_KINDS; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  int rc = SLIMPIPE_OK;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  for (const ProfRecord& r : g_prof_records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
      rc = SLIMPIPE_ELAUNCH;
    else if (r.kind >= 0 && r.kind < SLIMPIPE_KERNEL_KINDS) { total_ms[r.kind] += ms; launches[r.kind] += 1; }
    g_prof_free.push_back(r.start);
    g_prof_free.push_back(r.stop);
  }
  g_prof_records.clear();
  return rc;
}

int slimpipe_attn_validate(const slimpipe_attn_params* p, int is_bwd) {
  if (!p) return SLIMPIPE_EINVAL_NULL;
  if (p->batch <= 0 || p->s_q <= 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0) return SLIMPIPE_EINVAL_SHAPE;
  if (p->n_q_heads % p->n_kv_heads != 0) return SLIMPIPE_EINVAL_SHAPE;
  if (p->head_dim != 64 && p->head_dim != 128) return SLIMPIPE_EINVAL_SHAPE;
  if (!(p->scale > 0.0f) || !isfinite(p->scale)) return SLIMPIPE_EINVAL_SHAPE;
  if (p->causal != 0 && p->causal != 1) return SLIMPIPE_EINVAL_SHAPE;
  if (p->out_dtype != SLIMPIPE_BF16 && p->out_dtype != SLIMPIPE_F32) return SLIMPIPE_EINVAL_SHAPE;
  if (p->batch > 65535 || p->n_q_heads > 65535) return SLIMPIPE_EINVAL_SHAPE;   /* limits stated in the header */
  if (p->kv_capacity < 0 || p->q_offset < 0 || p->kv_begin < 0) return SLIMPIPE_EINVAL_RANGE;
  if (p->kv_begin > p->kv_end || p->kv_end > p->kv_capacity) return SLIMPIPE_EINVAL_RANGE;
  if (p->q_offset > (int64_t)1 << 40 || p->kv_capacity > (int64_t)1 << 40) return SLIMPIPE_EINVAL_RANGE;
  const int64_t s[9] = {p->q_stride_b, p->q_stride_s, p->q_stride_h, p->kv_stride_b, p->kv_stride_s,
                        p->kv_stride_h, p->o_stride_b, p->o_stride_s, p->o_stride_h};
  for (int i = 0; i < 9; ++i)
    if (!stride_ok(s[i])) return SLIMPIPE_EINVAL_STRIDE;
  if (is_bwd && (!stride_ok(p->do_stride_b) || !stride_ok(p->do_stride_s) || !stride_ok(p->do_stride_h) ||
                 p->do_stride_h < p->head_dim))
    return SLIMPIPE_EINVAL_STRIDE;
  if (p->q_stride_h < p->head_dim || p->kv_stride_h < p->head_dim || p->o_stride_h < p->head_dim)
    return SLIMPIPE_EINVAL_STRIDE;
  /* row strides enter 32-bit byte offsets inside a tile */
  if (p->q_stride_s >= (1 << 22) || p->kv_stride_s >= (1 << 22) || p->o_stride_s >= (1 << 22) ||
      (is_bwd && p->do_stride_s >= (1 << 22)))
    return SLIMPIPE_EINVAL_STRIDE;
  return SLIMPIPE_OK;
}

int slimpipe_attn_workspace_bytes(const slimpipe_attn_params* p, int is_bwd, size_t* bytes) {
  if (!bytes) return SLIMPIPE_EINVAL_NULL;
  int rc = slimpipe_attn_validate(p, is_bwd);
  if (rc != SLIMPIPE_OK) return rc;
  if (!is_bwd) { *bytes = kTicketBytes + fwd_parts_bytes(p, fwd_preferred_ranges(p)); return SLIMPIPE_OK; }
  // the tile grid of a chunked call can start up to 255 keys before kv_begin: room for whichever of the
  // two variants asks for more
  const size_t one = split_bytes(p, 1, preferred_split(p, 1, true)), many = split_bytes(p, 2, preferred_split(p, 2, true));
  *bytes = delta_bytes(p) + kTicketBytes + (one > many ? one : many) + dq_parts_bytes(p, fwd_preferred_ranges(p));
  return SLIMPIPE_OK;
}

// Forward over `n_ranges` key ranges in one launch.  With parts == nullptr there is one range and the result
// goes straight to (out, lse); otherwise range r writes float32 partials at part_out + r * part_out_elems,
// part_lse + r * part_lse_elems (contiguous [batch, s_q, heads, head_dim] / [batch, heads, s_q]) and, when
// `out` is given, the merge kernel folds them into (out, lse).
static int fwd_impl(const slimpipe_attn_params* p, const void* q_slice, const void* const* k_chunks,
                    const void* const* v_chunks, int32_t n_chunks, int64_t chunk_len, int32_t n_ranges,
                    const int64_t* range_begin, const int64_t* range_end, float* part_out, int64_t part_out_elems,
                    float* part_lse, int64_t part_lse_elems, void* out, float* lse, void* hip_stream, unsigned* ticket = nullptr) {
  int rc = slimpipe_attn_validate(p, 0);
  if (rc != SLIMPIPE_OK) return rc;
  const bool parts = part_out != nullptr;
  if (!q_slice || !k_chunks || !v_chunks || !range_begin || !range_end) return SLIMPIPE_EINVAL_NULL;
  if (parts ? !part_lse || ((out == nullptr) != (lse == nullptr)) : (!out || !lse)) return SLIMPIPE_EINVAL_NULL;
  if (n_ranges < 1 || n_ranges > kMaxRanges || (!parts && n_ranges != 1)) return SLIMPIPE_EINVAL_SHAPE;
  if ((int64_t)p->batch * n_ranges > 65535) return SLIMPIPE_EINVAL_SHAPE;
  rc = check_chunks(p, n_chunks, chunk_len);
  if (rc != SLIMPIPE_OK) return rc;
  if (!aligned16(q_slice) || (out && (!aligned16(out) || (reinterpret_cast<uintptr_t>(lse) & 3u)))) return SLIMPIPE_EINVAL_ALIGN;
  if (parts && (!aligned16(part_out) || (reinterpret_cast<uintptr_t>(part_lse) & 3u) || part_out_elems % 4 != 0)) return SLIMPIPE_EINVAL_ALIGN;
  FwdArgs a;
  memset(&a.kv, 0, sizeof(a.kv));
  int64_t last_key = 0;
  for (int r = 0; r < kMaxRanges; ++r) {
    a.range_begin[r] = a.range_end[r] = 0;
    if (r >= n_ranges) continue;
    if (range_begin[r] < 0 || range_begin[r] > range_end[r] || range_end[r] > p->kv_capacity) return SLIMPIPE_EINVAL_RANGE;
    a.range_begin[r] = range_begin[r];
    a.range_end[r] = range_end[r];
    if (range_end[r] > last_key) last_key = range_end[r];
  }
  for (int i = 0; i < n_chunks; ++i) {
    if (last_key > 0 && (!k_chunks[i] || !v_chunks[i])) return SLIMPIPE_EINVAL_NULL;
    if (!aligned16(k_chunks[i]) || !aligned16(v_chunks[i])) return SLIMPIPE_EINVAL_ALIGN;
    a.kv.k[i] = static_cast<const __bf16*>(k_chunks[i]);
    a.kv.v[i] = static_cast<const __bf16*>(v_chunks[i]);
  }
  a.kv.len = chunk_len;
  a.kv.n = n_chunks;
  a.q = static_cast<const __bf16*>(q_slice);
  a.n_ranges = n_ranges;
  a.s_q = p->s_q; a.n_q_heads = p->n_q_heads; a.group = p->n_q_heads / p->n_kv_heads;
  a.causal = p->causal;
  a.q_offset = p->q_offset; a.kv_capacity = p->kv_capacity;
  a.scale_log2e = p->scale * 1.4426950408889634f;
  a.q_stride_b = p->q_stride_b; a.q_stride_s = p->q_stride_s; a.q_stride_h = p->q_stride_h;
  a.kv_stride_b = p->kv_stride_b; a.kv_stride_s = p->kv_stride_s; a.kv_stride_h = p->kv_stride_h;
  if (parts) {
    a.out = part_out; a.lse = part_lse; a.out_f32 = 1;
    a.out_range_stride = part_out_elems; a.lse_range_stride = part_lse_elems;
    a.o_stride_h = p->head_dim; a.o_stride_s = (int64_t)p->n_q_heads * p->head_dim; a.o_stride_b = a.o_stride_s * p->s_q;
  } else {
    a.out = out; a.lse = lse; a.out_f32 = (p->out_dtype == SLIMPIPE_F32);
    a.out_range_stride = 0; a.lse_range_stride = 0;
    a.o_stride_b = p->o_stride_b; a.o_stride_s = p->o_stride_s; a.o_stride_h = p->o_stride_h;
  }
  a.items[0] = (p->s_q + 255) / 256;
  a.items[1] = p->n_q_heads;
  a.items[2] = p->batch * n_ranges;
  if ((int64_t)a.items[0] * a.items[1] * a.items[2] > (int64_t)1 << 30) return SLIMPIPE_EINVAL_SHAPE;
  // a counter only where there are more items than compute units (otherwise every workgroup starts at once)
  if ((int64_t)a.items[0] * a.items[1] * a.items[2] <= compute_units()) ticket = nullptr;
  a.ticket = ticket;
  if (ensure_device_ready() != SLIMPIPE_OK) return SLIMPIPE_ELAUNCH;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (ticket && launch_zero_counter(ticket, st) != hipSuccess) return SLIMPIPE_ELAUNCH;
  hipError_t e = timed(SLIMPIPE_KERNEL_FWD, st, [&] { return launch_fwd(a, p->batch, p->head_dim, st); });
  if (e != hipSuccess) return SLIMPIPE_ELAUNCH;
  if (parts && out) {
    MergeArgs m;
    memset(&m, 0, sizeof(m));
    for (int r = 0; r < n_ranges; ++r) {
      m.outs[r] = part_out + (int64_t)r * part_out_elems;
      m.lses[r] = part_lse + (int64_t)r * part_lse_elems;
    }
    m.n_parts = n_ranges; m.part_f32 = 1; m.out_f32 = (p->out_dtype == SLIMPIPE_F32);
    m.head_dim = p->head_dim; m.n_q_heads = p->n_q_heads; m.s_q = p->s_q; m.rows = (int64_t)p->batch * p->s_q;
    m.out = out; m.lse = lse;
    m.o_stride_b = p->o_stride_b; m.o_stride_s = p->o_stride_s; m.o_stride_h = p->o_stride_h;
    e = timed(SLIMPIPE_KERNEL_MERGE, st, [&] { return launch_merge(m, st); });
    if (e != hipSuccess) return SLIMPIPE_ELAUNCH;
  }
  return SLIMPIPE_OK;
}

// One range, or - when the caller lends a workspace and the launch would leave compute units idle - the
// range cut into pieces of equal work whose partial results are merged in the same call.
static int fwd_auto(const slimpipe_attn_params* p, const void* q_slice, const void* const* k_chunks,
                    const void* const* v_chunks, int32_t n_chunks, int64_t chunk_len, void* out, float* lse,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = slimpipe_attn_validate(p, 0);
  if (rc != SLIMPIPE_OK) return rc;
  // workspace: [ticket counter, 256 bytes][partial out of the ranges][partial lse of the ranges]
  if (workspace && !aligned16(workspace)) return SLIMPIPE_EINVAL_ALIGN;
  unsigned* ticket = (workspace && workspace_bytes >= kTicketBytes) ? static_cast<unsigned*>(workspace) : nullptr;
  char* parts_base = ticket ? static_cast<char*>(workspace) + kTicketBytes : static_cast<char*>(workspace);
  const size_t parts_room = ticket ? workspace_bytes - kTicketBytes : workspace_bytes;
  int ranges = workspace ? fwd_preferred_ranges(p) : 1;
  while (ranges > 1 && (fwd_parts_bytes(p, ranges) > parts_room || (int64_t)p->batch * ranges > 65535)) --ranges;
  if (ranges <= 1)
    return fwd_impl(p, q_slice, k_chunks, v_chunks, n_chunks, chunk_len, 1, &p->kv_begin, &p->kv_end, nullptr, 0, nullptr, 0, out,
                    lse, hip_stream, ticket);
  int64_t begin[kMaxRanges], end[kMaxRanges];
  equal_work_ranges(p, ranges, begin, end);
  float* part_out = reinterpret_cast<float*>(parts_base);
  float* part_lse = reinterpret_cast<float*>(parts_base + (size_t)ranges * fwd_part_out_bytes(p));
  return fwd_impl(p, q_slice, k_chunks, v_chunks, n_chunks, chunk_len, ranges, begin, end, part_out,
                  (int64_t)(fwd_part_out_bytes(p) / sizeof(float)), part_lse, (int64_t)(stat_bytes(p) / sizeof(float)), out, lse,
                  hip_stream, ticket);
}

int slimpipe_attn_fwd(const slimpipe_attn_params* p, const void* q_slice, const void* k_prefix,
                      const void* v_prefix, void* out, float* lse, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  if (!p) return SLIMPIPE_EINVAL_NULL;
  return fwd_auto(p, q_slice, &k_prefix, &v_prefix, 1, p->kv_capacity > 0 ? p->kv_capacity : 1, out, lse, workspace,
                  workspace_bytes, hip_stream);
}

int slimpipe_attn_fwd_chunked(const slimpipe_attn_params* p, const void* q_slice, const void* const* k_chunks,
                              const void* const* v_chunks, int32_t n_chunks, int64_t chunk_len, void* out, float* lse,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p) return SLIMPIPE_EINVAL_NULL;
  return fwd_auto(p, q_slice, k_chunks, v_chunks, n_chunks, chunk_len, out, lse, workspace, workspace_bytes, hip_stream);
}

int slimpipe_attn_fwd_ranges(const slimpipe_attn_params* p, const void* q_slice, const void* const* k_chunks,
                             const void* const* v_chunks, int32_t n_chunks, int64_t chunk_len, int32_t n_ranges,
                             const int64_t* kv_begin, const int64_t* kv_end, float* part_out, float* part_lse, void* out,
                             float* lse, void* hip_stream) {
  if (!p) return SLIMPIPE_EINVAL_NULL;
  if (!part_out || !part_lse) return SLIMPIPE_EINVAL_NULL;
  const int64_t out_elems = (int64_t)p->batch * p->s_q * p->n_q_heads * p->head_dim;
  const int64_t lse_elems = (int64_t)p->batch * p->n_q_heads * p->s_q;
  return fwd_impl(p, q_slice, k_chunks, v_chunks, n_chunks, chunk_len, n_ranges, kv_begin, kv_end, part_out, out_elems, part_lse,
                  lse_elems, out, lse, hip_stream);
}

static int bwd_impl(const slimpipe_attn_params* p, const void* q_slice, const void* const* k_chunks,
                    const void* const* v_chunks, int32_t n_chunks, int64_t chunk_len, const void* out,
                    const void* d_out, const float* lse, void* dq, int32_t dq_dtype, int32_t dq_accumulate,
                    float* const* dk_chunks, float* const* dv_chunks, int32_t dkv_accumulate, void* workspace,
                    size_t workspace_bytes, void* hip_stream, bool events = true) {
  int rc = slimpipe_attn_validate(p, 1);
  if (rc != SLIMPIPE_OK) return rc;
  if (!q_slice || !out || !d_out || !lse || !dq || !k_chunks || !v_chunks || !dk_chunks || !dv_chunks) return SLIMPIPE_EINVAL_NULL;
  rc = check_chunks(p, n_chunks, chunk_len);
  if (rc != SLIMPIPE_OK) return rc;
  if (dq_dtype != SLIMPIPE_BF16 && dq_dtype != SLIMPIPE_F32) return SLIMPIPE_EINVAL_SHAPE;
  if (dq_accumulate && dq_dtype != SLIMPIPE_F32) return SLIMPIPE_EINVAL_SHAPE;
  if (!aligned16(q_slice) || !aligned16(out) || !aligned16(d_out) || !aligned16(dq) || (reinterpret_cast<uintptr_t>(lse) & 3u))
    return SLIMPIPE_EINVAL_ALIGN;
  if (!workspace || workspace_bytes < delta_bytes(p)) return SLIMPIPE_EWORKSPACE;
  if (!aligned16(workspace)) return SLIMPIPE_EINVAL_ALIGN;
  BwdArgs a;
  memset(&a.kv, 0, sizeof(a.kv));
  memset(a.dk_acc, 0, sizeof(a.dk_acc));
  memset(a.dv_acc, 0, sizeof(a.dv_acc));
  for (int i = 0; i < n_chunks; ++i) {
    if (!dk_chunks[i] || !dv_chunks[i]) return SLIMPIPE_EINVAL_NULL;
    if (p->kv_end > 0 && (!k_chunks[i] || !v_chunks[i])) return SLIMPIPE_EINVAL_NULL;
    if (!aligned16(k_chunks[i]) || !aligned16(v_chunks[i]) || !aligned16(dk_chunks[i]) || !aligned16(dv_chunks[i])) return SLIMPIPE_EINVAL_ALIGN;
    a.kv.k[i] = static_cast<const __bf16*>(k_chunks[i]);
    a.kv.v[i] = static_cast<const __bf16*>(v_chunks[i]);
    a.dk_acc[i] = dk_chunks[i];
    a.dv_acc[i] = dv_chunks[i];
  }
  a.kv.len = chunk_len;
  a.kv.n = n_chunks;
  a.q = static_cast<const __bf16*>(q_slice);
  a.out = static_cast<const __bf16*>(out);
  a.d_out = static_cast<const __bf16*>(d_out);
  a.lse = lse;
  a.delta = static_cast<float*>(workspace);
  a.lse2 = reinterpret_cast<float*>(static_cast<char*>(workspace) + stat_bytes(p));
  // behind the statistics: the ticket counter of the dk/dv kernel (when there is room for it), the partial dk/dv sums
  // of a split query stream, the partial dq of key ranges
  const bool ticket = workspace_bytes >= delta_bytes(p) + kTicketBytes;
  const size_t fixed = delta_bytes(p) + (ticket ? kTicketBytes : 0);
  unsigned* const counters = ticket ? reinterpret_cast<unsigned*>(static_cast<char*>(workspace) + delta_bytes(p)) : nullptr;
  int split = preferred_split(p, n_chunks, ticket);
  while (split > 1 && fixed + split_bytes(p, n_chunks, split) > workspace_bytes) split /= 2;
  a.n_split = split;
  a.part = reinterpret_cast<float*>(static_cast<char*>(workspace) + fixed);
  // what is left of the workspace takes the partial dq of as many key ranges as fit
  const size_t used = fixed + split_bytes(p, n_chunks, split);
  int dq_ranges = fwd_preferred_ranges(p);
  while (dq_ranges > 1 && (used + dq_parts_bytes(p, dq_ranges) > workspace_bytes || (int64_t)p->batch * dq_ranges > 65535)) --dq_ranges;
  a.n_dq_ranges = dq_ranges;
  for (int r = 0; r < kMaxRanges; ++r) a.dq_range_begin[r] = a.dq_range_end[r] = 0;
  if (dq_ranges > 1) {
    equal_work_ranges(p, dq_ranges, a.dq_range_begin, a.dq_range_end);
    a.dq = static_cast<char*>(workspace) + used;
    a.dq_range_stride = (int64_t)(fwd_part_out_bytes(p) / sizeof(float));
    a.dq_stride_h = p->head_dim; a.dq_stride_s = (int64_t)p->n_q_heads * p->head_dim; a.dq_stride_b = a.dq_stride_s * p->s_q;
  } else {
    a.dq_range_begin[0] = p->kv_begin; a.dq_range_end[0] = p->kv_end;
    a.dq = dq;
    a.dq_range_stride = 0;
    a.dq_stride_b = p->q_stride_b; a.dq_stride_s = p->q_stride_s; a.dq_stride_h = p->q_stride_h;
  }
  a.dq_final = dq;
  a.dq_final_f32 = (dq_dtype == SLIMPIPE_F32); a.dq_final_accumulate = dq_accumulate ? 1 : 0;
  a.nkeys_pad = dkdv_key_tiles(p, n_chunks) * dkdv_keys_per_workgroup();
  a.dkdv_items[0] = (int32_t)(dkdv_key_tiles(p, n_chunks) * split);
  a.dkdv_items[1] = p->n_kv_heads;
  a.dkdv_items[2] = p->batch;
  a.dq_items[0] = (p->s_q + 255) / 256;
  a.dq_items[1] = p->n_q_heads;
  a.dq_items[2] = p->batch * dq_ranges;
  if ((int64_t)a.dq_items[0] * a.dq_items[1] * a.dq_items[2] > (int64_t)1 << 30) return SLIMPIPE_EINVAL_SHAPE;
  // a counter only where there are more items than compute units (otherwise every workgroup starts at once)
  const int64_t cus = compute_units();
  a.dkdv_wgs = (int32_t)cus;
  a.ticket_dkdv = (counters && (int64_t)a.dkdv_items[0] * a.dkdv_items[1] * a.dkdv_items[2] > cus) ? counters : nullptr;
  a.ticket_dq = (counters && (int64_t)a.dq_items[0] * a.dq_items[1] * a.dq_items[2] > cus) ? counters + 8 : nullptr;     // [0..7]: dk/dv, one per XCD
  if ((int64_t)a.dkdv_items[0] * a.dkdv_items[1] * a.dkdv_items[2] > (int64_t)1 << 30) return SLIMPIPE_EINVAL_SHAPE;
  a.s_q = p->s_q; a.n_q_heads = p->n_q_heads; a.n_kv_heads = p->n_kv_heads;
  a.group = p->n_q_heads / p->n_kv_heads; a.causal = p->causal;
  a.dq_f32 = dq_ranges > 1 ? 1 : a.dq_final_f32; a.dq_accumulate = dq_ranges > 1 ? 0 : a.dq_final_accumulate;
  a.dkv_accumulate = dkv_accumulate ? 1 : 0;
  a.q_offset = p->q_offset; a.kv_begin = p->kv_begin; a.kv_end = p->kv_end; a.kv_capacity = p->kv_capacity;
  a.scale = p->scale; a.scale_log2e = p->scale * 1.4426950408889634f;
  a.q_stride_b = p->q_stride_b; a.q_stride_s = p->q_stride_s; a.q_stride_h = p->q_stride_h;
  a.kv_stride_b = p->kv_stride_b; a.kv_stride_s = p->kv_stride_s; a.kv_stride_h = p->kv_stride_h;
  a.o_stride_b = p->o_stride_b; a.o_stride_s = p->o_stride_s; a.o_stride_h = p->o_stride_h;
  a.do_stride_b = p->do_stride_b; a.do_stride_s = p->do_stride_s; a.do_stride_h = p->do_stride_h;
  if (ensure_device_ready() != SLIMPIPE_OK) return SLIMPIPE_ELAUNCH;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (timed(SLIMPIPE_KERNEL_DELTA, st, [&] { return launch_delta(a, p->batch, p->head_dim, st); }, events) != hipSuccess) return SLIMPIPE_ELAUNCH;
  if (timed(SLIMPIPE_KERNEL_DQ, st, [&] { return launch_bwd_dq(a, p->batch, p->head_dim, st); }, events) != hipSuccess) return SLIMPIPE_ELAUNCH;
  if (dq_ranges > 1 &&
      timed(SLIMPIPE_KERNEL_DQ_REDUCE, st, [&] { return launch_dq_reduce(a, p->batch, p->head_dim, st); }, events) != hipSuccess)
    return SLIMPIPE_ELAUNCH;
  if (timed(SLIMPIPE_KERNEL_DKDV, st, [&] { return launch_bwd_dkdv(a, p->batch, p->head_dim, st); }, events) != hipSuccess) return SLIMPIPE_ELAUNCH;
  if (split > 1 &&
      timed(SLIMPIPE_KERNEL_DKDV_REDUCE, st, [&] { return launch_dkdv_reduce(a, p->batch, p->head_dim, st); }, events) != hipSuccess)
    return SLIMPIPE_ELAUNCH;
  return SLIMPIPE_OK;
}

int slimpipe_attn_bwd(const slimpipe_attn_params* p, const void* q_slice, const void* k_prefix,
                      const void* v_prefix, const void* out, const void* d_out, const float* lse, void* dq,
                      int32_t dq_dtype, int32_t dq_accumulate, float* dk_acc, float* dv_acc,
                      int32_t dkv_accumulate, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!p) return SLIMPIPE_EINVAL_NULL;
  return bwd_impl(p, q_slice, &k_prefix, &v_prefix, 1, p->kv_capacity > 0 ? p->kv_capacity : 1, out, d_out, lse, dq, dq_dtype,
                  dq_accumulate, &dk_acc, &dv_acc, dkv_accumulate, workspace, workspace_bytes, hip_stream);
}

int slimpipe_attn_bwd_noalloc(const slimpipe_attn_params* p, const void* q_slice, const void* k_prefix,
                              const void* v_prefix, const void* out, const void* d_out, const float* lse, void* dq,
                              int32_t dq_dtype, int32_t dq_accumulate, float* dk_acc, float* dv_acc,
                              int32_t dkv_accumulate, void* hip_stream) {
  if (!p) return SLIMPIPE_EINVAL_NULL;
  int rc = slimpipe_attn_validate(p, 1);
  if (rc != SLIMPIPE_OK) return rc;
  if (delta_bytes(p) > kScratchBytes) return SLIMPIPE_ETOOLARGE;
  void* ws = nullptr;
  if (ensure_device_ready(&ws) != SLIMPIPE_OK || !ws) return SLIMPIPE_ELAUNCH;
  // the two statistics arrays and the ticket counter behind them: no split of the dk/dv query stream, no key ranges for
  // dq (the sums of slimpipe_attn_bwd given a workspace of the minimum size), and no event records of the benchmark switch
  static_assert(kScratchTicketBytes == kTicketBytes, "the counter sits right behind the statistics");
  return bwd_impl(p, q_slice, &k_prefix, &v_prefix, 1, p->kv_capacity > 0 ? p->kv_capacity : 1, out, d_out, lse, dq, dq_dtype,
                  dq_accumulate, &dk_acc, &dv_acc, dkv_accumulate, ws, delta_bytes(p) + kTicketBytes, hip_stream, false);
}

int slimpipe_attn_noalloc_max_rows(void) { return (int)(kScratchBytes / (2 * sizeof(float))); }

int slimpipe_attn_bwd_chunked(const slimpipe_attn_params* p, const void* q_slice, const void* const* k_chunks,
                              const void* const* v_chunks, int32_t n_chunks, int64_t chunk_len, const void* out,
                              const void* d_out, const float* lse, void* dq, int32_t dq_dtype, int32_t dq_accumulate,
                              float* const* dk_chunks, float* const* dv_chunks, int32_t dkv_accumulate, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
  return bwd_impl(p, q_slice, k_chunks, v_chunks, n_chunks, chunk_len, out, d_out, lse, dq, dq_dtype, dq_accumulate, dk_chunks,
                  dv_chunks, dkv_accumulate, workspace, workspace_bytes, hip_stream);
}

int slimpipe_attn_merge(int32_t n_parts, const void* const* outs, const float* const* lses, int32_t part_dtype,
                        int32_t batch, int32_t s_q, int32_t n_q_heads, int32_t head_dim, void* out,
                        int32_t out_dtype, float* lse, void* hip_stream) {
  if (!outs || !lses || !out || !lse) return SLIMPIPE_EINVAL_NULL;
  if (n_parts < 1 || n_parts > 16) return SLIMPIPE_EINVAL_SHAPE;
  if (batch <= 0 || s_q <= 0 || n_q_heads <= 0 || head_dim <= 0 || head_dim % 8 != 0) return SLIMPIPE_EINVAL_SHAPE;
  if ((part_dtype != SLIMPIPE_BF16 && part_dtype != SLIMPIPE_F32) ||
      (out_dtype != SLIMPIPE_BF16 && out_dtype != SLIMPIPE_F32))
    return SLIMPIPE_EINVAL_SHAPE;
  MergeArgs a;
  memset(&a, 0, sizeof(a));
  for (int i = 0; i < n_parts; ++i) {
    if (!outs[i] || !lses[i]) return SLIMPIPE_EINVAL_NULL;
    if (!aligned16(outs[i]) || (reinterpret_cast<uintptr_t>(lses[i]) & 3u)) return SLIMPIPE_EINVAL_ALIGN;
    a.outs[i] = outs[i];
    a.lses[i] = lses[i];
  }
  if (!aligned16(out) || (reinterpret_cast<uintptr_t>(lse) & 3u)) return SLIMPIPE_EINVAL_ALIGN;
  a.n_parts = n_parts; a.part_f32 = (part_dtype == SLIMPIPE_F32); a.out_f32 = (out_dtype == SLIMPIPE_F32);
  a.head_dim = head_dim; a.n_q_heads = n_q_heads; a.s_q = s_q; a.rows = (int64_t)batch * s_q;
  a.out = out; a.lse = lse;
  a.o_stride_h = head_dim; a.o_stride_s = (int64_t)n_q_heads * head_dim; a.o_stride_b = a.o_stride_s * s_q;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = timed(SLIMPIPE_KERNEL_MERGE, st, [&] { return launch_merge(a, st); });
  return e == hipSuccess ? SLIMPIPE_OK : SLIMPIPE_ELAUNCH;
}

int slimpipe_attn_finalize_bf16(const float* acc, void* dst_bf16, int64_t n_elems, void* hip_stream) {
  if (!acc || !dst_bf16) return SLIMPIPE_EINVAL_NULL;
  if (n_elems < 0) return SLIMPIPE_EINVAL_SHAPE;
  if (!aligned16(acc) || (reinterpret_cast<uintptr_t>(dst_bf16) & 7u)) return SLIMPIPE_EINVAL_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipError_t e = timed(SLIMPIPE_KERNEL_FINALIZE, st, [&] { return launch_finalize(acc, static_cast<__bf16*>(dst_bf16), n_elems, st); });
  return e == hipSuccess ? SLIMPIPE_OK : SLIMPIPE_ELAUNCH;
}

int slimpipe_attn_mfma_rate(int random_operands, float* sink, double* tflops, void* hip_stream) {
  if (!sink || !tflops) return SLIMPIPE_EINVAL_NULL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int iters = 20000, wgs = 8 * compute_units();
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return SLIMPIPE_ELAUNCH;
  int rc = SLIMPIPE_OK;
  float ms = 0.f;
  // one untimed launch to get the clocks where they settle, then the timed one
  if (launch_mfma_rate(random_operands, iters, wgs, sink, st) != hipSuccess) rc = SLIMPIPE_ELAUNCH;
  if (rc == SLIMPIPE_OK && (hipEventRecord(e0, st) != hipSuccess || launch_mfma_rate(random_operands, iters, wgs, sink, st) != hipSuccess ||
                            hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                            hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = SLIMPIPE_ELAUNCH;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == SLIMPIPE_OK) *tflops = (double)wgs * 8 * 4 * iters * 32768.0 / (ms * 1e-3) / 1e12;
  return rc;
}

int slimpipe_attn_xcd_rate(int32_t iters, int32_t workgroups, int64_t* t_start, int64_t* t_end, uint32_t* xcc, void* hip_stream) {
  if (!t_start || !t_end || !xcc) return SLIMPIPE_EINVAL_NULL;
  if (iters < 1 || workgroups < 1 || workgroups > 1 << 16) return SLIMPIPE_EINVAL_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (launch_xcd_rate(iters, workgroups, reinterpret_cast<long long*>(t_start), reinterpret_cast<long long*>(t_end), xcc, st) != hipSuccess)
    return SLIMPIPE_ELAUNCH;
  return hipStreamSynchronize(st) == hipSuccess ? SLIMPIPE_OK : SLIMPIPE_ELAUNCH;
}

int slimpipe_attn_dq_atomic_probe(float* dq, int32_t s_q, int32_t heads, int32_t key_tiles, int32_t rows_per_step,
                                  int32_t placement, int32_t rotate, int32_t filler_mfma, int32_t with_atomics,
                                  uint32_t* xcc_mismatch, double* ms, void* hip_stream) {
  if (!dq || !xcc_mismatch || !ms) return SLIMPIPE_EINVAL_NULL;
  if (s_q <= 0 || heads <= 0 || key_tiles <= 0 || (rows_per_step != 32 && rows_per_step != 64) || s_q % rows_per_step != 0 ||
      filler_mfma < 0 || filler_mfma % 4 != 0 || (int64_t)key_tiles * heads > 1 << 20)
    return SLIMPIPE_EINVAL_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  // on failure *ms = -(1000 * step + HIP error code), so that a benchmark log names the call that failed
  float t = 0.f;
  int step = 0;
  hipError_t e = hipSuccess;
  auto run = [&](hipError_t r) { ++step; if (e == hipSuccess && r != hipSuccess) { e = r; return false; } return e == hipSuccess; };
  run(hipEventCreate(&e0)) && run(hipEventCreate(&e1)) && run(hipEventRecord(e0, st)) &&
      run(launch_dq_atomic_probe(dq, s_q, heads, key_tiles, rows_per_step, placement, rotate, filler_mfma, with_atomics, xcc_mismatch, st)) &&
      run(hipEventRecord(e1, st)) && run(hipEventSynchronize(e1)) && run(hipEventElapsedTime(&t, e0, e1));
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  *ms = e == hipSuccess ? (double)t : -(1000.0 * step + (double)(int)e);
  return e == hipSuccess ? SLIMPIPE_OK : SLIMPIPE_ELAUNCH;
}

const char* slimpipe_attn_strerror(int code) {
  switch (code) {
    case SLIMPIPE_OK: return "ok";
    case SLIMPIPE_EINVAL_NULL: return "a required pointer is NULL";
    case SLIMPIPE_EINVAL_SHAPE: return "invalid shape, head_dim, scale, flag or dtype";
    case SLIMPIPE_EINVAL_RANGE: return "invalid q_offset / kv range / kv_capacity";
    case SLIMPIPE_EINVAL_STRIDE: return "strides must be positive multiples of 8 elements and cover head_dim";
    case SLIMPIPE_EINVAL_ALIGN: return "pointer not 16-byte aligned";
    case SLIMPIPE_EWORKSPACE: return "workspace missing or too small";
    case SLIMPIPE_ELAUNCH: return "HIP launch failed";
    case SLIMPIPE_ETOOLARGE: return "batch * heads * rows exceeds the fixed scratch of slimpipe_attn_bwd_noalloc";
    default: return "unknown slimpipe status";
  }
}

}  // extern "C"
