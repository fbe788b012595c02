// Device-side building blocks shared by the gfx950 attention kernels: bf16 MFMA operand types,
// the swizzled LDS tile layout, cooperative global->LDS tile staging and the two LDS read
// patterns (row-packed for contraction over head_dim, transposed for contraction over rows).
#pragma once
#include <hip/hip_runtime.h>

#include "kernels.hpp"
#include <stdint.h>

namespace slimpipe {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define SP_DEV __device__ __forceinline__

// v_mfma_f32_32x32x16_bf16.  With lane = 32*g + r (r = lane & 31, g = lane >> 5):
//   A (32 x 16): lane holds row r, k = 8g .. 8g+7
//   B (16 x 32): lane holds column r, k = 8g .. 8g+7
//   C (32 x 32): lane holds column r; register i is row 8*(i/4) + 4g + (i%4)
// Because the contraction index is a dummy, the 8 k-slots of group g may stand for ANY 8 rows
// of the contracted dimension as long as A and B agree; the kernels use that to feed a C-layout
// tile straight back in as a B operand (slots of group g = rows 4g..4g+3 and 8+4g..8+4g+3 of a
// 16-row step), with the matching A operand coming from the transposed LDS read below.
SP_DEV f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

SP_DEV float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// max / sum over the two half-waves (lanes l and l^32 hold the same column of a C tile).
SP_DEV float xhalf_max(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
SP_DEV float xhalf_sum(float v) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Pack 8 consecutive C-tile registers (float) into one bf16x8 B operand (RNE).
SP_DEV bf16x8 pack8(const f32x16& c, int base) {
  bf16x8 r;
#pragma unroll
  for (int j = 0; j < 8; j += 2) {
    f32x2 f = {c[base + j], c[base + j + 1]};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    r[j] = h[0];
    r[j + 1] = h[1];
  }
  return r;
}

// ---------------------------------------------------------------------------------------------
// LDS tile: ROWS x D bf16, row-major, rows of D*2 bytes split into 16-byte chunks whose position
// inside the row is XOR-swizzled with the row index.  For D = 128 (16 chunks, one 256-byte bank
// line per row) chunk c = 4u+i of row 4a+k sits at 4(u^k) + (i ^ (a&3)): both the row-packed read
// (16 consecutive rows, same chunk) and the transposed read (4 consecutive rows x 4 consecutive
// chunks) then touch 16 distinct 16-byte bank groups.  D = 64 uses c ^ (row & 7).
template <int D>
SP_DEV int tile_off(int row, int chunk) {
  if constexpr (D == 128) {
    const int u = chunk >> 2, i = chunk & 3;
    const int p = (((u ^ row) & 3) << 2) | ((i ^ (row >> 2)) & 3);
    return row * (D * 2) + (p << 4);
  } else {
    return row * (D * 2) + (((chunk ^ row) & (D / 8 - 1)) << 4);
  }
}

// The two LDS read patterns.
//   Row-packed operand (contraction over head_dim): lane (r, g) reads the 8 consecutive head_dim
//   elements [16*ks + 8g, +8) of tile row r with one ds_read_b128.
//   Transposed operand (contraction over rows) through ds_read_b64_tr_b16: within each block of 16
//   lanes the instruction returns to lane i, element e, the (i%4)-th 16-bit element of the 8 bytes
//   addressed by lane 4e + i/4 of the block.  Pointing lane j of block b at row (row0 + 4*(b>>1) + j/4),
//   columns 32*db + 16*(b&1) + 4*(j%4) .. +3 therefore hands lane l the column 32*db + (l&31) of rows
//   row0 + 4g .. row0 + 4g+3; a second read 8 rows further completes the 8 k-slots of group g.
//
// The offsets below are LDS byte ADDRESSES (the kernel adds the address of its shared memory when it sets
// them up): a read is "register + immediate" with no pointer arithmetic left.  (Through a pointer into
// the shared array every read pays a vector add of the array's link-time address.)
template <class T>
SP_DEV T __attribute__((address_space(3))) * lds_ptr(int addr, int const_off) {
  typedef char __attribute__((address_space(3))) * lds_char_ptr;
  return reinterpret_cast<T __attribute__((address_space(3))) *>(reinterpret_cast<lds_char_ptr>(static_cast<uintptr_t>((unsigned)addr)) + const_off);
}

// Per-lane byte offsets of the two read patterns for a tile row block that starts at a multiple of
// 16 rows.  Adding a multiple of 16 rows does not change the swizzle bits, so every read of a
// kernel is (one of these registers) + (compile-time constant): the constant goes into the
// instruction's offset field and no address arithmetic is left in the loops.
template <int D>
struct RpOffsets {       // row-packed: row = lane & 31, chunk 2*ks + g
  int off[D / 16];
  SP_DEV void init(int lane, int base) {
    const int g = lane >> 5, ql = lane & 31;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) off[ks] = base + tile_off<D>(ql, 2 * ks + g);
  }
  SP_DEV void add(int delta) {
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) off[ks] += delta;
  }
};
template <int D>
struct TrOffsets {       // transposed: rows 4g + j/4 (+8 for the second read), column block db
  int off[D / 32][2];
  SP_DEV void init(int lane, int base) {
    const int j = lane & 15, b = lane >> 4;
    const int row = ((b >> 1) << 2) + (j >> 2);
    const int sub = (j & 1) << 3;
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      const int chunk = 4 * db + 2 * (b & 1) + ((j & 3) >> 1);
      off[db][0] = base + tile_off<D>(row, chunk) + sub;
      off[db][1] = base + tile_off<D>(row + 8, chunk) + sub;
    }
  }
  SP_DEV void add(int delta) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db) { off[db][0] += delta; off[db][1] += delta; }
  }
};

// Reads through the lane offsets; `const_off` is a compile-time byte offset (tile selector + 16-row
// block * row bytes).
template <int D>
SP_DEV bf16x8 lds_rp(const RpOffsets<D>& lo, int ks, int const_off) {
  return *lds_ptr<bf16x8>(lo.off[ks], const_off);
}
template <int D>
SP_DEV bf16x8 lds_tr(const TrOffsets<D>& lo, int db, int const_off) {
  bf16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(lds_ptr<bf16x4>(lo.off[db][0], const_off));
  bf16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(lds_ptr<bf16x4>(lo.off[db][1], const_off));
  bf16x8 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = a[2]; r[3] = a[3];
  r[4] = b[0]; r[5] = b[1]; r[6] = b[2]; r[7] = b[3];
  return r;
}

// The same two read patterns from ONE register each.  With tile bases at multiples of 256 bytes the
// swizzle makes the offset of head_dim block ks (row-packed) or db (transposed) the offset of block 0
// XOR a compile-time constant, so a kernel short of registers keeps one offset per tile and pays one
// v_xor per read instead of holding D/16 offsets.
template <int D>
struct RpBase {
  int off0;
  SP_DEV void init(int lane, int base) { off0 = base + tile_off<D>(lane & 31, lane >> 5); }
  SP_DEV void add(int delta) { off0 += delta; }
};
template <int D>
struct TrBase {
  int off0;
  SP_DEV void init(int lane, int base) {
    const int j = lane & 15, b = lane >> 4;
    off0 = base + tile_off<D>(((b >> 1) << 2) + (j >> 2), 2 * (b & 1) + ((j & 3) >> 1)) + ((j & 1) << 3);
  }
  SP_DEV void add(int delta) { off0 += delta; }
};
template <int D>
SP_DEV bf16x8 lds_rp(const RpBase<D>& lo, int ks, int const_off) {
  return *lds_ptr<bf16x8>(lo.off0 ^ (32 * ks), const_off);
}
template <int D>
SP_DEV bf16x8 lds_tr(const TrBase<D>& lo, int db, int const_off) {
  constexpr int X1 = D == 128 ? 32 : 0;       // rows +8 flip bit 1 of the swizzled chunk for D = 128
  const int o = lo.off0 ^ (64 * db);
  bf16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(lds_ptr<bf16x4>(o, const_off));
  bf16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(lds_ptr<bf16x4>(o ^ X1, 8 * D * 2 + const_off));
  bf16x8 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = a[2]; r[3] = a[3];
  r[4] = b[0]; r[5] = b[1]; r[6] = b[2]; r[7] = b[3];
  return r;
}

// Asynchronous staging of a ROWS x D bf16 tile with global_load_lds_dwordx4: every lane hands in a
// global address, the hardware writes the 16 bytes of lane L of a wave to (M0 = wave-uniform LDS
// base) + 16*L.  One wave instruction therefore fills 1 KB of consecutive PHYSICAL chunks; the lane
// picks the global chunk that the swizzle maps to its physical slot.  No staging registers.
// The instruction is issued from inline assembly on purpose: through the compiler builtin every
// later LDS read is assumed to alias the copy and the wave is made to wait for it on the spot.
// Here the kernel owns the ordering: the copy targets a buffer nobody reads until the issuing wave
// has executed wait_async() and the workgroup has passed a barrier.  The assembly statements are
// compiler barriers for memory operations: an LDS read written after one is not moved above it.

// LDS byte address of a pointer into shared memory (uniform).  Kernels take it once for the start of
// their dynamic shared memory and do integer arithmetic from there: every cast of a generic pointer
// costs a null check and a scalar read-back.
// An opaque copy of a value: what is computed from it is computed afresh at this point instead of
// being kept in a register from wherever the compiler first saw it (kernels at the register limit
// derive lane-dependent quantities from the thread index where they need them).
SP_DEV int fresh(int x) {
  asm volatile("" : "+v"(x));
  return x;
}
// A pointer the program knows to be the same in all lanes, read back into scalar registers (for
// values that went through vector instructions on the way, e.g. an integer division).
template <class T>
SP_DEV T* uniform_ptr(T* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<T*>(((uint64_t)hi << 32) | lo);
}
SP_DEV unsigned lds_addr(const void* p) {
  return __builtin_amdgcn_readfirstlane(
      (unsigned)reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const char*)p));
}
// one dword per lane: lane i lands at lds_base + 4*i
SP_DEV void dma4(const void* base, uint32_t lane_off, unsigned lds_base) {      // base uniform, lane_off in bytes
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(lane_off), "s"(base), "s"(lds_base) : "memory", "m0");
}
// A tile copy with nothing but two per-lane constants (packed into one register): THREADS/NC rows per pass with THREADS a
// multiple of 16*NC (THREADS = 256, NC = 16: 16 rows per pass), so pass n handles row
// r0 + (THREADS/NC)*n of the tile and, the row step being a multiple of 16, the SAME swizzled chunk.
// A tile copy is "uniform base + 32-bit lane offset" with the row clamped to the rows that exist
// (`rows_avail` >= 1, uniform): branch-free, four VALU operations per copy instruction.
template <int D, int ROWS, int THREADS>
struct TileDma {
  static constexpr int NC = D / 8, RPP = THREADS / NC, PASSES = ROWS / RPP;
  static_assert(RPP % 16 == 0 && ROWS % RPP == 0, "row step keeps the swizzle phase");
  uint32_t rc;       // this lane's row in pass 0 (low half) and the byte offset of its swizzled chunk inside the row (high half)
  SP_DEV void init(int tid) {
    const int r = tid / NC, p = tid % NC;
    int c;
    if constexpr (D == 128) c = ((((p >> 2) ^ r) & 3) << 2) | (((p & 3) ^ (r >> 2)) & 3);
    else c = (p ^ r) & (NC - 1);
    rc = (uint32_t)r | ((uint32_t)c * 16 << 16);
  }
  // pass n of the tile whose first row starts at `tile_base` (uniform) into the LDS tile at byte address
  // `lds_tile` (uniform); `wave` is the uniform index of the calling wave among the THREADS/64 that copy
  SP_DEV void issue(unsigned lds_tile, const bf16_t* tile_base, uint32_t row_bytes, int rows_avail, int wave, int n) const {
    const unsigned lds = lds_tile + (n * THREADS + wave * 64) * 16;
    // (from an opaque copy: the row of every pass would otherwise be kept in a register of its own
    // across the caller's loop)
    const uint32_t rcv = (uint32_t)fresh((int)rc);
    int r = (int)(rcv & 0xffffu) + RPP * n;
    r = r < rows_avail ? r : rows_avail - 1;
    // (24-bit multiply, full rate: r < 2^16 and a row is shorter than 2^23 bytes, checked by the host)
    const uint32_t off = __umul24((uint32_t)r, row_bytes) + (rcv >> 16);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(tile_base), "s"(lds) : "memory", "m0");
  }
};

// Walks the key tiles of a chunked K/V prefix in increasing order: where the tile "now" starts.  All
// members are uniform.  A step is two additions; the chunk's base pointer (a scalar load from the
// kernel arguments) and the product row * stride are needed only when the walk enters a new chunk.
struct KvWalk {
  const bf16_t* ptr;       // first row of the tile (batch and head offset included)
  int chunk, row;          // current chunk, first row of the tile inside it
  SP_DEV void seek(const bf16_t* const* table, const KvChunks& kv, int64_t key0, int64_t head_off, int64_t stride_s) {
    chunk = kv.n > 1 ? __builtin_amdgcn_readfirstlane((int)(key0 / kv.len)) : 0;
    row = (int)(key0 - (int64_t)chunk * kv.len);
    ptr = table[chunk] + head_off + (int64_t)row * stride_s;
  }
  // to the next tile; tile_step = tile * stride_s
  SP_DEV void step(const bf16_t* const* table, const KvChunks& kv, int tile, int64_t tile_step, int64_t head_off, int64_t stride_s) {
    row += tile;
    ptr += tile_step;
    if (row >= kv.len && chunk + 1 < kv.n) {
      row -= (int)kv.len;
      ++chunk;
      ptr = table[chunk] + head_off + (int64_t)row * stride_s;
    }
  }
  // rows of the chunk from the tile's first row on, at most `tile`
  SP_DEV int rows(const KvChunks& kv, int tile) const {
    const int64_t left = kv.len - row;
    return left > tile ? tile : (int)left;
  }
};

// vmcnt(0), other counters untouched (gfx9 encoding: vmcnt[3:0]|[15:14], expcnt[6:4], lgkmcnt[11:8]).
SP_DEV void wait_async() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// ---- scheduling helpers ------------------------------------------------------------------------
#define SP_FENCE() __builtin_amdgcn_sched_barrier(0)
// Issue priority of a wave while it is in a matrix phase.  Waves are served oldest first, so without
// this the younger group's MFMAs wait behind the vector instructions of the older group that shares
// its SIMDs; a wave in a matrix phase issues only a handful of instructions per MFMA, so letting it
// go first costs the vector phase little.
SP_DEV void matrix_phase_begin() { __builtin_amdgcn_s_setprio(3); }
SP_DEV void matrix_phase_end() { __builtin_amdgcn_s_setprio(0); }

// End of a phase of the two-group schedules: nothing may be scheduled across the barrier.
SP_DEV void phase_end() {
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  __builtin_amdgcn_sched_barrier(0);
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

}  // namespace slimpipe
