// Forward of slice-wise causal attention over a key range (paper Sec. 4.1.2; partial ranges and
// the normaliser that travels with the output: Sec. 4.2.2, Sec. 5).
//
// One workgroup = 8 wavefronts, each owning 32 query rows of one head.  The key range is walked
// in tiles of BN keys staged in LDS.  Per tile and wave:
//   S^T = K Q^T        A = K rows from LDS (row-packed), B = Q held in registers
//   online softmax     the C layout gives every lane ONE query column, so the row max / row sum
//                      are in-lane reductions plus one exchange between the two half-waves
//   O^T += V^T P^T     A = V through the transposed LDS read, B = P straight from the C registers
// Scores and probabilities never leave registers.
//
// Schedule.  All 8 waves walk the tiles in step (S, softmax, PV, one barrier per tile).  A SIMD hosts
// two of them, so in the S and PV parts the LDS latency of one wave is covered by the MFMAs of the
// other.  K(t+1) and V(t+1) are copied global->LDS asynchronously into the other buffer set while
// tile t is computed; the copy instructions are spread over the tile because the L1 path moves
// 64 bytes per clock for the whole CU and a wave stalls at issue while it is busy.
#include <stdlib.h>

#include "kernels.hpp"
#include "tile_common.hpp"

namespace slimpipe {

template <int D, int BN>
struct FwdState {
  static constexpr int KS = D / 16, DB = D / 32, KB = BN / 32;
  bf16x8 qreg[KS];
  f32x16 o[DB];
  f32x16 s[KB];
  bf16x8 p[KB][2];
  float m_run, l_run;
  float mx;          // row maximum of the raw scores of the tile in `s` (two-group variant)
};

// S(t)^T = K(t) Q^T for this wave's 32 queries.
template <int D, int BN>
SP_DEV void fwd_scores(const char* smem, const RpOffsets<D>& lo_k, FwdState<D, BN>& st) {
  constexpr int KB = BN / 32, KS = D / 16;
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.s[kb][i] = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {          // the KB accumulator chains interleaved
      const bf16x8 ka = lds_rp<D>(smem, lo_k, ks, kb * 32 * D * 2);
      st.s[kb] = mfma32(ka, st.qreg[ks], st.s[kb]);
    }
  sched_reads_ahead<KB * KS, 1, 2>();
  __builtin_amdgcn_sched_barrier(0);
}

// O^T += V(t)^T P(t)^T.
template <int D, int BN>
SP_DEV void fwd_pv(const char* smem, const TrOffsets<D>& lo_v, FwdState<D, BN>& st) {
  constexpr int KB = BN / 32, DB = D / 32;
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 va = lds_tr<D>(smem, lo_v, db, (kb * 32 + 16 * half) * D * 2);
        st.o[db] = mfma32(va, st.p[kb][half], st.o[db]);
      }
  sched_reads_ahead<KB * 2 * DB, 2, 2>();
  __builtin_amdgcn_sched_barrier(0);
}

// Mask the scores of a tile and take this lane's row maximum (raw scores; both half-waves combined).
template <int D, int BN>
SP_DEV float fwd_rowmax(FwdState<D, BN>& st, bool need_mask, int kmax_rel, int g) {
  constexpr int KB = BN / 32;
  if (need_mask) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key_rel = kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
        st.s[kb][i] = key_rel <= kmax_rel ? st.s[kb][i] : -INFINITY;
      }
  }
  float mx = -INFINITY;
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int i = 0; i < 16; i += 2) mx = fmaxf(fmaxf(st.s[kb][i], st.s[kb][i + 1]), mx);   // v_max3_f32
  return xhalf_max(mx);
}

// P(t) = online softmax of S(t); rescales O and the running sum when a row maximum moves.
// kmax_rel: last visible key of this lane's query relative to the tile (>= BN: no mask needed).
template <int D, int BN, bool PIN, bool PRE, class H>
SP_DEV void fwd_softmax(FwdState<D, BN>& st, float c, bool need_mask, int kmax_rel, int g, H&& hook) {
  constexpr int KB = BN / 32, DB = D / 32;
  hook(0);
  const float mx = PRE ? st.mx : fwd_rowmax<D, BN>(st, need_mask, kmax_rel, g);
  hook(1);
  const float m_new = fmaxf(st.m_run, mx * c);
  const float m_eff = (m_new == -INFINITY) ? 0.f : m_new;
  // rescale only when some row of the wave moved its maximum (rare once a few tiles are in)
  if (__builtin_amdgcn_ballot_w64(m_new != st.m_run) != 0) {
    const float alpha = exp2_fast(st.m_run - m_eff);     // m_run = -inf -> 0
    st.l_run *= alpha;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) st.o[db][i] *= alpha;
  }
  st.m_run = m_new;
  float l_add = 0.f;
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    hook(2 + kb);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float p = exp2_fast(__builtin_fmaf(st.s[kb][i], c, -m_eff));
      st.s[kb][i] = p;
      l_add += p;
    }
    st.p[kb][0] = pack8(st.s[kb], 0);
    st.p[kb][1] = pack8(st.s[kb], 8);
    // PIN: without a use here the optimiser sinks this arithmetic past the phase barrier that follows
    if (PIN) asm volatile("" : "+v"(st.p[kb][0]), "+v"(st.p[kb][1]));
  }
  st.l_run += l_add;
  if (PIN) asm volatile("" : "+v"(st.l_run));
}

// out = O / l, lse = (m + log2 l) ln 2; rows that saw no key: out = 0, lse = -inf.
template <int D, int BN>
SP_DEV void fwd_epilogue(const FwdArgs& a, FwdState<D, BN>& st, int myrow, int h, int b, int g) {
  constexpr int DB = D / 32;
  const float l_tot = xhalf_sum(st.l_run);
  const bool has = l_tot > 0.f;
  const float inv = has ? 1.0f / l_tot : 0.f;
  if (myrow < a.s_q) {
    if (g == 0) {
      const float lse = has ? (st.m_run + __builtin_log2f(l_tot)) * kLn2 : -INFINITY;
      a.lse[((int64_t)b * a.n_q_heads + h) * a.s_q + myrow] = lse;
    }
    const int64_t obase = (int64_t)b * a.o_stride_b + (int64_t)myrow * a.o_stride_s + (int64_t)h * a.o_stride_h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 32 * db + 8 * i4 + 4 * g;
        f32x4 v4 = {st.o[db][4 * i4] * inv, st.o[db][4 * i4 + 1] * inv, st.o[db][4 * i4 + 2] * inv,
                    st.o[db][4 * i4 + 3] * inv};
        if (a.out_f32) {
          *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + obase + d) = v4;
        } else {
          bf16x4 h4 = __builtin_convertvector(v4, bf16x4);
          *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(a.out) + obase + d) = h4;
        }
      }
  }
}

template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64) void attn_fwd_kernel(const FwdArgs a) {
  constexpr int BM = NW * 32, KS = D / 16, DB = D / 32, T = NW * 64;
  constexpr int TILE_BYTES = BN * D * 2;
  static_assert((TILE_BYTES & (TILE_BYTES - 1)) == 0, "buffer toggle is an XOR");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // LDS: K set 0, K set 1, V set 0, V set 1
  constexpr int K_BASE = 0, V_BASE = 2 * TILE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int qblk = (int)gridDim.x - 1 - (int)blockIdx.x;   // heaviest (latest) query block first
  const int h = blockIdx.y, b = blockIdx.z, hk = h / a.group;
  const int m0 = qblk * BM, wrow0 = m0 + wave * 32;
  const int myrow = wrow0 + ql;
  const int myrow_c = myrow < a.s_q ? myrow : a.s_q - 1;
  const int64_t qpos = a.q_offset + myrow;

  FwdState<D, BN> st;
  {
    // Q as B operand: column = my query, k-slots = head_dim 16*ks + 8g ..
    const bf16_t* qp = a.q + (int64_t)b * a.q_stride_b + (int64_t)myrow_c * a.q_stride_s + (int64_t)h * a.q_stride_h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) st.qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * g);
  }
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[db][i] = 0.f;
  st.m_run = -INFINITY;    // running max of score * c (log2 domain)
  st.l_run = 0.f;          // this lane's share of the running row sum

  // keys this workgroup walks: [lo, hi)
  const int64_t lo = a.kv_begin;
  int64_t hi = a.kv_end;
  if (a.causal) {
    const int last_row = (m0 + BM < a.s_q ? m0 + BM : a.s_q);   // exclusive
    const int64_t lim = a.q_offset + last_row;
    hi = hi < lim ? hi : lim;
  }
  const int nt = hi > lo ? (int)((hi - lo + BN - 1) / BN) : 0;
  const float c = a.scale_log2e;

  if (nt > 0) {
    const bf16_t* kbase = a.k + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
    const bf16_t* vbase = a.v + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
    RpOffsets<D> lo_k;
    TrOffsets<D> lo_v;
    lo_k.init(lane, K_BASE);
    lo_v.init(lane, V_BASE);
    auto key0_of = [&](int t) { return lo + (int64_t)t * BN; };
    constexpr int PASSES = BN * (D / 8) / T;             // copy instructions per tile and wave
    TileDma<D, BN, T> dma;
    dma.init(tid);
    const unsigned smem_lds = lds_addr(smem);
    const int wave_u = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2;
    // quarter `part` of the copies of K(t), V(t) into set t & 1 (parts 0,1: K; 2,3: V)
    auto issue_part = [&](int t, int part) {
      if (t >= nt) return;
      const bf16_t* base = part < 2 ? kbase : vbase;
      const unsigned dst = smem_lds + (part < 2 ? K_BASE : V_BASE) + (t & 1) * TILE_BYTES;
      const int64_t key0 = key0_of(t);
      const int64_t avail = a.kv_capacity - key0;
#pragma unroll
      for (int n = 0; n < PASSES; ++n)
        if (PASSES == 1 ? (part & 1) == 0 : (n & 1) == (part & 1))
          dma.issue(dst, base + key0 * a.kv_stride_s, row_bytes, avail > BN ? BN : (int)avail, wave_u, n);
    };

    for (int part = 0; part < 4; ++part) issue_part(0, part);
    wait_async();
    __syncthreads();

#ifdef SLIMPIPE_TRACE
    long long tr_s = 0, tr_v = 0, tr_pv = 0, tr_b = 0, tr_w = 0, tr_t0 = clock64(), tr_w0 = wall_clock64(), tr_last = clock64();
#define TR_MARK(var) { long long _n = clock64(); var += _n - tr_last; tr_last = _n; }
#else
#define TR_MARK(var)
#endif
    for (int t = 0; t < nt; ++t) {
      const int64_t key0 = key0_of(t);
      // whole tile above this wave's causal frontier -> nothing visible (the wave still helps copying)
      const bool skip = a.causal && key0 > a.q_offset + wrow0 + 31;
      if (!skip) {
        issue_part(t + 1, 0);
        issue_part(t + 1, 1);
        fwd_scores<D, BN>(smem, lo_k, st);
        TR_MARK(tr_s)
        const bool need_mask = (key0 + BN > a.kv_end) || (a.causal && key0 + BN - 1 > a.q_offset + wrow0);
        int64_t kmax = a.kv_end - 1;
        if (a.causal && qpos < kmax) kmax = qpos;
        kmax -= key0;
        const int kmax_rel = kmax < -1 ? -1 : (kmax > BN ? BN : (int)kmax);
        fwd_softmax<D, BN, false, false>(st, c, need_mask, kmax_rel, g, [](int) {});
        TR_MARK(tr_v)
        issue_part(t + 1, 2);
        issue_part(t + 1, 3);
        fwd_pv<D, BN>(smem, lo_v, st);
        TR_MARK(tr_pv)
      } else {
        for (int part = 0; part < 4; ++part) issue_part(t + 1, part);
      }
      const int d = (t & 1) ? -TILE_BYTES : TILE_BYTES;
      lo_k.add(d);
      lo_v.add(d);
      wait_async();
      TR_MARK(tr_w)
      __syncthreads();
      TR_MARK(tr_b)
    }
#ifdef SLIMPIPE_TRACE
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid == 0) {
      long long* dbg = reinterpret_cast<long long*>(a.lse + (int64_t)a.n_q_heads * a.s_q);   // caller over-allocates lse
      dbg[0] = tr_s; dbg[1] = tr_v; dbg[2] = tr_pv; dbg[3] = tr_b; dbg[4] = tr_w; dbg[5] = 0;
      dbg[6] = clock64() - tr_t0; dbg[7] = wall_clock64() - tr_w0; dbg[8] = nt;
    }
#endif
  }

  fwd_epilogue<D, BN>(a, st, myrow, h, b, g);
}

// ---------------------------------------------------------------------------------------------
// Variant with the two wave groups one phase apart.  A wave alternates a matrix phase
// M(t): O += P(t) V(t), S(t+1) = K(t+1) Q^T  with a vector phase  V(t): P(t) = softmax(S(t)).
// Waves 0-3 (group A) and 4-7 (group B) run the same sequence shifted by one phase, one workgroup
// barrier per phase, so every SIMD hosts one wave in each kind of phase.  The pair (V(t), K(t+1))
// that M(t) needs lives in one of two LDS buffer sets; the next pair is copied asynchronously during
// the two phases before it is needed.
template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64) void attn_fwd_pp_kernel(const FwdArgs a) {
  static_assert(NW == 8, "two groups of four waves");
  constexpr int BM = NW * 32, KS = D / 16, DB = D / 32, T = NW * 64;
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int K_BASE = 0, V_BASE = 2 * TILE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const bool group_b = wave >= NW / 2;
  const int qblk = (int)gridDim.x - 1 - (int)blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z, hk = h / a.group;
  const int m0 = qblk * BM, wrow0 = m0 + wave * 32;
  const int myrow = wrow0 + ql;
  const int myrow_c = myrow < a.s_q ? myrow : a.s_q - 1;
  const int64_t qpos = a.q_offset + myrow;

  FwdState<D, BN> st;
  {
    const bf16_t* qp = a.q + (int64_t)b * a.q_stride_b + (int64_t)myrow_c * a.q_stride_s + (int64_t)h * a.q_stride_h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) st.qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * g);
  }
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.o[db][i] = 0.f;
  st.m_run = -INFINITY;
  st.l_run = 0.f;

  const int64_t lo = a.kv_begin;
  int64_t hi = a.kv_end;
  if (a.causal) {
    const int last_row = (m0 + BM < a.s_q ? m0 + BM : a.s_q);
    const int64_t lim = a.q_offset + last_row;
    hi = hi < lim ? hi : lim;
  }
  const int nt = hi > lo ? (int)((hi - lo + BN - 1) / BN) : 0;
  const float c = a.scale_log2e;

  if (nt > 0) {
    const bf16_t* kbase = a.k + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
    const bf16_t* vbase = a.v + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
    RpOffsets<D> lo_k;
    TrOffsets<D> lo_v;
    auto key0_of = [&](int t) { return lo + (int64_t)t * BN; };
    // Tile copies are issued from vector phases only, by the four waves of the group that is in one
    // (next to the LDS reads and MFMAs of a matrix phase they stall the wave): group B copies V(t+1)
    // during its V(t), group A copies K(t+1) during its V(t).  Copies are branch-free: a tile past the
    // end of the range re-copies the last tile (nobody reads it), rows past the allocation are clamped.
    constexpr int GT = T / 2;                            // threads of one group
    const int gtid = tid & (GT - 1);
    TileDma<D, BN, GT> dma;
    constexpr int PASSES = TileDma<D, BN, GT>::PASSES;   // copy instructions per tile and wave
    static_assert(PASSES <= 4, "one copy instruction per softmax hook");
    dma.init(gtid);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2;
    const unsigned smem_lds = lds_addr(smem);
    const int gwave_u = __builtin_amdgcn_readfirstlane(gtid >> 6);
    struct CopyJob { const bf16_t* src; unsigned dst; int rows; };
    auto make_copy = [&](bool is_k, int t, int set) {
      const int64_t key0 = key0_of(t < nt ? t : nt - 1);
      const int64_t avail = a.kv_capacity - key0;
      CopyJob j;
      j.src = (is_k ? kbase : vbase) + key0 * a.kv_stride_s;
      j.dst = smem_lds + (is_k ? K_BASE : V_BASE) + set * TILE_BYTES;
      j.rows = avail > BN ? BN : (int)avail;
      return j;
    };
    auto copy_pass = [&](const CopyJob& j, int n) {
#ifndef SLIMPIPE_NODMA
      dma.issue(j.dst, j.src, row_bytes, j.rows, gwave_u, n);
#endif
    };
    // vector phase of tile t that also copies one tile of the next pair
    auto vector_phase = [&](int t, const CopyJob& j) {
      fwd_softmax<D, BN, true, true>(st, c, false, 0, g, [&](int part) { if (part < PASSES) copy_pass(j, part); });
    };
    // tail of a matrix phase: mask S(t) and take its row maxima (balances the two kinds of phase)
    auto rowmax_tile = [&](int t) {
      const int64_t key0 = key0_of(t);
      const bool need_mask = (key0 + BN > a.kv_end) || (a.causal && key0 + BN - 1 > a.q_offset + wrow0);
      int64_t kmax = a.kv_end - 1;
      if (a.causal && qpos < kmax) kmax = qpos;
      kmax -= key0;
      const int kmax_rel = kmax < -1 ? -1 : (kmax > BN ? BN : (int)kmax);
      st.mx = fwd_rowmax<D, BN>(st, need_mask, kmax_rel, g);
      asm volatile("" : "+v"(st.mx));      // keep it on this side of the phase barrier
    };

    // prologue: K(0) into K set 1 (the set "pair -1" would use), half of it by each group
    {
      // both groups copy the whole tile (the same bytes twice): simplest way to keep the copy code single
      const CopyJob j = make_copy(true, 0, 1);
      for (int n = 0; n < PASSES; ++n) copy_pass(j, n);
    }
    wait_async();
    lo_k.init(lane, K_BASE + TILE_BYTES);   // S(t) reads K(t) from set (t-1)&1: starts at set 1
    lo_v.init(lane, V_BASE);                // PV(t) reads V(t) from set t&1: starts at set 0
    __syncthreads();

    if (!group_b) {
      // phase 0
      fwd_scores<D, BN>(smem, lo_k, st);
      rowmax_tile(0);
      lo_k.add(-TILE_BYTES);
      phase_end();
#ifdef SLIMPIPE_TRACE
      long long tp_v = 0, tp_w = 0, tp_b1 = 0, tp_pv = 0, tp_s = 0, tp_b2 = 0, tp_t0 = clock64(), tp_w0 = wall_clock64(), tp_last = clock64();
#define TP_MARK(var) { long long _n = clock64(); var += _n - tp_last; tp_last = _n; }
#else
#define TP_MARK(var)
#endif
      for (int t = 0; t < nt; ++t) {
        // phase 2t+1: vector phase, copying K(t+1) for the matrix phase that follows
        vector_phase(t, make_copy(true, t + 1, t & 1));
        TP_MARK(tp_v)
        wait_async();
        TP_MARK(tp_w)
        phase_end();
        TP_MARK(tp_b1)
        // phase 2t+2: matrix phase
        fwd_pv<D, BN>(smem, lo_v, st);
        TP_MARK(tp_pv)
        if (t + 1 < nt) {
          fwd_scores<D, BN>(smem, lo_k, st);
          rowmax_tile(t + 1);
        }
        const int d = (t & 1) ? -TILE_BYTES : TILE_BYTES;
        lo_k.add(d);
        lo_v.add(d);
        TP_MARK(tp_s)
        phase_end();
        TP_MARK(tp_b2)
      }
#ifdef SLIMPIPE_TRACE
      if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid == 0) {
        long long* dbg = reinterpret_cast<long long*>(a.lse + (int64_t)a.n_q_heads * a.s_q);   // caller over-allocates lse
        dbg[0] = tp_v; dbg[1] = tp_w; dbg[2] = tp_b1; dbg[3] = tp_pv; dbg[4] = tp_s; dbg[5] = tp_b2;
        dbg[6] = clock64() - tp_t0; dbg[7] = wall_clock64() - tp_w0; dbg[8] = nt;
      }
#endif
      phase_end();                          // group B's last matrix phase
    } else {
      // phase 0: nothing to compute yet; V(0)
      {
        const CopyJob j = make_copy(false, 0, 0);
        for (int n = 0; n < PASSES; ++n) copy_pass(j, n);
      }
      phase_end();
      // phase 1
      fwd_scores<D, BN>(smem, lo_k, st);
      rowmax_tile(0);
      lo_k.add(-TILE_BYTES);
      wait_async();
      phase_end();
      for (int t = 0; t < nt; ++t) {
        // phase 2t+2: vector phase, copying V(t+1)
        vector_phase(t, make_copy(false, t + 1, (t + 1) & 1));
        phase_end();
        // phase 2t+3: matrix phase
        fwd_pv<D, BN>(smem, lo_v, st);
        if (t + 1 < nt) {
          fwd_scores<D, BN>(smem, lo_k, st);
          rowmax_tile(t + 1);
        }
        const int d = (t & 1) ? -TILE_BYTES : TILE_BYTES;
        lo_k.add(d);
        lo_v.add(d);
        wait_async();
        phase_end();
      }
    }
  }
  fwd_epilogue<D, BN>(a, st, myrow, h, b, g);
}

template <int D, int NW, int BN, bool PP>
static hipError_t launch_fwd_t(const FwdArgs& a, int batch, hipStream_t st) {
  constexpr int BM = NW * 32;
  const size_t smem = (size_t)4 * BN * D * 2;
  auto kern = PP ? &attn_fwd_pp_kernel<D, NW, BN> : &attn_fwd_kernel<D, NW, BN>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid((a.s_q + BM - 1) / BM, a.n_q_heads, batch), block(NW * 64);
  hipLaunchKernelGGL(kern, grid, block, smem, st, a);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs& a, int batch, int head_dim, hipStream_t st) {
  static const int pp = [] { const char* e = getenv("SLIMPIPE_FWD_PP"); return e ? atoi(e) : 1; }();
  if (head_dim == 128) return pp ? launch_fwd_t<128, 8, 64, true>(a, batch, st) : launch_fwd_t<128, 8, 64, false>(a, batch, st);
  return pp ? launch_fwd_t<64, 8, 64, true>(a, batch, st) : launch_fwd_t<64, 8, 64, false>(a, batch, st);
}

}  // namespace slimpipe
