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
// Schedule.  A wave that has issued an MFMA issues nothing else until the matrix pipe has taken it,
// so vector work only hides behind the MFMAs of ANOTHER wave of the same SIMD.  A wave therefore
// alternates a matrix phase MM(t): O += P(t-1) V(t-1), S(t) = K(t) Q^T with a vector phase
// VV(t): P(t) = softmax(S(t)); waves 0-3 (group A) and 4-7 (group B) run the same sequence shifted by
// one phase, one workgroup barrier per phase, so every SIMD hosts one wave in each kind of phase.
#include "kernels.hpp"
#include "tile_common.hpp"

namespace slimpipe {

// Keys per tile of the forward kernel.  128 instead of 64 halves the per-tile bookkeeping and the number of phase
// barriers per key (measured: 4 % less forward time); five 128-key tiles of head_dim 128 are the whole 160 KB of LDS.
constexpr int kFwdKeysPerTile = 128;
// operand look-ahead of the matrix phase (LDS reads issued this many MFMAs early)
constexpr int kFwdLook = 2;
// 32-key blocks of a tile whose row maxima are taken at the tail of the matrix phase (the rest: vector phase)
constexpr int fwd_rowmax_first_blocks(int kb) { return (kb + 1) / 2; }

template <int D, int BN>
struct FwdState {
  static constexpr int KS = D / 16, DB = D / 32, KB = BN / 32;
  bf16x8 qreg[KS];
  f32x16 o[DB];
  f32x16 s[KB];
  bf16x8 p[KB][2];
  float m_run, l_run;
  float mx;          // two-group kernel: maximum of this lane's raw scores over the first half of the tile's keys in `s`
};

// Row maxima of the raw scores of a tile, in two parts (the vector unit is the bottleneck of this
// kernel, so the work is split evenly between the two kinds of phase): mask + maximum over the first
// half of the keys at the tail of the matrix phase, the rest in the vector phase.
template <int D, int BN>
SP_DEV float fwd_rowmax_first(FwdState<D, BN>& st, bool need_mask, int kmin_rel, int kmax_rel, int g) {
  constexpr int KB = BN / 32;
  if (need_mask) {
    // kmin_rel <= key (kb*32 + 8*(i/4) + 4g + i%4) <= kmax_rel, with the lane's part moved to the bounds: the
    // key numbers are immediates then (a register per element otherwise, hoisted out of the tile loop)
    const int kmin_lane = kmin_rel - 4 * g, kmax_lane = kmax_rel - 4 * g;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = kb * 32 + 8 * (i >> 2) + (i & 3);
        st.s[kb][i] = ((key >= kmin_lane) & (key <= kmax_lane)) ? st.s[kb][i] : -INFINITY;
      }
  }
  float mx = -INFINITY;
#pragma unroll
  for (int kb = 0; kb < fwd_rowmax_first_blocks(KB); ++kb)
#pragma unroll
    for (int i = 0; i < 16; i += 2) mx = fmaxf(fmaxf(st.s[kb][i], st.s[kb][i + 1]), mx);
  return mx;
}
template <int D, int BN>
SP_DEV float fwd_rowmax_rest(const FwdState<D, BN>& st, float mx) {
  constexpr int KB = BN / 32;
#pragma unroll
  for (int kb = fwd_rowmax_first_blocks(KB); kb < KB; ++kb)
#pragma unroll
    for (int i = 0; i < 16; i += 2) mx = fmaxf(fmaxf(st.s[kb][i], st.s[kb][i + 1]), mx);
  return xhalf_max(mx);
}

// P(t) = online softmax of S(t); rescales O and the running sum when a row maximum moves.
// kmax_rel: last visible key of this lane's query relative to the tile (>= BN: no mask needed).
template <int D, int BN, class H>
SP_DEV void fwd_softmax(FwdState<D, BN>& st, float c, H&& hook) {
  constexpr int KB = BN / 32, DB = D / 32;
  hook(0);
  const float mx = fwd_rowmax_rest<D, BN>(st, st.mx);
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
    // pin: without a use here the optimiser sinks this arithmetic past the phase barrier that follows
    asm volatile("" : "+v"(st.p[kb][0]), "+v"(st.p[kb][1]));
  }
  st.l_run += l_add;
  asm volatile("" : "+v"(st.l_run));
}

// out = O / l, lse = (m + log2 l) ln 2; rows that saw no key: out = 0, lse = -inf.
template <int D, int BN>
SP_DEV void fwd_epilogue(const FwdArgs& a, FwdState<D, BN>& st, int myrow, int h, int b, int r, int g) {
  constexpr int DB = D / 32;
  const float l_tot = xhalf_sum(st.l_run);
  const bool has = l_tot > 0.f;
  const float inv = has ? 1.0f / l_tot : 0.f;
  if (myrow < a.s_q) {
    if (g == 0) {
      const float lse = has ? (st.m_run + __builtin_log2f(l_tot)) * kLn2 : -INFINITY;
      a.lse[(int64_t)r * a.lse_range_stride + ((int64_t)b * a.n_q_heads + h) * a.s_q + myrow] = lse;
    }
    const int64_t obase = (int64_t)r * a.out_range_stride + (int64_t)b * a.o_stride_b + (int64_t)myrow * a.o_stride_s +
                          (int64_t)h * a.o_stride_h;
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

// One matrix phase of the two-group kernel as an explicit software pipeline: the 2*KB*DB MFMAs of
// O^T += V(t-1)^T P(t-1)^T, then the KB*KS of S(t)^T = K(t) Q^T, numbered m = 0 .. N-1; the LDS reads of
// MFMA m+LOOK are issued right before MFMA m into a ring of LOOK+1 operand buffers, and scheduling
// fences keep that order (left to the scheduler, reads end up right in front of their MFMA whenever
// registers are short).
template <int D, int BN, bool WITH_PV, bool WITH_S, int LOOK>
struct FwdMatrixPhase {
  static constexpr int KB = BN / 32, DB = D / 32, KS = D / 16;
  static constexpr int N_PV = WITH_PV ? 2 * KB * DB : 0, N_S = WITH_S ? KB * KS : 0, N = N_PV + N_S;
  static constexpr int NBUF = LOOK + 1;
  const TrOffsets<D>& lo_v;    // V(t-1), transposed
  const RpOffsets<D>& lo_k;    // K(t), row-packed
  FwdState<D, BN>& st;
  bf16x8 abuf[NBUF];

  template <int M>
  SP_DEV void reads() {
    if constexpr (M < N_PV) {
      constexpr int db = M % DB, blk = M / DB;                 // blk = 2*kb + half: 16 keys each
      abuf[M % NBUF] = lds_tr<D>(lo_v, db, blk * 16 * D * 2);
    } else if constexpr (M < N) {
      constexpr int j = M - N_PV, ks = j / KB, kb = j % KB;
      abuf[M % NBUF] = lds_rp<D>(lo_k, ks, kb * 32 * D * 2);
    }
  }
  template <int M>
  SP_DEV void mfma() {
    if constexpr (M < N_PV) {
      constexpr int db = M % DB, blk = M / DB;
      st.o[db] = mfma32(abuf[M % NBUF], st.p[blk / 2][blk % 2], st.o[db]);
    } else {
      constexpr int j = M - N_PV, ks = j / KB, kb = j % KB;
      const f32x16 zero = {0};
      st.s[kb] = mfma32(abuf[M % NBUF], st.qreg[ks], ks == 0 ? zero : st.s[kb]);
    }
  }
  template <int M>
  SP_DEV void step() {
    if constexpr (M < N) {
      reads<M + LOOK>();
      SP_FENCE();
      mfma<M>();
      SP_FENCE();
      step<M + 1>();
    }
  }
  template <int M>
  SP_DEV void prologue() {
    if constexpr (M < LOOK) { reads<M>(); prologue<M + 1>(); }
  }
  SP_DEV void run() {
    SP_FENCE();
    matrix_phase_begin();
    prologue<0>();
    SP_FENCE();
    step<0>();
    matrix_phase_end();
    SP_FENCE();
  }
};

template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64) void attn_fwd_kernel(const FwdArgs a) {
  static_assert(NW == 8, "two groups of four waves");
  constexpr int BM = NW * 32, KS = D / 16, DB = D / 32, T = NW * 64;
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int KSLOTS = 3, VSLOTS = 2;
  constexpr int K_BASE = 0, V_BASE = KSLOTS * TILE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);      // known uniform to the compiler
  const bool group_b = wave_u >= NW / 2;
  // Work item: index -> (query block, q head, batch index x key range), the first fastest: the workgroup's own
  // index, or the next value of the ticket counter (surplus workgroups leave at once).
  int item = blockIdx.x;
  if (a.ticket) {
    unsigned* slot = reinterpret_cast<unsigned*>(smem);      // (the tile rings are not in use yet)
    if (threadIdx.x == 0) *slot = atomicAdd(a.ticket, 1u);
    __syncthreads();
    item = (int)*slot;
    __syncthreads();
    if (item >= a.items[0] * a.items[1] * a.items[2]) return;
  }
  item = __builtin_amdgcn_readfirstlane(item);
  const int per_z = a.items[0] * a.items[1];
  const int bz = __builtin_amdgcn_readfirstlane(item / per_z), item_xy = item - bz * per_z;
  const int h = __builtin_amdgcn_readfirstlane(item_xy / a.items[0]), bx = item_xy - h * a.items[0];
  const int qblk = a.items[0] - 1 - bx;
  const int b = bz / a.n_ranges, r = bz - b * a.n_ranges, hk = h / a.group;
  const int64_t kv_begin = a.range_begin[r], kv_end = a.range_end[r];      // this workgroup's key range
  const int m0 = qblk * BM, wrow0 = m0 + wave_u * 32;
  const int myrow = wrow0 + ql;
  const int myrow_c = myrow < a.s_q ? myrow : a.s_q - 1;

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

  const int64_t lo = kv_grid_origin(kv_begin, a.kv.n, BN);     // first key of the tile grid
  int64_t hi = kv_end;
  if (a.causal) {
    const int last_row = (m0 + BM < a.s_q ? m0 + BM : a.s_q);
    const int64_t lim = a.q_offset + last_row;
    hi = hi < lim ? hi : lim;
  }
  const int nt = hi > lo ? (int)((hi - lo + BN - 1) / BN) : 0;
  const float c = a.scale_log2e;

  if (nt > 0) {
    const int64_t head_off = (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
    auto key0_of = [&](int t) { return lo + (int64_t)t * BN; };
    // Per tile t a wave runs the matrix phase MM(t): O^T += V(t-1)^T P(t-1)^T, S(t)^T = K(t) Q^T, row maxima
    // of S(t); and the vector phase VV(t): P(t) = online softmax of S(t).  K(t) is read in MM(t) only, V(t) in
    // MM(t+1) only.  Tile copies are issued from vector phases only, by the four waves of the group that
    // is in one (next to the LDS reads and MFMAs of a matrix phase they stall the wave): group A copies
    // K(t+2) during VV(t) into a ring of three slots, group B copies V(t+1) during its VV(t) into a ring
    // of two, and each group waits for its copies at the end of its next matrix phase.  Copies are
    // branch-free: a tile past the end of the range re-copies the last tile (nobody reads it), rows
    // past the end of the chunk are clamped.  Each group walks its operand's chunk list tile by tile.
    constexpr int GT = T / 2;                            // threads of one group
    const int gtid = tid & (GT - 1);
    TileDma<D, BN, GT> dma;
    constexpr int PASSES = TileDma<D, BN, GT>::PASSES;   // copy instructions per tile and wave
    constexpr int HOOKS = 2 + BN / 32, PPH = (PASSES + HOOKS - 1) / HOOKS;   // copy instructions per softmax hook
    dma.init(gtid);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2;
    const unsigned smem_lds = lds_addr(smem);
    const int gwave_u = wave_u & (NW / 2 - 1);
    const bool copies_k = !group_b;
    const bf16_t* const* table = copies_k ? a.kv.k : a.kv.v;
    KvWalk walk;             // the next tile this group copies
    walk.seek(table, a.kv, lo, head_off, a.kv_stride_s);
    const int64_t kv_tile_step = (int64_t)BN * a.kv_stride_s;
    struct CopyJob { const bf16_t* src; unsigned dst; int rows; };
    // tile t (the one the walk stands on) into its ring slot; the walk moves on unless t is the last tile
    auto make_copy = [&](int t) {
      CopyJob j;
      j.src = walk.ptr;
      j.dst = smem_lds + (copies_k ? K_BASE + (t % KSLOTS) * TILE_BYTES : V_BASE + (t % VSLOTS) * TILE_BYTES);
      j.rows = walk.rows(a.kv, BN);
      if (t + 1 < nt) walk.step(table, a.kv, BN, kv_tile_step, head_off, a.kv_stride_s);
      return j;
    };
    auto copy_pass = [&](const CopyJob& j, int n) { dma.issue(j.dst, j.src, row_bytes, j.rows, gwave_u, n); };
    auto copy_all = [&](const CopyJob& j) {
      for (int n = 0; n < PASSES; ++n) copy_pass(j, n);
    };
    // vector phase of tile t that also copies one tile
    auto vector_phase = [&](const CopyJob& j) {
      fwd_softmax<D, BN>(st, c, [&](int part) {
        for (int n = part * PPH; n < (part + 1) * PPH && n < PASSES; ++n) copy_pass(j, n);
      });
    };
    // tail of a matrix phase: mask S(t) and take its row maxima (balances the two kinds of phase)
    auto rowmax_tile = [&](int t) {
      const int64_t key0 = key0_of(t);
      const bool need_mask = (key0 < kv_begin) || (key0 + BN > kv_end) || (a.causal && key0 + BN - 1 > a.q_offset + wrow0);
      const int t2 = fresh(tid);
      int kmin_rel = 0, kmax_rel = BN;
      if (need_mask) {       // first key of the range and last visible key of this lane's query, relative to the tile
        const int64_t kmin = kv_begin - key0;
        kmin_rel = kmin < 0 ? 0 : (int)kmin;
        const int64_t qpos = a.q_offset + wrow0 + (t2 & 31);
        int64_t kmax = kv_end - 1;
        if (a.causal && qpos < kmax) kmax = qpos;
        kmax -= key0;
        kmax_rel = kmax < -1 ? -1 : (kmax > BN ? BN : (int)kmax);
      }
      st.mx = fwd_rowmax_first<D, BN>(st, need_mask, kmin_rel, kmax_rel, (t2 >> 5) & 1);
      asm volatile("" : "+v"(st.mx));      // keep it on this side of the phase barrier
    };

    // prologue: K(0), K(1) (group A), V(0) (group B)
    if (copies_k) { copy_all(make_copy(0)); copy_all(make_copy(1)); }
    else copy_all(make_copy(0));
    wait_async();
    RpOffsets<D> lo_k;       // K(t), row-packed (registers are plentiful here: one offset per head_dim block)
    TrOffsets<D> lo_v;       // V(t-1), transposed
    lo_k.init(lane, (int)smem_lds + K_BASE);
    lo_v.init(lane, (int)smem_lds + V_BASE + TILE_BYTES);        // "V(-1)": never read
    __syncthreads();

    int kslot = 0, vslot = 1;       // slots of K(t) and V(t-1)
    auto advance = [&]() {
      lo_k.add(kslot == KSLOTS - 1 ? -(KSLOTS - 1) * TILE_BYTES : TILE_BYTES);
      lo_v.add(vslot ? -TILE_BYTES : TILE_BYTES);
      kslot = (kslot == KSLOTS - 1) ? 0 : kslot + 1;
      vslot ^= 1;
    };
    // Both groups run the same code; group B starts one phase (one barrier) later and group A idles
    // one phase at the end.
    if (group_b) phase_end();
    { FwdMatrixPhase<D, BN, false, true, kFwdLook> ph{lo_v, lo_k, st}; ph.run(); }
    rowmax_tile(0);
    advance();
    wait_async();
    phase_end();
    for (int t = 0; t + 1 < nt; ++t) {
      vector_phase(make_copy(copies_k ? t + 2 : t + 1));
      phase_end();
      { FwdMatrixPhase<D, BN, true, true, kFwdLook> ph{lo_v, lo_k, st}; ph.run(); }
      rowmax_tile(t + 1);
      advance();
      wait_async();                                      // the copies of the vector phase before have landed
      phase_end();
    }
    vector_phase(make_copy(copies_k ? nt + 1 : nt));
    phase_end();
    { FwdMatrixPhase<D, BN, true, false, kFwdLook> ph{lo_v, lo_k, st}; ph.run(); }
    wait_async();
    phase_end();
    if (!group_b) phase_end();
  }
  fwd_epilogue<D, BN>(a, st, myrow, h, b, r, g);
}

template <int D>
constexpr size_t fwd_lds_bytes() { return (size_t)5 * kFwdKeysPerTile * D * 2; }       // K ring of three, V ring of two

template <int D, int NW, int BN>
static hipError_t launch_fwd_t(const FwdArgs& a, int batch, hipStream_t st) {
  const int64_t items = (int64_t)a.items[0] * a.items[1] * a.items[2];
  // with a ticket counter: a quarter more workgroups than items (an XCD that is 10 % faster than the others takes
  // 10 % more than its eighth of the items; the surplus workgroups take a ticket, see that the items are gone and leave)
  const int64_t wgs = a.ticket ? items + items / 4 + 64 : items;
  dim3 grid((unsigned)wgs), block(NW * 64);
  hipLaunchKernelGGL((attn_fwd_kernel<D, NW, BN>), grid, block, fwd_lds_bytes<D>(), st, a);
  return hipGetLastError();
}

__global__ void zero_counter_kernel(unsigned* counter) { *counter = 0u; }
hipError_t launch_zero_counter(unsigned* counter, hipStream_t st) {
  hipLaunchKernelGGL(zero_counter_kernel, dim3(1), dim3(1), 0, st, counter);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs& a, int batch, int head_dim, hipStream_t st) {
  if (head_dim == 128) return launch_fwd_t<128, 8, kFwdKeysPerTile>(a, batch, st);
  return launch_fwd_t<64, 8, kFwdKeysPerTile>(a, batch, st);
}

hipError_t opt_in_fwd_kernels() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<128, 8, kFwdKeysPerTile>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)fwd_lds_bytes<128>());
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<64, 8, kFwdKeysPerTile>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)fwd_lds_bytes<64>());
}

}  // namespace slimpipe
