// Backward of slice-wise causal attention over a key range (paper Sec. 4.1.2: backward per slice,
// in reverse slice order, against the retained K/V; partial ranges: Sec. 4.2.2).
//
// With p_ij = exp(scale q_i.k_j - lse_i) on visible pairs and delta_i = dO_i . O_i:
//   dV_j = sum_i p_ij dO_i            dS_ij = p_ij (dO_i . v_j - delta_i)
//   dQ_i = scale sum_j dS_ij k_j      dK_j  = scale sum_i dS_ij q_i
// Two kernels, neither of which needs atomics or a layout change through LDS:
//   * dq kernel, query-stationary (same shape as the forward): S^T = K Q^T and dP^T = V dO^T
//     land with one query per lane, so lse/delta are per-lane scalars and dS^T feeds
//     dQ^T += K^T dS^T directly as the B operand (K through the transposed LDS read).
//   * dk/dv kernel, key-stationary: each wave owns 32 keys (K, V as B operands in registers,
//     dK^T/dV^T accumulators in registers) and walks the query tiles of every head of its GQA
//     group in a fixed order: S = Q K^T, dP = dO V^T land with one key per lane and 16 query rows
//     in the registers, which is the B operand of dV^T += dO^T P and dK^T += Q^T dS.
//     One workgroup owns a key row outright, so dK/dV are bit-reproducible.
#include "kernels.hpp"
#include "tile_common.hpp"

namespace slimpipe {

// ------------------------------------------------------------------------------------ delta
// delta[b,h,r] = -sum_d dO[b,r,h,d] * O[b,r,h,d] (NEGATED: the dk/dv kernel starts the accumulator of dP
// from it, so that the matrix pipe delivers dP - delta) and lse2 = lse * log2(e) (+inf for rows that saw no
// key, which makes every p of the row exp2(-inf) = 0).  One 16-byte chunk per lane, D/8 lanes per row.
template <int D>
__global__ __launch_bounds__(256) void attn_delta_kernel(const BwdArgs a, int batch) {
  constexpr int NC = D / 8;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid < 8) {      // the dq and dk/dv kernels of this call, later on the stream, count from zero
    if (gid == 0 && a.ticket_dq) *a.ticket_dq = 0u;
    if (a.ticket_dkdv) a.ticket_dkdv[gid] = 0u;      // one counter per XCD
  }
  const int64_t rh = gid / NC;                 // (b, r, h) flattened
  const int c = (int)(gid % NC);
  const int64_t total = (int64_t)batch * a.s_q * a.n_q_heads;
  float acc = 0.f;
  int h = 0, r = 0, b = 0;
  if (rh < total) {
    h = (int)(rh % a.n_q_heads);
    const int64_t br = rh / a.n_q_heads;
    r = (int)(br % a.s_q);
    b = (int)(br / a.s_q);
    const int64_t off = (int64_t)b * a.o_stride_b + (int64_t)r * a.o_stride_s + (int64_t)h * a.o_stride_h + c * 8;
    const bf16x8 o = *reinterpret_cast<const bf16x8*>(a.out + off);
    const int64_t doff = (int64_t)b * a.do_stride_b + (int64_t)r * a.do_stride_s + (int64_t)h * a.do_stride_h + c * 8;
    const bf16x8 d = *reinterpret_cast<const bf16x8*>(a.d_out + doff);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc += (float)o[j] * (float)d[j];
  }
#pragma unroll
  for (int w = NC / 2; w >= 1; w >>= 1) acc += __shfl_xor(acc, w, 64);
  if (rh < total && c == 0) {
    const int64_t sidx = ((int64_t)b * a.n_q_heads + h) * a.s_q + r;
    a.delta[sidx] = -acc;
    const float l = a.lse[sidx];
    a.lse2[sidx] = (l == -INFINITY) ? INFINITY : l * kLog2e;
  }
}

hipError_t launch_delta(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  const int64_t lanes = (int64_t)batch * a.s_q * a.n_q_heads * (head_dim / 8);
  dim3 grid((unsigned)((lanes + 255) / 256)), block(256);
  if (head_dim == 128) hipLaunchKernelGGL(attn_delta_kernel<128>, grid, block, 0, st, a, batch);
  else hipLaunchKernelGGL(attn_delta_kernel<64>, grid, block, 0, st, a, batch);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------ dq
// Query-stationary: 8 waves x 32 query rows of one head; Q lives in registers and dO in LDS as B
// operands (both in registers do not fit 256 registers a wave next to the accumulators), dQ^T
// accumulates in registers, K/V tiles of BN keys stream through LDS.  Per tile u a wave runs
//   matrix phase MM(u): dQ^T += K(u-1)^T dS(u-1)^T   (transposed read of K(u-1))
//                       S(u)^T = K(u) Q^T,  dP(u)^T = V(u) dO^T          (row-packed reads)
//   vector phase VV(u): dS(u)^T = exp2(c S - lse2) (dP - delta), packed to bf16
// Waves 0-3 (group A) and 4-7 (group B) run the same sequence one phase apart with one workgroup
// barrier per phase, so each SIMD hosts one wave in each kind of phase (the VALU work of one covers
// the matrix pipe time of the other).  K lives in a ring of four LDS slots, V in a ring of two; the
// group that is in a vector phase issues the asynchronous copies of the tiles two steps ahead
// (A: K(u+2), B: V(u+2)) and waits for them at the end of its next matrix phase.
template <int D, int BN>
struct DqState {
  static constexpr int KS = D / 16, DB = D / 32, KB = BN / 32;
  bf16x8 qreg[KS];
  f32x16 dq[DB];
  f32x16 s[KB], dp[KB];
  bf16x8 ds[KB][2];
  float lse2;
  f32x16 ndelta;      // -delta of the lane's query in all 16 registers: the initial accumulator of every dP tile,
                      // so that the matrix pipe delivers dP - delta (the vector unit is the scarcer resource)
};

// One matrix phase as an explicit software pipeline.  The MFMAs are numbered m = 0 .. N-1 (first the
// 2*KB*DB of dQ^T += K(u-1)^T dS^T, then per head_dim block ks the 2*KB of S0, dP0, S1, dP1, ...);
// the LDS reads of MFMA m+LOOK are issued right before MFMA m into a ring of LOOK+1 operand buffers,
// and scheduling fences keep that order.  (Leaving the order to the scheduler gave reads right in
// front of their MFMA whenever registers were short: about 60 cycles an MFMA instead of 32.)
template <int D, int BN, bool WITH_DQ, bool WITH_SCORES, int LOOK>
struct DqMatrixPhase {
  static constexpr int KB = BN / 32, DB = D / 32, KS = D / 16;
  static constexpr int N_DQ = WITH_DQ ? 2 * KB * DB : 0, N_SC = WITH_SCORES ? 2 * KB * KS : 0, N = N_DQ + N_SC;
  static constexpr int NBUF = LOOK + 1;
  const TrBase<D>& lo_kt;
  const RpBase<D>& lo_k;
  const RpBase<D>& lo_v;
  const RpBase<D>& lo_do;
  DqState<D, BN>& st;
  bf16x8 abuf[NBUF];
  bf16x8 dob[2];

  template <int M>
  SP_DEV void reads() {
    if constexpr (M < N_DQ) {
      constexpr int db = M % DB, blk = M / DB;                 // blk = 2*kb + half: 16 keys each
      abuf[M % NBUF] = lds_tr<D>(lo_kt, db, blk * 16 * D * 2);
    } else if constexpr (M < N) {
      constexpr int j = M - N_DQ, ks = j / (2 * KB), r = j % (2 * KB), kb = r / 2;
      if constexpr ((r & 1) == 0) {
        abuf[M % NBUF] = lds_rp<D>(lo_k, ks, kb * 32 * D * 2);
      } else {
        abuf[M % NBUF] = lds_rp<D>(lo_v, ks, kb * 32 * D * 2);
        if constexpr (kb == 0) dob[ks & 1] = lds_rp<D>(lo_do, ks, 0);
      }
    }
  }
  template <int M>
  SP_DEV void mfma() {
    if constexpr (M < N_DQ) {
      constexpr int db = M % DB, blk = M / DB;
      st.dq[db] = mfma32(abuf[M % NBUF], st.ds[blk / 2][blk % 2], st.dq[db]);
    } else {
      constexpr int j = M - N_DQ, ks = j / (2 * KB), r = j % (2 * KB), kb = r / 2;
      const f32x16 zero = {0};
      if constexpr ((r & 1) == 0) st.s[kb] = mfma32(abuf[M % NBUF], st.qreg[ks], ks == 0 ? zero : st.s[kb]);
      else st.dp[kb] = mfma32(abuf[M % NBUF], dob[ks & 1], ks == 0 ? st.ndelta : st.dp[kb]);
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

template <int D, int BN, bool WITH_DQ, bool WITH_SCORES>
SP_DEV void dq_matrix_phase(const TrBase<D>& lo_kt, const RpBase<D>& lo_k, const RpBase<D>& lo_v,
                            const RpBase<D>& lo_do, DqState<D, BN>& st) {
  DqMatrixPhase<D, BN, WITH_DQ, WITH_SCORES, 2> ph{lo_kt, lo_k, lo_v, lo_do, st};
  ph.run();
}

// dS^T = p (dP^T - delta) with p = exp2(c S^T - lse2) on visible pairs (`dp` arrives as dP^T - delta); `hook(i)`, i = 0..3, is called at
// four points spread over the phase (asynchronous tile copies ride there).
template <int D, int BN, class H>
SP_DEV void dq_vector_phase(DqState<D, BN>& st, float c, bool need_mask, int kmin_rel, int kmax_rel, int g, H&& hook) {
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
        st.s[kb][i] = ((key >= kmin_lane) & (key <= kmax_lane)) ? st.s[kb][i] : -INFINITY;     // exp2(-inf) = 0
      }
  }
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      hook(kb * 2 + half);
#pragma unroll
      for (int i = 8 * half; i < 8 * half + 8; ++i) {
        const float p = exp2_fast(__builtin_fmaf(st.s[kb][i], c, -st.lse2));
        st.s[kb][i] = p * st.dp[kb][i];          // dp arrives as dP - delta
      }
      st.ds[kb][half] = pack8(st.s[kb], 8 * half);
      // pin: without a use here the optimiser sinks this arithmetic past the phase barrier
      asm volatile("" : "+v"(st.ds[kb][half]));
    }
}

template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dq_kernel(const BwdArgs a) {
  static_assert(NW == 8, "two groups of four waves");
  constexpr int BM = NW * 32, KS = D / 16, DB = D / 32, T = NW * 64, GT = T / 2;
  constexpr int TILE_BYTES = BN * D * 2;
  constexpr int KSLOTS = 4, VSLOTS = 2;
  constexpr int K_BASE = 0, V_BASE = KSLOTS * TILE_BYTES, DO_BASE = (KSLOTS + VSLOTS) * TILE_BYTES;
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);      // known uniform to the compiler
  const bool group_b = wave_u >= NW / 2;
  const int gtid = tid & (GT - 1);
  // Work item: index -> (query block, q head, batch index x key range), the first fastest: the workgroup's own
  // index, or the next value of the ticket counter (surplus workgroups leave at once).
  int item = blockIdx.x;
  if (a.ticket_dq) {
    unsigned* slot = reinterpret_cast<unsigned*>(smem);      // (the tile rings are not in use yet)
    if (threadIdx.x == 0) *slot = atomicAdd(a.ticket_dq, 1u);
    __syncthreads();
    item = (int)*slot;
    __syncthreads();
    if (item >= a.dq_items[0] * a.dq_items[1] * a.dq_items[2]) return;
  }
  item = __builtin_amdgcn_readfirstlane(item);
  const int per_z = a.dq_items[0] * a.dq_items[1];
  const int bz = __builtin_amdgcn_readfirstlane(item / per_z), item_xy = item - bz * per_z;
  const int h = __builtin_amdgcn_readfirstlane(item_xy / a.dq_items[0]), bx = item_xy - h * a.dq_items[0];
  const int qblk = a.dq_items[0] - 1 - bx;
  const int b = bz / a.n_dq_ranges, r = bz - b * a.n_dq_ranges, hk = h / a.group;
  const int64_t kv_begin = a.dq_range_begin[r], kv_end = a.dq_range_end[r];      // this workgroup's key range
  const int m0 = qblk * BM, wrow0 = m0 + wave_u * 32;
  const int myrow = wrow0 + ql;
  const int myrow_c = myrow < a.s_q ? myrow : a.s_q - 1;

  DqState<D, BN> st;
  {
    const bf16_t* qp = a.q + (int64_t)b * a.q_stride_b + (int64_t)myrow_c * a.q_stride_s + (int64_t)h * a.q_stride_h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) st.qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * g);
    const int64_t stat = ((int64_t)b * a.n_q_heads + h) * a.s_q + myrow_c;
    st.lse2 = a.lse2[stat];          // +inf for an empty row -> p = 0
    const float nd = a.delta[stat];  // (stored negated)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.ndelta[i] = nd;
  }
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.dq[db][i] = 0.f;

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
    TileDma<D, BN, GT> dma;
    constexpr int PASSES = TileDma<D, BN, GT>::PASSES;
    static_assert(PASSES <= 4, "one copy instruction per hook of the vector phase");
    dma.init(gtid);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2;
    const unsigned smem_lds = lds_addr(smem);
    const int gwave_u = wave_u & (NW / 2 - 1);
    // Group A copies K tiles, group B V tiles; each walks its operand's chunk list tile by tile.
    const bool copies_k = !group_b;
    const bf16_t* const* table = copies_k ? a.kv.k : a.kv.v;
    KvWalk walk;             // the next tile this group copies
    walk.seek(table, a.kv, lo, head_off, a.kv_stride_s);
    const int64_t kv_tile_step = (int64_t)BN * a.kv_stride_s;
    struct CopyJob { const bf16_t* src; unsigned dst; int rows; };
    // tile t (the one the walk stands on) of K (slot t % KSLOTS) or V (slot t % VSLOTS); the walk moves on
    // unless t is the last tile: past the end the last tile is copied again
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
    auto vector_phase = [&](int u, const CopyJob& j) {
      const int64_t key0 = key0_of(u);
      const bool need_mask = (key0 < kv_begin) || (key0 + BN > kv_end) || (a.causal && key0 + BN - 1 > a.q_offset + wrow0);
      // first key of the range and last visible key of this lane's query relative to the tile: worked out in
      // the masked tiles only, from the thread index (nothing lane-dependent is kept in registers across the
      // loop for it)
      const int t2 = fresh(tid);
      int kmin_rel = 0, kmax_rel = BN;
      if (need_mask) {
        const int64_t kmin = kv_begin - key0;
        kmin_rel = kmin < 0 ? 0 : (int)kmin;
        const int64_t qpos = a.q_offset + wrow0 + (t2 & 31);
        int64_t kmax = kv_end - 1;
        if (a.causal && qpos < kmax) kmax = qpos;
        kmax -= key0;
        kmax_rel = kmax < -1 ? -1 : (kmax > BN ? BN : (int)kmax);
      }
      dq_vector_phase<D, BN>(st, c, need_mask, kmin_rel, kmax_rel, (t2 >> 5) & 1, [&](int part) { if (part < PASSES) copy_pass(j, part); });
    };

    // prologue: the dO rows of the block (all threads), K(0), K(1) (group A), V(0), V(1) (group B)
    {
      TileDma<D, BM, T> dma_do;
      dma_do.init(tid);
      const bf16_t* dobase = a.d_out + (int64_t)b * a.do_stride_b + (int64_t)m0 * a.do_stride_s + (int64_t)h * a.do_stride_h;
      for (int n = 0; n < TileDma<D, BM, T>::PASSES; ++n)
        dma_do.issue(smem_lds + DO_BASE, dobase, (uint32_t)a.do_stride_s * 2, a.s_q - m0, wave_u, n);
    }
    copy_all(make_copy(0));
    copy_all(make_copy(1));
    wait_async();
    TrBase<D> lo_kt;         // K(u-1), transposed
    RpBase<D> lo_k, lo_v;    // K(u), V(u), row-packed
    lo_kt.init(lane, (int)smem_lds + K_BASE + (KSLOTS - 1) * TILE_BYTES);      // "K(-1)": never read
    lo_k.init(lane, (int)smem_lds + K_BASE);
    lo_v.init(lane, (int)smem_lds + V_BASE);
    RpBase<D> lo_do;         // this wave's 32 rows of dO
    lo_do.init(lane, (int)smem_lds + DO_BASE + wave * 32 * D * 2);
    __syncthreads();

    // ring bookkeeping after matrix phase u: every pointer moves one tile on
    int kslot = 0;           // slot of K(u)
    auto advance = [&]() {
      const int dk = (kslot == KSLOTS - 1) ? -(KSLOTS - 1) * TILE_BYTES : TILE_BYTES;
      const int dkt = (kslot == 0) ? -(KSLOTS - 1) * TILE_BYTES : TILE_BYTES;   // K(u-1) slot = kslot - 1
      lo_k.add(dk);
      lo_kt.add(dkt);
      lo_v.add((kslot & 1) ? -TILE_BYTES : TILE_BYTES);
      kslot = (kslot == KSLOTS - 1) ? 0 : kslot + 1;
    };
    // Both groups run the same code; group B starts one phase (one barrier) later and group A idles
    // one phase at the end.  Group A copies K tiles, group B V tiles.
    if (group_b) phase_end();
    dq_matrix_phase<D, BN, false, true>(lo_kt, lo_k, lo_v, lo_do, st);       // scores of tile 0
    advance();
    wait_async();
    phase_end();
    for (int u = 0; u + 1 < nt; ++u) {
      vector_phase(u, make_copy(u + 2));                 // tile u+2 rides along
      phase_end();
      dq_matrix_phase<D, BN, true, true>(lo_kt, lo_k, lo_v, lo_do, st);      // dQ of tile u, scores of tile u+1
      advance();
      wait_async();                                      // the copies of the vector phase before have landed
      phase_end();
    }
    vector_phase(nt - 1, make_copy(nt + 1));             // (copies the last tile once more)
    phase_end();
    dq_matrix_phase<D, BN, true, false>(lo_kt, lo_k, lo_v, lo_do, st);       // dQ of the last tile
    wait_async();
    phase_end();
    if (!group_b) phase_end();
  }

  const int tid_out = fresh(tid), myrow_out = wrow0 + (tid_out & 31), g_out = (tid_out >> 5) & 1;
  if (myrow_out < a.s_q) {
    const int64_t base = (int64_t)r * a.dq_range_stride + (int64_t)b * a.dq_stride_b + (int64_t)myrow_out * a.dq_stride_s +
                         (int64_t)h * a.dq_stride_h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 32 * db + 8 * i4 + 4 * g_out;
        f32x4 v4 = {st.dq[db][4 * i4] * a.scale, st.dq[db][4 * i4 + 1] * a.scale, st.dq[db][4 * i4 + 2] * a.scale,
                    st.dq[db][4 * i4 + 3] * a.scale};
        if (a.dq_f32) {
          f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.dq) + base + d);
          if (a.dq_accumulate) v4 += *dst;
          *dst = v4;
        } else {
          *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(a.dq) + base + d) = __builtin_convertvector(v4, bf16x4);
        }
      }
  }
}

constexpr int kDqKeysPerTile = 64;
template <int D>
constexpr size_t dq_lds_bytes() { return (size_t)6 * kDqKeysPerTile * D * 2 + (size_t)256 * D * 2; }   // 4 K slots + 2 V slots + dO rows

template <int D, int NW, int BN>
static hipError_t launch_dq_t(const BwdArgs& a, int batch, hipStream_t st) {
  constexpr int BM = NW * 32;
  static_assert(BM == 256 && BN == kDqKeysPerTile, "dq_lds_bytes assumes this shape");
  const int64_t items = (int64_t)a.dq_items[0] * a.dq_items[1] * a.dq_items[2];
  const int64_t wgs = a.ticket_dq ? items + items / 4 + 64 : items;      // (see launch_dkdv_t)
  dim3 grid((unsigned)wgs), block(NW * 64);
  hipLaunchKernelGGL((attn_bwd_dq_kernel<D, NW, BN>), grid, block, dq_lds_bytes<D>(), st, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dq(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  if (head_dim == 128) return launch_dq_t<128, 8, kDqKeysPerTile>(a, batch, st);
  return launch_dq_t<64, 8, kDqKeysPerTile>(a, batch, st);
}

// ------------------------------------------------------------------------------------ dk / dv
// Key-stationary twin of the dq kernel: 8 waves x 32 keys of one KV head; K lives in registers and V
// in LDS as B operands, dK^T and dV^T accumulate in registers, and the query rows that can see the
// keys (every query tile, for every head of the GQA group, in a fixed order: the sums are
// reproducible) stream through LDS as tiles of 32 rows of Q and dO.  Per tile u a wave runs
//   matrix phase MM(u): dV^T += dO(u-1)^T P(u-1),  dK^T += Q(u-1)^T dS(u-1)    (transposed reads)
//                       S(u) = Q(u) K^T,  dP(u) = dO(u) V^T - delta              (row-packed reads; the
//                       accumulator of dP starts from -delta, and lse2 of the tile is fetched on the way)
//   vector phase VV(u): P = exp2(c S - lse2),  dS = P (dP - delta), packed to bf16
// and the two wave groups run one phase apart exactly as in the dq kernel.  (One wave per SIMD with
// twice the registers cannot overlap the two kinds of work: a wave that has issued an MFMA issues
// nothing else until the matrix pipe has taken it, so vector work only hides behind the MFMAs of
// ANOTHER wave of the same SIMD.)  Q and dO tiles sit in rings of four LDS slots, the row statistics
// in a ring of four; group A copies Q(u+2) and the statistics, group B copies dO(u+2).
template <int D>
struct DkdvState {
  static constexpr int KS = D / 16, DB = D / 32;
  bf16x8 kreg[KS];
  f32x16 dk[DB], dv[DB];
  f32x16 s, dp;
  bf16x8 pb[2], dsb[2];      // 16 query rows each
  f32x4 lse2v[4];            // lse2 of this lane's 16 rows of the tile in `s`: fetched by the matrix phase (the LDS
                             // latency passes while the score MFMAs run), used first thing by the vector phase
};

// LDS layout (bytes): Q ring, dO ring, V rows of the workgroup, statistics ring
template <int D, int NW>
struct DkdvLds {
  static constexpr int BMQ = 32, SLOTS = 4;
  static constexpr int TILE_BYTES = BMQ * D * 2;
  static constexpr int Q_BASE = 0, DO_BASE = SLOTS * TILE_BYTES, V_BASE = 2 * SLOTS * TILE_BYTES;
  static constexpr int V_BYTES = NW * 32 * D * 2;
  static constexpr int STAT_BASE = V_BASE + V_BYTES;          // [SLOTS][lse2[BMQ], delta[BMQ]] floats
  static constexpr int STAT_BYTES = 2 * BMQ * 4;
  static constexpr int TOTAL = STAT_BASE + SLOTS * STAT_BYTES;
};

template <int D, int NW, bool WITH_ACC, bool WITH_SCORES, int LOOK>
struct DkdvMatrixPhase {
  using L = DkdvLds<D, NW>;
  static constexpr int KS = D / 16, DB = D / 32;
  static constexpr int N_AC = WITH_ACC ? 4 * DB : 0, N_SC = WITH_SCORES ? 2 * KS : 0, N = N_AC + N_SC;
  static constexpr int NBUF = LOOK + 1, HALF = 16 * D * 2;
  const TrBase<D>& lo_qt;      // Q(u-1), transposed; dO(u-1) sits DO_BASE further
  const RpBase<D>& lo_q;       // Q(u), row-packed; dO(u) sits DO_BASE further
  const RpBase<D>& lo_v;       // this wave's 32 rows of V
  DkdvState<D>& st;
  const float* stat;           // LDS: lse2 of the rows of tile u, this lane's half (rows 8 i4 + 4 g .. + 3 at [8 i4 .. + 3]);
                               // -delta of the same rows 32 floats further
  bf16x8 abuf[NBUF];
  bf16x8 vb[2];

  template <int M>
  SP_DEV void reads() {
    if constexpr (WITH_SCORES && M == N_AC + LOOK + 2) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) st.lse2v[i4] = *reinterpret_cast<const f32x4*>(stat + 8 * i4);
    }
    // the accumulator of dP(u) starts from -delta of its rows (dP of the tile before was packed into dsb by the
    // vector phase and is dead): the matrix pipe delivers dP - delta
    if constexpr (WITH_SCORES && M == (N_AC > 0 ? 2 : 0)) {
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 nd = *reinterpret_cast<const f32x4*>(stat + 32 + 8 * i4);
#pragma unroll
        for (int e = 0; e < 4; ++e) st.dp[4 * i4 + e] = nd[e];
      }
    }
    if constexpr (M < N_AC) {
      constexpr int h = M / (2 * DB), db = (M % (2 * DB)) / 2;
      abuf[M % NBUF] = lds_tr<D>(lo_qt, db, ((M & 1) ? 0 : L::DO_BASE) + h * HALF);
    } else if constexpr (M < N) {
      constexpr int j = M - N_AC, ks = j / 2;
      if constexpr ((j & 1) == 0) {
        abuf[M % NBUF] = lds_rp<D>(lo_q, ks, 0);
      } else {
        abuf[M % NBUF] = lds_rp<D>(lo_q, ks, L::DO_BASE);
        vb[ks & 1] = lds_rp<D>(lo_v, ks, 0);
      }
    }
  }
  template <int M>
  SP_DEV void mfma() {
    if constexpr (M < N_AC) {
      constexpr int h = M / (2 * DB), db = (M % (2 * DB)) / 2;
      if constexpr ((M & 1) == 0) st.dv[db] = mfma32(abuf[M % NBUF], st.pb[h], st.dv[db]);
      else st.dk[db] = mfma32(abuf[M % NBUF], st.dsb[h], st.dk[db]);
    } else {
      constexpr int j = M - N_AC, ks = j / 2;
      const f32x16 zero = {0};
      if constexpr ((j & 1) == 0) st.s = mfma32(abuf[M % NBUF], st.kreg[ks], ks == 0 ? zero : st.s);
      else st.dp = mfma32(abuf[M % NBUF], vb[ks & 1], st.dp);
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

// P = exp2(c S - lse2) on visible pairs, dS = P (dP - delta), where `dp` arrives as dP - delta; element i of a lane is query row
// 8*(i/4) + 4g + i%4 of the tile, the lane's column is its key.  `hook(i)`, i = 0..3, is called at four
// points spread over the phase (asynchronous tile copies ride there).
template <int D, class H>
SP_DEV void dkdv_vector_phase(DkdvState<D>& st, const float* stat, float c, bool need_mask, int rmin_rel, int rmax_rel,
                              int g, H&& hook) {
  if (need_mask) {
    // row (8*(i/4) + 4g + i%4) in [rmin_rel, rmax_rel), with the lane's part moved to the bounds: the row
    // numbers are immediates then (a register per element otherwise, hoisted out of the tile loop)
    const int lo = rmin_rel - 4 * g, hi = rmax_rel - 4 * g;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = 8 * (i >> 2) + (i & 3);
      st.s[i] = ((r >= lo) & (r < hi)) ? st.s[i] : -INFINITY;      // exp2(-inf) = 0
    }
  }
  // Stage by stage over all 16 elements, so that neighbouring instructions do not depend on each other.
  // No LDS read here: lse2 is in registers (the matrix phase fetched it) and delta is in dP already.  This
  // phase is the longer of the two, and an LDS read in it waits for about 280 cycles behind the reads of the
  // group that is in its matrix phase.
  hook(0);
#pragma unroll
  for (int i = 0; i < 16; ++i) st.s[i] = __builtin_fmaf(st.s[i], c, -st.lse2v[i >> 2][i & 3]);
  hook(1);
#pragma unroll
  for (int i = 0; i < 16; ++i) st.s[i] = exp2_fast(st.s[i]);
  hook(2);
#pragma unroll
  for (int i = 0; i < 16; ++i) st.dp[i] *= st.s[i];       // dp holds dP - delta
  hook(3);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    st.pb[h] = pack8(st.s, 8 * h);
    st.dsb[h] = pack8(st.dp, 8 * h);
    // pin: without a use here the optimiser sinks this arithmetic past the phase barrier
    asm volatile("" : "+v"(st.pb[h]), "+v"(st.dsb[h]));
  }
}

static_assert((DkdvLds<128, 8>::SLOTS & (DkdvLds<128, 8>::SLOTS - 1)) == 0, "ring slots are stepped with a mask");

// One work item: index -> (key tile * n_split + chunk of that tile's query stream, kv head, batch index), the first
// fastest.
template <int D, int NW>
SP_DEV void dkdv_item(const BwdArgs& a, int item, char* smem) {
  static_assert(NW == 8, "two groups of four waves");
  using L = DkdvLds<D, NW>;
  constexpr int BNK = NW * 32, BMQ = L::BMQ, KS = D / 16, DB = D / 32, T = NW * 64, GT = T / 2;
  constexpr int TILE_BYTES = L::TILE_BYTES, SLOTS = L::SLOTS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);      // known uniform to the compiler
  const bool group_b = wave_u >= NW / 2;
  const int gtid = tid & (GT - 1);
  // (the quotients come out of vector instructions: read them back so that the compiler knows they are uniform)
  item = __builtin_amdgcn_readfirstlane(item);
  const int per_b = a.dkdv_items[0] * a.dkdv_items[1];
  const int b = __builtin_amdgcn_readfirstlane(item / per_b), item_hb = item - b * per_b;
  const int hk = __builtin_amdgcn_readfirstlane(item_hb / a.dkdv_items[0]), item_x = item_hb - hk * a.dkdv_items[0];
  const int ktile = __builtin_amdgcn_readfirstlane((int)((unsigned)item_x / (unsigned)a.n_split));
  const int split = item_x - ktile * a.n_split;
  // key tiles sit on the grid of kv_grid_origin (absolute multiples of 256 when K/V are chunked): a tile
  // lies inside one chunk; keys of the first tile before kv_begin are computed and not stored
  const int64_t grid0 = kv_grid_origin(a.kv_begin, a.kv.n, BNK);
  const int64_t tile_key0 = grid0 + (int64_t)ktile * BNK;
  const int kchunk = a.kv.n > 1 ? __builtin_amdgcn_readfirstlane((int)(tile_key0 / a.kv.len)) : 0;
  const int64_t chunk_row0 = tile_key0 - (int64_t)kchunk * a.kv.len;      // the tile's first row inside its chunk
  const int64_t head_off = (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
  const int64_t mykey = tile_key0 + wave_u * 32 + ql;
  const int64_t mykey_c = mykey < a.kv_end ? mykey : a.kv_end - 1;

  DkdvState<D> st;
  {
    // K as B operand: column = my key, k-slots = head_dim 16*ks + 8g ..
    const bf16_t* kp = a.kv.k[kchunk] + head_off + (chunk_row0 + (mykey_c - tile_key0)) * a.kv_stride_s;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) st.kreg[ks] = *reinterpret_cast<const bf16x8*>(kp + 16 * ks + 8 * g);
  }
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { st.dk[db][i] = 0.f; st.dv[db][i] = 0.f; }

  // Query tiles that can see this key tile: [qt0, nqt).  Tiles that need a mask (they straddle the
  // causal diagonal of this key tile, or hold rows past s_q) are walked first, for every head of the
  // group, then the unmasked rest.
  const int nqt = (a.s_q + BMQ - 1) / BMQ;
  int qt0 = 0, qtm = 0;                                      // masked: [qt0, qtm) (+ a partial last tile)
  if (a.causal && tile_key0 > a.q_offset) {
    const int64_t first = tile_key0 - a.q_offset;            // first row that sees tile_key0
    qt0 = first >= a.s_q ? nqt : (int)(first / BMQ);
  }
  if (a.causal) {
    const int64_t full = tile_key0 + BNK - 1 - a.q_offset;   // first row that sees every key of the tile
    qtm = full <= 0 ? 0 : (full >= a.s_q ? nqt : (int)((full + BMQ - 1) / BMQ));
  }
  if (qtm < qt0) qtm = qt0;
  const bool partial_last = (a.s_q % BMQ) != 0 && nqt - 1 >= qtm;
  const int nm = (qtm - qt0) + (partial_last ? 1 : 0);       // masked tiles per head
  const int nu = (nqt - qtm) - (partial_last ? 1 : 0);       // unmasked tiles per head
  const int total_m = nm * a.group, total = (nm + nu) * a.group;
  const float c = a.scale_log2e;
  // first row (within the slice) that sees this lane's key
  // this workgroup's part of the stream: tiles [seq_lo, seq_hi)
  const int seq_lo = __builtin_amdgcn_readfirstlane((int)((int64_t)total * split / a.n_split));
  const int seq_hi = __builtin_amdgcn_readfirstlane((int)((int64_t)total * (split + 1) / a.n_split));
  const int cnt = seq_hi - seq_lo;

  if (cnt > 0) {
    // lse2 and delta are two arrays of one workspace; (a per-lane choice between the two pointers would
    // become a vector load of the kernel argument, and the wait for it would sit inside the loop)
    const int64_t stat_gap = a.delta - a.lse2;
    TileDma<D, BMQ, GT> dma;
    constexpr int PASSES = TileDma<D, BMQ, GT>::PASSES;
    static_assert(PASSES <= 3, "copy instructions of a tile fit the hooks of a vector phase");
    dma.init(gtid);
    const unsigned smem_lds = lds_addr(smem);
    const int gwave_u = wave_u & (NW / 2 - 1);
    // this group's operand: Q (group A, with the row statistics) or dO (group B)
    const bool copies_q = !group_b;
    const bf16_t* const src_base = copies_q ? a.q + (int64_t)b * a.q_stride_b : a.d_out + (int64_t)b * a.do_stride_b;
    const int64_t src_stride_h = copies_q ? a.q_stride_h : a.do_stride_h;
    const int64_t src_stride_s = copies_q ? a.q_stride_s : a.do_stride_s;
    // lanes 0..31 read lse2, lanes 32..63 delta: one uniform base (the lower array) + a 32-bit lane offset
    // (the workspace is far below 4 GB)
    const float* const stat_base = (stat_gap < 0 ? a.delta : a.lse2) + (int64_t)b * a.n_q_heads * a.s_q;
    const uint32_t stat_off_lse2 = stat_gap < 0 ? (uint32_t)(-stat_gap) * 4u : 0u, stat_off_delta = stat_gap < 0 ? 0u : (uint32_t)stat_gap * 4u;
    const uint32_t src_row_bytes = (uint32_t)src_stride_s * 2;
    const int64_t src_tile_step = src_stride_s * BMQ;

    // Copy cursor over the stream of query tiles: masked tiles of head 0, 1, .. of the group, then the
    // unmasked tiles of head 0, 1, ..  The stream is a sequence of RUNS of tiles that follow each other in
    // one head; inside a run a step is a decrement and three additions, and only the start of a run
    // costs products and selects.  (A wave issues in order: every scalar instruction of the vector
    // phase, of which the first version of this cursor had a hundred per tile, delays the vector work
    // behind it.)  It stays on the last tile of the chunk once it is there.
    struct Cursor {
      int seq;               // index of the tile in the stream
      int run_left;          // tiles of the current run from this one on (cut at the end of the chunk)
      int run_len;           // tiles of the current run from its first tile of this chunk on
      int hh, r;             // head within the group, index of the run's first tile in the head's masked / unmasked list
      bool unmasked;
      int row0;              // first query row of the tile
      const bf16_t* tile;    // global address of its first row of Q / dO
      const float* stat;     // and of its first row statistic
    };
    auto run_start = [&](Cursor& cur) {
      int qt, len;
      if (cur.unmasked) { qt = qtm + cur.r; len = nu - cur.r; }
      else if (cur.r < qtm - qt0) { qt = qt0 + cur.r; len = (qtm - qt0) - cur.r; }
      else { qt = nqt - 1; len = 1; }                      // the partial last tile of the slice
      const int room = seq_hi - cur.seq;
      cur.run_left = cur.run_len = len < room ? len : room;
      cur.row0 = qt * BMQ;
      const int h = hk * a.group + cur.hh;
      cur.tile = uniform_ptr(src_base + h * src_stride_h + cur.row0 * src_stride_s);
      cur.stat = uniform_ptr(stat_base + (int64_t)h * a.s_q + cur.row0);
    };
    auto cursor_begin = [&]() {
      Cursor cur;
      cur.seq = seq_lo;
      cur.unmasked = seq_lo >= total_m;
      const int u = cur.unmasked ? seq_lo - total_m : seq_lo, per = cur.unmasked ? nu : nm;   // per > 0: the chunk is not empty
      cur.hh = __builtin_amdgcn_readfirstlane(u / per);
      cur.r = u - cur.hh * per;
      run_start(cur);
      return cur;
    };
    auto cursor_next = [&](Cursor& cur) {
      if (cur.run_left > 1) {
        --cur.run_left;
        ++cur.seq;
        cur.row0 += BMQ;
        cur.tile += src_tile_step;
        cur.stat += BMQ;
      } else if (cur.seq + 1 < seq_hi) {
        ++cur.seq;
        cur.r += cur.run_len;
        if (cur.r == (cur.unmasked ? nu : nm)) {
          cur.r = 0;
          ++cur.hh;
          if (cur.hh == a.group) { cur.hh = 0; cur.unmasked = true; }
        }
        run_start(cur);
      }
    };
    struct CopyJob { const bf16_t* src; unsigned dst; uint32_t row_bytes; int rows; const float* stat_src; uint32_t stat_off; unsigned stat_dst; };
    // the tile at the cursor into ring slot `slot`
    auto make_copy = [&](const Cursor& cc, int slot) {
      CopyJob j;
      j.src = cc.tile;
      j.row_bytes = src_row_bytes;
      j.dst = smem_lds + (copies_q ? L::Q_BASE : L::DO_BASE) + slot * TILE_BYTES;
      j.rows = a.s_q - cc.row0;
      // lanes 0..31: lse2 of rows row0 .. row0+31, lanes 32..63: delta of the same rows (clamped to the slice)
      const int t2 = fresh(tid), ql2 = t2 & 31, g2 = (t2 >> 5) & 1;
      const int rr = ql2 < j.rows ? ql2 : j.rows - 1;
      j.stat_src = cc.stat;
      j.stat_off = (g2 ? stat_off_delta : stat_off_lse2) + (uint32_t)rr * 4u;
      j.stat_dst = smem_lds + L::STAT_BASE + slot * L::STAT_BYTES;
      return j;
    };
    auto copy_pass = [&](const CopyJob& j, int n) { dma.issue(j.dst, j.src, j.row_bytes, j.rows, gwave_u, n); };
    // every wave of group A writes the same 64 statistics (no branch in the phase: identical data)
    auto copy_part = [&](const CopyJob& j, bool with_stats, int part) {
      if (part < PASSES) copy_pass(j, part);
      if (part == 3 && with_stats) dma4(j.stat_src, j.stat_off, j.stat_dst);
    };
    auto copy_all = [&](const CopyJob& j, bool with_stats) {
      for (int part = 0; part < 4; ++part) copy_part(j, with_stats, part);
    };

    // prologue: V rows of the workgroup (all threads), Q(0), Q(1) + statistics (group A), dO(0), dO(1) (group B)
    {
      TileDma<D, BNK, T> dma_v;
      dma_v.init(tid);
      const bf16_t* vbase = a.kv.v[kchunk] + head_off + chunk_row0 * a.kv_stride_s;
      const int64_t avail = a.kv_end - tile_key0;
      for (int n = 0; n < TileDma<D, BNK, T>::PASSES; ++n)
        dma_v.issue(smem_lds + L::V_BASE, vbase, (uint32_t)a.kv_stride_s * 2, avail > BNK ? BNK : (int)avail, wave_u, n);
    }
    Cursor cc = cursor_begin();          // copy cursor: two tiles ahead of the tile being worked on
    // first rows of the tile of the vector phase and of the one after it (the masks need them)
    int row0_cur = cc.row0;
    copy_all(make_copy(cc, 0), copies_q);
    cursor_next(cc);
    int row0_nxt = cc.row0;
    copy_all(make_copy(cc, 1), copies_q);
    cursor_next(cc);
    wait_async();
    TrBase<D> lo_qt;         // Q(u-1), transposed
    RpBase<D> lo_q, lo_v;    // Q(u) and this wave's V rows, row-packed
    lo_qt.init(lane, (int)smem_lds + L::Q_BASE + (SLOTS - 1) * TILE_BYTES);     // "Q(-1)": never read
    lo_q.init(lane, (int)smem_lds + L::Q_BASE);
    lo_v.init(lane, (int)smem_lds + L::V_BASE + wave_u * 32 * D * 2);
    __syncthreads();

    int slot = 0;            // ring slot of tile u
    auto advance = [&]() {
      lo_q.add(slot == SLOTS - 1 ? -(SLOTS - 1) * TILE_BYTES : TILE_BYTES);
      lo_qt.add(slot == 0 ? -(SLOTS - 1) * TILE_BYTES : TILE_BYTES);      // Q(u-1) sits in slot - 1
      slot = (slot == SLOTS - 1) ? 0 : slot + 1;
    };
    // this lane's half of the lse2 of the tile in ring slot `sl`
    auto stat_of = [&](int sl) {
      return reinterpret_cast<const float*>(smem + L::STAT_BASE + sl * L::STAT_BYTES) + 4 * ((fresh(tid) >> 5) & 1);
    };
    // vector phase of tile u (ring slot vslot, first row row0), with the copies of job j riding along
    auto vector_phase = [&](int u, int vslot, int row0, const CopyJob& j) {
      const bool need_mask = seq_lo + u < total_m;
      int rmin_rel = 0, rmax_rel = 32;
      if (need_mask) {
        // first row of the tile that sees this lane's key (worked out here, in the rare masked tiles,
        // rather than kept in a register across the loop)
        const int64_t rl = a.causal ? tile_key0 + wave_u * 32 + (fresh(tid) & 31) - a.q_offset - row0 : 0;
        rmin_rel = rl < 0 ? 0 : (rl > 32 ? 32 : (int)rl);
        const int left = a.s_q - row0;
        rmax_rel = left > 32 ? 32 : left;
      }
      const float* stat = reinterpret_cast<const float*>(smem + L::STAT_BASE + vslot * L::STAT_BYTES);
      dkdv_vector_phase<D>(st, stat, c, need_mask, rmin_rel, rmax_rel, (fresh(tid) >> 5) & 1, [&](int part) { copy_part(j, copies_q, part); });
    };
    // Both groups run the same code; group B starts one phase (one barrier) later and group A idles
    // one phase at the end.
    if (group_b) phase_end();
    { DkdvMatrixPhase<D, NW, false, true, 2> ph{lo_qt, lo_q, lo_v, st, stat_of(0)}; ph.run(); }     // scores of tile 0
    advance();
    wait_async();
    phase_end();
    // (a fresh live range for K right in front of the loop: if the register allocator had to park part of
    // it in scratch memory during the prologue, it comes back here and not inside the loop)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(st.kreg[ks]));
    int vslot = 0, cslot = 2;            // ring slots of the tile of the vector phase and of the tile being copied
    for (int u = 0; u + 1 < cnt; ++u) {
      const int row0_new = cc.row0;
      vector_phase(u, vslot, row0_cur, make_copy(cc, cslot));      // tile u+2 rides along
      cursor_next(cc);
      row0_cur = row0_nxt;
      row0_nxt = row0_new;
      vslot = (vslot + 1) & (SLOTS - 1);
      cslot = (cslot + 1) & (SLOTS - 1);
      phase_end();
      // (V never moves: without this the eight offsets of its head_dim blocks are kept in registers across the loop)
      asm volatile("" : "+v"(lo_v.off0));
      { DkdvMatrixPhase<D, NW, true, true, 2> ph{lo_qt, lo_q, lo_v, st, stat_of(vslot)}; ph.run(); }    // sums of tile u, scores of tile u+1
      advance();
      wait_async();                                      // the copies of the vector phase before have landed
      phase_end();
    }
    vector_phase(cnt - 1, vslot, row0_cur, make_copy(cc, cslot));   // (copies the last tile once more)
    phase_end();
    { DkdvMatrixPhase<D, NW, true, false, 2> ph{lo_qt, lo_q, lo_v, st, nullptr}; ph.run(); }     // sums of the last tile
    wait_async();
    phase_end();
    if (!group_b) phase_end();
  }

  // (the key is worked out afresh from an opaque copy of the lane number: otherwise its 64 bits stay in
  // registers across the whole loop, and registers are what this kernel is short of)
  const int tid_out = fresh(tid), ql_out = tid_out & 31, g_out = (tid_out >> 5) & 1;
  const int64_t mykey_out = tile_key0 + wave_u * 32 + ql_out;
  if (mykey_out >= a.kv_begin && mykey_out < a.kv_end) {
    // one chunk: straight into the accumulators; several: this chunk's partial sums, added up in a
    // fixed order by the reduce kernel
    float* kdst;
    float* vdst;
    bool accumulate;
    if (a.n_split > 1) {
      const int64_t plane = (int64_t)a.dkdv_items[2] * a.dkdv_items[1] * a.nkeys_pad * D;          // one of dk / dv of one chunk
      const int64_t row = (((int64_t)b * a.dkdv_items[1] + hk) * a.nkeys_pad + (mykey_out - grid0)) * D;
      kdst = a.part + (int64_t)split * 2 * plane + row;
      vdst = kdst + plane;
      accumulate = false;
    } else {
      const int64_t base = head_off + (chunk_row0 + (mykey_out - tile_key0)) * a.kv_stride_s;
      kdst = a.dk_acc[kchunk] + base;
      vdst = a.dv_acc[kchunk] + base;
      accumulate = a.dkv_accumulate != 0;
    }
    // One gradient at a time.  When the call adds to the accumulators, all 16 loads of the old values are issued
    // before the first of them is needed: a load, add, store chain per 16 bytes pays the memory latency 16 times over
    // (a store may alias a later load for all the compiler knows, so it does not batch them by itself), and with few
    // query tiles per key tile (many KV heads, short slices) that was a sixth of the kernel's time.
    auto flush = [&](const f32x16 (&acc)[DB], float* dst, float factor) {
      f32x4 old[DB * 4];
      if (accumulate) {
#pragma unroll
        for (int j = 0; j < DB * 4; ++j) old[j] = *reinterpret_cast<const f32x4*>(dst + 32 * (j >> 2) + 8 * (j & 3) + 4 * g_out);
      }
#pragma unroll
      for (int j = 0; j < DB * 4; ++j) {
        const int db = j >> 2, i4 = j & 3;
        f32x4 x4 = {acc[db][4 * i4] * factor, acc[db][4 * i4 + 1] * factor, acc[db][4 * i4 + 2] * factor, acc[db][4 * i4 + 3] * factor};
        if (accumulate) x4 += old[j];
        *reinterpret_cast<f32x4*>(dst + 32 * db + 8 * i4 + 4 * g_out) = x4;
      }
    };
    flush(st.dk, kdst, a.scale);
    flush(st.dv, vdst, 1.0f);
  }
}

// Without ticket counters the workgroup's index is its one item.  With them (set to zero before the launch), the
// launch has one workgroup per compute unit and each takes items until none is left: a compute unit (or XCD) that runs
// faster does more of them, and an item costs no workgroup dispatch (with one query head per KV head an item is 60 to
// 120 us of work).  There is one counter per XCD: the items with index = c (mod 8) form class c, the workgroups of
// XCD c take class c in order first and move on to the next class when theirs is used up.  Items of one class are the
// same chunk of the query stream (8 or 4 chunks) for one key tile after the other, so the workgroups that share an
// L2 walk the same eighth of Q and dO.  A workgroup leaves after it has found all eight classes empty.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dkdv_kernel(const BwdArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int n_items = a.dkdv_items[0] * a.dkdv_items[1] * a.dkdv_items[2];
  int cls = (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7u);      // XCC_ID
  int empty = 0;                                            // classes found empty so far
  for (;;) {                                                // (one copy of the item's code for both ways of getting an item)
    int item = blockIdx.x;
    if (a.ticket_dkdv) {
      int* slot = reinterpret_cast<int*>(smem);            // the item goes through the first bytes of the tile rings
      __syncthreads();                                      // every wave is done with the rings of the item before
      if (threadIdx.x == 0) {
        int it = -1;
        while (empty < 8) {
          const unsigned t = atomicAdd(a.ticket_dkdv + cls, 1u);
          if ((int64_t)t * 8 + cls < n_items) { it = (int)t * 8 + cls; break; }
          cls = (cls + 1) & 7;
          ++empty;
        }
        *slot = it;
      }
      __syncthreads();
      item = *slot;
      __syncthreads();                                      // read by all before the first tile copy lands there
      if (item < 0) return;
    }
    dkdv_item<D, NW>(a, item, smem);
    if (!a.ticket_dkdv) return;
  }
}

// dk_acc, dv_acc (+)= the partial sums of the chunks, chunk 0 first.
__global__ __launch_bounds__(256) void dkdv_reduce_kernel(const BwdArgs a, int batch, int head_dim) {
  const int64_t nkeys = a.kv_end - a.kv_begin;
  const int dvec = head_dim / 4;
  const int64_t total = (int64_t)batch * a.n_kv_heads * nkeys * dvec;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= total) return;
  const int d = (int)(gid % dvec) * 4;
  const int64_t key = (gid / dvec) % nkeys;
  const int64_t bh = gid / dvec / nkeys;
  const int hk = (int)(bh % a.n_kv_heads), b = (int)(bh / a.n_kv_heads);
  const int64_t plane = (int64_t)batch * a.n_kv_heads * a.nkeys_pad * head_dim;
  const int64_t grid0 = kv_grid_origin(a.kv_begin, a.kv.n, dkdv_keys_per_workgroup());
  const float* src = a.part + (bh * a.nkeys_pad + (a.kv_begin - grid0) + key) * head_dim + d;
  f32x4 k4 = *reinterpret_cast<const f32x4*>(src);
  f32x4 v4 = *reinterpret_cast<const f32x4*>(src + plane);
  for (int s = 1; s < a.n_split; ++s) {
    k4 += *reinterpret_cast<const f32x4*>(src + (int64_t)s * 2 * plane);
    v4 += *reinterpret_cast<const f32x4*>(src + (int64_t)s * 2 * plane + plane);
  }
  const int64_t kabs = a.kv_begin + key;
  const int chunk = a.kv.n > 1 ? (int)(kabs / a.kv.len) : 0;
  const int64_t base = (int64_t)b * a.kv_stride_b + (kabs - (int64_t)chunk * a.kv.len) * a.kv_stride_s + (int64_t)hk * a.kv_stride_h + d;
  f32x4* kd = reinterpret_cast<f32x4*>(a.dk_acc[chunk] + base);
  f32x4* vd = reinterpret_cast<f32x4*>(a.dv_acc[chunk] + base);
  if (a.dkv_accumulate) { k4 += *kd; v4 += *vd; }
  *kd = k4;
  *vd = v4;
}

// dq (+)= the partial dq of the key ranges, range 0 first; four head_dim elements per thread.
__global__ __launch_bounds__(256) void dq_reduce_kernel(const BwdArgs a, int batch, int head_dim) {
  const int dvec = head_dim / 4;
  const int64_t total = (int64_t)batch * a.s_q * a.n_q_heads * dvec;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= total) return;
  const int d = (int)(gid % dvec) * 4;
  const int64_t rh = gid / dvec;                     // (b * s_q + row) * heads + h
  const int h = (int)(rh % a.n_q_heads);
  const int64_t brow = rh / a.n_q_heads;
  const int64_t b = brow / a.s_q, row = brow % a.s_q;
  const float* src = static_cast<const float*>(a.dq) + b * a.dq_stride_b + row * a.dq_stride_s + (int64_t)h * a.dq_stride_h + d;
  f32x4 v4 = *reinterpret_cast<const f32x4*>(src);
  for (int r = 1; r < a.n_dq_ranges; ++r) v4 += *reinterpret_cast<const f32x4*>(src + (int64_t)r * a.dq_range_stride);
  const int64_t base = b * a.q_stride_b + row * a.q_stride_s + (int64_t)h * a.q_stride_h + d;
  if (a.dq_final_f32) {
    f32x4* dst = reinterpret_cast<f32x4*>(static_cast<float*>(a.dq_final) + base);
    if (a.dq_final_accumulate) v4 += *dst;
    *dst = v4;
  } else {
    *reinterpret_cast<bf16x4*>(static_cast<bf16_t*>(a.dq_final) + base) = __builtin_convertvector(v4, bf16x4);
  }
}

template <int D, int NW>
static hipError_t launch_dkdv_t(const BwdArgs& a, int batch, hipStream_t st) {
  if (a.kv_end <= a.kv_begin) return hipSuccess;
  const int64_t items = (int64_t)a.dkdv_items[0] * a.dkdv_items[1] * a.dkdv_items[2];
  // with a ticket counter: one workgroup per compute unit (the kernel's LDS allows one at a time), each looping over items
  const int64_t wgs = a.ticket_dkdv ? (items < a.dkdv_wgs ? items : a.dkdv_wgs) : items;
  dim3 grid((unsigned)wgs), block(NW * 64);
  constexpr size_t smem = DkdvLds<D, NW>::TOTAL;
  hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, NW>), grid, block, smem, st, a);
  return hipGetLastError();
}

hipError_t opt_in_bwd_kernels() {
  const hipFuncAttribute attr = hipFuncAttributeMaxDynamicSharedMemorySize;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dq_kernel<128, 8, kDqKeysPerTile>), attr, (int)dq_lds_bytes<128>());
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dq_kernel<64, 8, kDqKeysPerTile>), attr, (int)dq_lds_bytes<64>());
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dkdv_kernel<128, 8>), attr, DkdvLds<128, 8>::TOTAL);
  if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dkdv_kernel<64, 8>), attr, DkdvLds<64, 8>::TOTAL);
  return e;
}

hipError_t launch_bwd_dkdv(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  if (head_dim == 128) return launch_dkdv_t<128, 8>(a, batch, st);
  return launch_dkdv_t<64, 8>(a, batch, st);
}

hipError_t launch_dq_reduce(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  if (a.n_dq_ranges <= 1) return hipSuccess;
  const int64_t total = (int64_t)batch * a.s_q * a.n_q_heads * (head_dim / 4);
  hipLaunchKernelGGL(dq_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, batch, head_dim);
  return hipGetLastError();
}

hipError_t launch_dkdv_reduce(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  const int64_t nkeys = a.kv_end - a.kv_begin;
  if (nkeys <= 0 || a.n_split <= 1) return hipSuccess;
  const int64_t total = (int64_t)batch * a.n_kv_heads * nkeys * (head_dim / 4);
  hipLaunchKernelGGL(dkdv_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, batch, head_dim);
  return hipGetLastError();
}



}  // namespace slimpipe
