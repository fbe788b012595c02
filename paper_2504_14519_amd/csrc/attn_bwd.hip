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
#include <stdlib.h>

#include <type_traits>

#include "kernels.hpp"
#include "tile_common.hpp"

namespace slimpipe {

// ------------------------------------------------------------------------------------ delta
// delta[b,h,r] = sum_d dO[b,r,h,d] * O[b,r,h,d] and lse2 = lse * log2(e) (+inf for rows that saw no
// key, which makes every p of the row exp2(-inf) = 0).  One 16-byte chunk per lane, D/8 lanes per row.
template <int D>
__global__ __launch_bounds__(256) void attn_delta_kernel(const BwdArgs a, int batch) {
  constexpr int NC = D / 8;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
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
    a.delta[sidx] = acc;
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
  float lse2, delta;
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
  const char* smem;
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
      abuf[M % NBUF] = lds_tr<D>(smem, lo_kt, db, blk * 16 * D * 2);
    } else if constexpr (M < N) {
      constexpr int j = M - N_DQ, ks = j / (2 * KB), r = j % (2 * KB), kb = r / 2;
      if constexpr ((r & 1) == 0) {
        abuf[M % NBUF] = lds_rp<D>(smem, lo_k, ks, kb * 32 * D * 2);
      } else {
        abuf[M % NBUF] = lds_rp<D>(smem, lo_v, ks, kb * 32 * D * 2);
        if constexpr (kb == 0) dob[ks & 1] = lds_rp<D>(smem, lo_do, ks, 0);
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
      else st.dp[kb] = mfma32(abuf[M % NBUF], dob[ks & 1], ks == 0 ? zero : st.dp[kb]);
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
    prologue<0>();
    SP_FENCE();
    step<0>();
  }
};

template <int D, int BN, bool WITH_DQ, bool WITH_SCORES>
SP_DEV void dq_matrix_phase(const char* smem, const TrBase<D>& lo_kt, const RpBase<D>& lo_k, const RpBase<D>& lo_v,
                            const RpBase<D>& lo_do, DqState<D, BN>& st) {
  DqMatrixPhase<D, BN, WITH_DQ, WITH_SCORES, 2> ph{smem, lo_kt, lo_k, lo_v, lo_do, st};
  ph.run();
}

// dS^T = p (dP^T - delta) with p = exp2(c S^T - lse2) on visible pairs; `hook(i)`, i = 0..3, is called at
// four points spread over the phase (asynchronous tile copies ride there).
template <int D, int BN, class H>
SP_DEV void dq_vector_phase(DqState<D, BN>& st, float c, bool need_mask, int kmax_rel, int g, H&& hook) {
  constexpr int KB = BN / 32;
  if (need_mask) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key_rel = kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
        st.s[kb][i] = key_rel <= kmax_rel ? st.s[kb][i] : -INFINITY;     // exp2(-inf) = 0
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
        st.s[kb][i] = p * (st.dp[kb][i] - st.delta);
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
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);      // known uniform to the compiler
  const bool group_b = wave_u >= NW / 2;
  const int gtid = tid & (GT - 1);
  const int qblk = (int)gridDim.x - 1 - (int)blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z, hk = h / a.group;
  const int m0 = qblk * BM, wrow0 = m0 + wave_u * 32;
  const int myrow = wrow0 + ql;
  const int myrow_c = myrow < a.s_q ? myrow : a.s_q - 1;
  const int64_t qpos = a.q_offset + myrow;

  DqState<D, BN> st;
  {
    const bf16_t* qp = a.q + (int64_t)b * a.q_stride_b + (int64_t)myrow_c * a.q_stride_s + (int64_t)h * a.q_stride_h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) st.qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * g);
    const int64_t stat = ((int64_t)b * a.n_q_heads + h) * a.s_q + myrow_c;
    st.lse2 = a.lse2[stat];          // +inf for an empty row -> p = 0
    st.delta = a.delta[stat];
  }
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.dq[db][i] = 0.f;

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
    auto key0_of = [&](int t) { return lo + (int64_t)t * BN; };
    TileDma<D, BN, GT> dma;
    constexpr int PASSES = TileDma<D, BN, GT>::PASSES;
    static_assert(PASSES <= 4, "one copy instruction per hook of the vector phase");
    dma.init(gtid);
    const uint32_t row_bytes = (uint32_t)a.kv_stride_s * 2;
    struct CopyJob { const bf16_t* src; char* dst; int rows; };
    // tile t of K (slot t % KSLOTS) or V (slot t % VSLOTS); past the end the last tile is copied again
    auto make_copy = [&](bool is_k, int t) {
      const int64_t key0 = key0_of(t < nt ? t : nt - 1);
      const int64_t avail = a.kv_capacity - key0;
      CopyJob j;
      j.src = (is_k ? kbase : vbase) + key0 * a.kv_stride_s;
      j.dst = smem + (is_k ? K_BASE + (t % KSLOTS) * TILE_BYTES : V_BASE + (t % VSLOTS) * TILE_BYTES);
      j.rows = avail > BN ? BN : (int)avail;
      return j;
    };
    auto copy_pass = [&](const CopyJob& j, int n) { dma.issue(j.dst, j.src, row_bytes, j.rows, gtid, n); };
    auto copy_all = [&](const CopyJob& j) {
      for (int n = 0; n < PASSES; ++n) copy_pass(j, n);
    };
    auto vector_phase = [&](int u, const CopyJob& j) {
      const int64_t key0 = key0_of(u);
      const bool need_mask = (key0 + BN > a.kv_end) || (a.causal && key0 + BN - 1 > a.q_offset + wrow0);
      int64_t kmax = a.kv_end - 1;
      if (a.causal && qpos < kmax) kmax = qpos;
      kmax -= key0;
      const int kmax_rel = kmax < -1 ? -1 : (kmax > BN ? BN : (int)kmax);
      dq_vector_phase<D, BN>(st, c, need_mask, kmax_rel, g, [&](int part) { if (part < PASSES) copy_pass(j, part); });
    };

    // prologue: the dO rows of the block (all threads), K(0), K(1) (group A), V(0), V(1) (group B)
    {
      TileDma<D, BM, T> dma_do;
      dma_do.init(tid);
      const bf16_t* dobase = a.d_out + (int64_t)b * a.do_stride_b + (int64_t)m0 * a.do_stride_s + (int64_t)h * a.do_stride_h;
      for (int n = 0; n < TileDma<D, BM, T>::PASSES; ++n)
        dma_do.issue(smem + DO_BASE, dobase, (uint32_t)a.do_stride_s * 2, a.s_q - m0, tid, n);
    }
    if (!group_b) { copy_all(make_copy(true, 0)); copy_all(make_copy(true, 1)); }
    else { copy_all(make_copy(false, 0)); copy_all(make_copy(false, 1)); }
    wait_async();
    TrBase<D> lo_kt;         // K(u-1), transposed
    RpBase<D> lo_k, lo_v;    // K(u), V(u), row-packed
    lo_kt.init(lane, K_BASE + (KSLOTS - 1) * TILE_BYTES);      // "K(-1)": never read
    lo_k.init(lane, K_BASE);
    lo_v.init(lane, V_BASE);
    RpBase<D> lo_do;         // this wave's 32 rows of dO
    lo_do.init(lane, DO_BASE + wave * 32 * D * 2);
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
    const bool copies_k = !group_b;
#ifdef SLIMPIPE_TRACE
    long long tq_v = 0, tq_b1 = 0, tq_m = 0, tq_w = 0, tq_b2 = 0, tq_t0 = clock64(), tq_w0 = wall_clock64(), tq_last = clock64();
#define TQ_MARK(var) { long long _n = clock64(); var += _n - tq_last; tq_last = _n; }
#else
#define TQ_MARK(var)
#endif
    if (group_b) phase_end();
    dq_matrix_phase<D, BN, false, true>(smem, lo_kt, lo_k, lo_v, lo_do, st);       // scores of tile 0
    advance();
    wait_async();
    phase_end();
    TQ_MARK(tq_b2)
    for (int u = 0; u + 1 < nt; ++u) {
      vector_phase(u, make_copy(copies_k, u + 2));       // tile u+2 rides along
      TQ_MARK(tq_v)
      phase_end();
      TQ_MARK(tq_b1)
      dq_matrix_phase<D, BN, true, true>(smem, lo_kt, lo_k, lo_v, lo_do, st);      // dQ of tile u, scores of tile u+1
      advance();
      TQ_MARK(tq_m)
      wait_async();                                      // the copies of the vector phase before have landed
      TQ_MARK(tq_w)
      phase_end();
      TQ_MARK(tq_b2)
    }
    vector_phase(nt - 1, make_copy(copies_k, nt + 1));   // (clamped: copies the last tile once more)
    phase_end();
    dq_matrix_phase<D, BN, true, false>(smem, lo_kt, lo_k, lo_v, lo_do, st);       // dQ of the last tile
    wait_async();
    phase_end();
    if (!group_b) phase_end();
#ifdef SLIMPIPE_TRACE
    if (blockIdx.x == gridDim.x - 1 && blockIdx.y == 0 && blockIdx.z == 0 && tid == 0) {
      long long* dbg = reinterpret_cast<long long*>(a.lse2 + (int64_t)a.n_q_heads * a.s_q) + 8;   // behind the workspace proper
      dbg[0] = tq_v; dbg[1] = tq_b1; dbg[2] = tq_m; dbg[3] = tq_w; dbg[4] = tq_b2;
      dbg[5] = clock64() - tq_t0; dbg[6] = wall_clock64() - tq_w0; dbg[7] = nt;
    }
#endif
  }

  if (myrow < a.s_q) {
    const int64_t base = (int64_t)b * a.q_stride_b + (int64_t)myrow * a.q_stride_s + (int64_t)h * a.q_stride_h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 32 * db + 8 * i4 + 4 * g;
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

template <int D, int NW, int BN>
static hipError_t launch_dq_t(const BwdArgs& a, int batch, hipStream_t st) {
  constexpr int BM = NW * 32;
  const size_t smem = (size_t)6 * BN * D * 2 + (size_t)BM * D * 2;   // 4 K slots + 2 V slots + dO rows
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dq_kernel<D, NW, BN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid((a.s_q + BM - 1) / BM, a.n_q_heads, batch), block(NW * 64);
  hipLaunchKernelGGL((attn_bwd_dq_kernel<D, NW, BN>), grid, block, smem, st, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dq(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  if (head_dim == 128) return launch_dq_t<128, 8, 64>(a, batch, st);
  return launch_dq_t<64, 8, 64>(a, batch, st);
}

// ------------------------------------------------------------------------------------ dk / dv
// The dk/dv kernel treats the query rows it has to visit (all query tiles that can see its keys,
// for every head of the GQA group, in a fixed order) as ONE stream of 32-row blocks and runs a
// software pipeline over that stream.  For block j:
//   region X: score MFMAs of block j+1  ||  softmax of block j  ||  transposed operand reads of j
//   region Y: accumulate MFMAs of block j  ||  score operand reads of block j+2
// A wave issues in order, so the overlap has to be in the instruction stream itself; each region
// is one scheduling region and the group barriers ask for "1 MFMA, then a few VALU / LDS reads".
// Query tiles (BMQ rows of Q and dO) sit in a ring of three LDS buffers: while tile t is consumed,
// tile t+1 is already resident (its first block's scores are computed ahead) and tile t+2 is in
// flight, so one barrier per tile is enough.

// Operands of one 32-row query block for S = Q K^T and dP = dO V^T (row-packed reads).
template <int D>
struct ScoreOps { bf16x8 qa[D / 16], da[D / 16]; };

template <int D, int TILE_BYTES>
SP_DEV void dkdv_load_ops(const char* smem, const RpOffsets<D>& lo, int blk_off, ScoreOps<D>& o) {
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    o.qa[ks] = lds_rp<D>(smem, lo, ks, blk_off);
    o.da[ks] = lds_rp<D>(smem, lo, ks, TILE_BYTES + blk_off);
  }
}
template <int D>
SP_DEV void dkdv_scores(const ScoreOps<D>& o, const bf16x8 (&kreg)[D / 16], const bf16x8 (&vreg)[D / 16],
                        f32x16& s, f32x16& dp) {
#pragma unroll
  for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    s = mfma32(o.qa[ks], kreg[ks], s);
    dp = mfma32(o.da[ks], vreg[ks], dp);
  }
}

// p = exp2(c s - lse2) on visible pairs (in s), dS = p (dP - delta) (in dp).
template <bool MASK>
SP_DEV void dkdv_softmax(f32x16& s, f32x16& dp, const float* lse_t, const float* del_t, int qb, int g, float c,
                         int rmin_rel, int rmax_rel) {
  if (MASK) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = 8 * (i >> 2) + 4 * g + (i & 3);
      s[i] = ((r >= rmin_rel) & (r < rmax_rel)) ? s[i] : -INFINITY;      // exp2(-inf) = 0
    }
  }
#pragma unroll
  for (int i4 = 0; i4 < 4; ++i4) {
    const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_t + qb * 32 + 8 * i4 + 4 * g);
    const f32x4 d4 = *reinterpret_cast<const f32x4*>(del_t + qb * 32 + 8 * i4 + 4 * g);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = 4 * i4 + j;
      const float p = exp2_fast(__builtin_fmaf(s[i], c, -l4[j]));
      s[i] = p;
      dp[i] = p * (dp[i] - d4[j]);
    }
  }
}

// Transposed operands of one 16-row half block for dV^T += dO^T P and dK^T += Q^T dS.
template <int D>
struct AccOps { bf16x8 dot[D / 32], qt[D / 32]; };

template <int D, int TILE_BYTES>
SP_DEV void dkdv_load_acc(const char* smem, const TrOffsets<D>& lo, int half_off, AccOps<D>& o) {
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    o.dot[db] = lds_tr<D>(smem, lo, db, TILE_BYTES + half_off);
    o.qt[db] = lds_tr<D>(smem, lo, db, half_off);
  }
}
template <int D>
SP_DEV void dkdv_accumulate(const AccOps<D>& o, bf16x8 pb, bf16x8 dsb, f32x16 (&dk)[D / 32], f32x16 (&dv)[D / 32]) {
#pragma unroll
  for (int db = 0; db < D / 32; ++db) {
    dv[db] = mfma32(o.dot[db], pb, dv[db]);
    dk[db] = mfma32(o.qt[db], dsb, dk[db]);
  }
}

// The global->LDS traffic of the tile two steps ahead.  It is staged through registers (global
// loads early in a tile, LDS writes at its end): the compiler must assume that an asynchronous
// global->LDS copy aliases every later LDS read and would make the wave wait for it on the spot.
struct DkdvDma {
  const bf16_t* q;         // head base of Q
  const bf16_t* dout;      // head base of dO
  const float* lse2;       // head base of the row statistics
  const float* delta;
  int64_t q_stride_s, do_stride_s;
  int row0, row_last;      // first row of the tile, last valid row of the slice
  char* dst;               // LDS: Q tile, dO tile behind it
  float* dst_stats;        // LDS: lse2[BMQ], delta[BMQ]
};
template <int D, int BMQ, int T>
struct DkdvStage {
  static constexpr int NC = D / 8, PASSES = BMQ * NC / T, PARTS = 4;
  static constexpr int part_of(int n) { return PASSES >= PARTS ? n % PARTS : n * (PARTS / PASSES); }
  u32x4 q[PASSES], o[PASSES];
  float stat;
  // Part P of the global loads of one tile.  The L1 path moves 64 bytes per clock for the whole CU
  // and a wave stalls at issue while it is busy, so the parts are spread over the pipeline steps.
  template <int P>
  SP_DEV void load_part(const DkdvDma& j, int tid) {
#pragma unroll
    for (int n = 0; n < PASSES; ++n) {
      if (part_of(n) != P) continue;
      const int id = tid + n * T;
      const int r = id / NC, c = id % NC;
      int64_t gr = j.row0 + r;
      gr = gr < j.row_last ? gr : j.row_last;
      q[n] = *reinterpret_cast<const u32x4*>(j.q + gr * j.q_stride_s + c * 8);
      o[n] = *reinterpret_cast<const u32x4*>(j.dout + gr * j.do_stride_s + c * 8);
    }
    if (P == PARTS - 1 && tid < 2 * BMQ) {     // threads [0,BMQ): lse2 rows, [BMQ,2BMQ): delta rows
      int r = j.row0 + (tid & (BMQ - 1));
      r = r < j.row_last ? r : j.row_last;
      stat = (tid < BMQ ? j.lse2 : j.delta)[r];
    }
  }
  SP_DEV void load(const DkdvDma& j, int tid) {
    load_part<0>(j, tid); load_part<1>(j, tid); load_part<2>(j, tid); load_part<3>(j, tid);
  }
  SP_DEV void store(char* dst, float* dst_stats, int tid) const {
#pragma unroll
    for (int n = 0; n < PASSES; ++n) {
      const int id = tid + n * T;
      const int r = id / NC, c = id % NC;
      *reinterpret_cast<u32x4*>(dst + tile_off<D>(r, c)) = q[n];
      *reinterpret_cast<u32x4*>(dst + BMQ * D * 2 + tile_off<D>(r, c)) = o[n];
    }
    if (tid < 2 * BMQ) dst_stats[tid] = stat;
  }
};

// One pipeline step: consumes the scores (s, dp) of block (tile t, block qb), produces the scores of
// the following block into (s_n, dp_n) from `ops`, then refills `ops` with the block after that.
//   cur: tile t (transposed reads), nxt_blk_off: where block j+1 .. the refill reads from (row-packed,
//   through lo_rp which already points at the right tile).
template <int D, int BMQ, int T, bool MASK, int QB_IDX>
SP_DEV void dkdv_step(const char* smem, const TrOffsets<D>& lo_tr, const RpOffsets<D>& lo_rp, int refill_off,
                      DkdvStage<D, BMQ, T>& stage, const DkdvDma& dma, char* store_dst, float* store_stats, int tid,
                      const float* lse_t, const float* del_t, int g, float c, int rmin_tile, int rows_left,
                      const bf16x8 (&kreg)[D / 16], const bf16x8 (&vreg)[D / 16], ScoreOps<D>& ops,
                      f32x16& s, f32x16& dp, f32x16& s_n, f32x16& dp_n, f32x16 (&dk)[D / 32], f32x16 (&dv)[D / 32]) {
  constexpr int TILE_BYTES = BMQ * D * 2, BLK = 32 * D * 2, HALF = 16 * D * 2;
  constexpr int NM = 2 * (D / 16);
  AccOps<D> acc0, acc1;
  constexpr int qb = QB_IDX;
  SP_FENCE();
  // ---- region X
  if (QB_IDX == 1) { stage.template load_part<0>(dma, tid); stage.template load_part<1>(dma, tid); }
  dkdv_scores<D>(ops, kreg, vreg, s_n, dp_n);
  int rmin_rel = 0, rmax_rel = 32;
  if (MASK) {
    const int rmin = rmin_tile - qb * 32, left = rows_left - qb * 32;
    rmin_rel = rmin < 0 ? 0 : (rmin > 32 ? 32 : rmin);
    rmax_rel = left < 0 ? 0 : (left > 32 ? 32 : left);
  }
  dkdv_softmax<MASK>(s, dp, lse_t, del_t, qb, g, c, rmin_rel, rmax_rel);
  const bf16x8 pb0 = pack8(s, 0), pb1 = pack8(s, 8);
  const bf16x8 ds0 = pack8(dp, 0), ds1 = pack8(dp, 8);
  dkdv_load_acc<D, TILE_BYTES>(smem, lo_tr, qb * BLK, acc0);
  dkdv_load_acc<D, TILE_BYTES>(smem, lo_tr, qb * BLK + HALF, acc1);
#pragma unroll
  for (int i = 0; i < NM; ++i) {
    __builtin_amdgcn_sched_group_barrier(SP_SG_MFMA, 1, 0);
    __builtin_amdgcn_sched_group_barrier(SP_SG_VALU, 7, 0);
    __builtin_amdgcn_sched_group_barrier(SP_SG_DSRD, 3, 0);
  }
  SP_FENCE();
  // ---- region Y
  if (QB_IDX == 1) { stage.template load_part<2>(dma, tid); stage.template load_part<3>(dma, tid); }
  if (QB_IDX == 0) stage.store(store_dst, store_stats, tid);
  dkdv_accumulate<D>(acc0, pb0, ds0, dk, dv);
  dkdv_accumulate<D>(acc1, pb1, ds1, dk, dv);
  dkdv_load_ops<D, TILE_BYTES>(smem, lo_rp, refill_off, ops);
#pragma unroll
  for (int i = 0; i < NM; ++i) {
    __builtin_amdgcn_sched_group_barrier(SP_SG_MFMA, 1, 0);
    __builtin_amdgcn_sched_group_barrier(SP_SG_DSRD, 1, 0);
  }
  SP_FENCE();
}

template <int D, int NW, int BMQ>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dkdv_kernel(const BwdArgs a) {
  constexpr int BNK = NW * 32, KS = D / 16, DB = D / 32, T = NW * 64;
  constexpr int TILE_BYTES = BMQ * D * 2, BLK = 32 * D * 2;
  constexpr int BUF_BYTES = 2 * TILE_BYTES;                    // Q tile, dO tile
  constexpr int NBUF = 3;
  static_assert(BMQ == 64, "the pipeline below is written for two 32-row blocks per tile");
  static_assert(2 * BMQ <= T, "one thread per staged row statistic");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* stats = reinterpret_cast<float*>(smem + NBUF * BUF_BYTES);   // [NBUF][lse2[BMQ], delta[BMQ]]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int hk = blockIdx.y, b = blockIdx.z;
  const int64_t tile_key0 = a.kv_begin + (int64_t)blockIdx.x * BNK;
  const int64_t wkey0 = tile_key0 + wave * 32;
  const int64_t mykey = wkey0 + ql;
  const int64_t mykey_c = mykey < a.kv_end ? mykey : a.kv_end - 1;

  // K, V as B operands: column = my key, k-slots = head_dim 16*ks + 8g ..
  bf16x8 kreg[KS], vreg[KS];
  {
    const int64_t off = (int64_t)b * a.kv_stride_b + mykey_c * a.kv_stride_s + (int64_t)hk * a.kv_stride_h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kreg[ks] = *reinterpret_cast<const bf16x8*>(a.k + off + 16 * ks + 8 * g);
      vreg[ks] = *reinterpret_cast<const bf16x8*>(a.v + off + 16 * ks + 8 * g);
    }
  }
  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dk[db][i] = 0.f; dv[db][i] = 0.f; }

  // Query tiles that can see this key tile: [qt0, nqt).  Tiles that need a mask (they straddle the
  // causal diagonal of this key tile, or hold rows past s_q) are walked first, for every head of the
  // group, then the unmasked rest; the order is fixed, so the sums are reproducible.
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
  // first row (absolute, within the slice) that sees this lane's key
  const int64_t rmin_abs = a.causal ? mykey - a.q_offset : 0;

  // sequence index -> (head of the group, query tile)
  auto locate = [&](int seq, int& hh, int& qt) {
    if (seq < total_m) {
      hh = seq / nm;
      const int r = seq % nm;
      qt = (r < qtm - qt0) ? qt0 + r : nqt - 1;
    } else {
      const int u = seq - total_m;
      hh = u / nu;
      qt = qtm + u % nu;
    }
  };

  auto make_dma = [&](int seq, int buf) {
    int hh, qt;
    locate(seq, hh, qt);
    const int h = hk * a.group + hh;
    DkdvDma j;
    j.q = a.q + (int64_t)b * a.q_stride_b + (int64_t)h * a.q_stride_h;
    j.dout = a.d_out + (int64_t)b * a.do_stride_b + (int64_t)h * a.do_stride_h;
    j.lse2 = a.lse2 + ((int64_t)b * a.n_q_heads + h) * a.s_q;
    j.delta = a.delta + ((int64_t)b * a.n_q_heads + h) * a.s_q;
    j.q_stride_s = a.q_stride_s;
    j.do_stride_s = a.do_stride_s;
    j.row0 = qt * BMQ;
    j.row_last = a.s_q - 1;
    j.dst = smem + buf * BUF_BYTES;
    j.dst_stats = stats + buf * 2 * BMQ;
    return j;
  };
  if (total > 0) {
    // ---- prologue: tiles 0 and 1 resident, scores of block 0 computed, operands of block 1 loaded
    DkdvStage<D, BMQ, T> stage;
    // tiles 0 and 1 go to LDS, tile 2 waits in the staging registers (tile indices past the end of
    // the stream are clamped: the last tile is fetched again and nobody reads it)
    for (int t = 0; t < 3; ++t) {
      const int tt = t < total ? t : total - 1;
      const DkdvDma j = make_dma(tt, t);
      stage.load(j, tid);
      if (t < 2) stage.store(smem + t * BUF_BYTES, stats + t * 2 * BMQ, tid);
    }
    __syncthreads();

    TrOffsets<D> lo_tr;      // tile being consumed
    RpOffsets<D> lo_rp;      // tile the score operands are read from
    lo_tr.init(lane, 0);
    lo_rp.init(lane, 0);
    ScoreOps<D> ops;
    f32x16 sA, dpA, sB, dpB;
    dkdv_load_ops<D, TILE_BYTES>(smem, lo_rp, 0, ops);
    dkdv_scores<D>(ops, kreg, vreg, sA, dpA);
    dkdv_load_ops<D, TILE_BYTES>(smem, lo_rp, BLK, ops);
    lo_rp.add(BUF_BYTES);    // from now on: one tile ahead of lo_tr

    int cur = 0;             // ring slot of the tile being consumed
#ifdef SLIMPIPE_TRACE
    long long tr_wait = 0, tr_issue = 0, tr_s0 = 0, tr_s1 = 0, tr_t0 = clock64(), tr_w0 = wall_clock64();
#define TR_MARK(var) { long long _n = clock64(); var += _n - tr_last; tr_last = _n; }
#else
#define TR_MARK(var)
#endif
    auto tile_body = [&](int seq, auto mask_tag) {
      constexpr bool MASK = decltype(mask_tag)::value;
#ifdef SLIMPIPE_TRACE
      long long tr_last = clock64();
#endif
      // tile seq+1 is written (it was stored one tile ago), every wave is done with tile seq-1
      if (seq > 0) __syncthreads();
      TR_MARK(tr_wait)
      // the tile two steps ahead goes into the slot tile seq-1 just left; past the end of the stream
      // the last tile is fetched again (nobody reads it) so that the steps stay branch-free
      const int free_slot = cur == 0 ? NBUF - 1 : cur - 1;
      // tile seq+2, loaded during the second step of tile seq-1, goes into the slot that tile just left
      // (written during the first step below); the loads of tile seq+3 are issued in the second step
      const DkdvDma dma = make_dma(seq + 3 < total ? seq + 3 : total - 1, 0);
      TR_MARK(tr_issue)
      const float* lse_t = stats + cur * 2 * BMQ;
      int rmin_tile = 0, rows_left = BMQ;
      if (MASK) {
        int hh, qt;
        locate(seq, hh, qt);
        const int row0 = qt * BMQ;
        const int64_t rl = rmin_abs - row0;
        rmin_tile = rl < 0 ? 0 : (rl > BMQ ? BMQ : (int)rl);
        rows_left = a.s_q - row0;
      }
      // block 0 of the tile: next scores = block 1 of this tile (ops already hold it);
      // refill ops with block 0 of the next tile
      dkdv_step<D, BMQ, T, MASK, 0>(smem, lo_tr, lo_rp, 0, stage, dma, smem + free_slot * BUF_BYTES, stats + free_slot * 2 * BMQ, tid, lse_t, lse_t + BMQ, g, c,
                                 rmin_tile, rows_left, kreg, vreg, ops, sA, dpA, sB, dpB, dk, dv);
      TR_MARK(tr_s0)
      // block 1: next scores = block 0 of the next tile; refill with block 1 of the next tile
      dkdv_step<D, BMQ, T, MASK, 1>(smem, lo_tr, lo_rp, BLK, stage, dma, smem + free_slot * BUF_BYTES, stats + free_slot * 2 * BMQ, tid, lse_t, lse_t + BMQ, g, c,
                                 rmin_tile, rows_left, kreg, vreg, ops, sB, dpB, sA, dpA, dk, dv);
      TR_MARK(tr_s1)
      // advance the ring
      const int step_tr = (cur == NBUF - 1) ? -(NBUF - 1) * BUF_BYTES : BUF_BYTES;
      const int step_rp = (cur == NBUF - 2) ? -(NBUF - 1) * BUF_BYTES : BUF_BYTES;
      lo_tr.add(step_tr);
      lo_rp.add(step_rp);
      cur = (cur == NBUF - 1) ? 0 : cur + 1;
    };

    int seq = 0;
    for (; seq < total_m; ++seq) tile_body(seq, std::true_type{});     // masked tiles
    for (; seq < total; ++seq) tile_body(seq, std::false_type{});      // unmasked tiles: the bulk
#ifdef SLIMPIPE_TRACE
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid == 0) {
      long long* dbg = reinterpret_cast<long long*>(a.lse2 + (int64_t)a.n_q_heads * a.s_q);   // behind the workspace proper
      dbg[0] = tr_wait; dbg[1] = tr_issue; dbg[2] = tr_s0; dbg[3] = tr_s1;
      dbg[4] = clock64() - tr_t0; dbg[5] = wall_clock64() - tr_w0; dbg[6] = total;
    }
#endif
  }

  if (mykey < a.kv_end) {
    const int64_t base = (int64_t)b * a.kv_stride_b + mykey * a.kv_stride_s + (int64_t)hk * a.kv_stride_h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 32 * db + 8 * i4 + 4 * g;
        f32x4 k4 = {dk[db][4 * i4] * a.scale, dk[db][4 * i4 + 1] * a.scale, dk[db][4 * i4 + 2] * a.scale,
                    dk[db][4 * i4 + 3] * a.scale};
        f32x4 v4 = {dv[db][4 * i4], dv[db][4 * i4 + 1], dv[db][4 * i4 + 2], dv[db][4 * i4 + 3]};
        f32x4* kd = reinterpret_cast<f32x4*>(a.dk_acc + base + d);
        f32x4* vd = reinterpret_cast<f32x4*>(a.dv_acc + base + d);
        if (a.dkv_accumulate) { k4 += *kd; v4 += *vd; }
        *kd = k4;
        *vd = v4;
      }
  }
}

template <int D, int NW, int BMQ>
static hipError_t launch_dkdv_t(const BwdArgs& a, int batch, hipStream_t st) {
  constexpr int BNK = NW * 32;
  const size_t smem = (size_t)3 * (2 * BMQ * D * 2) + 3 * 2 * BMQ * 4;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dkdv_kernel<D, NW, BMQ>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int64_t nkeys = a.kv_end - a.kv_begin;
  if (nkeys <= 0) return hipSuccess;
  dim3 grid((unsigned)((nkeys + BNK - 1) / BNK), a.n_kv_heads, batch), block(NW * 64);
  hipLaunchKernelGGL((attn_bwd_dkdv_kernel<D, NW, BMQ>), grid, block, smem, st, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dkdv(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  if (head_dim == 128) return launch_dkdv_t<128, 4, 64>(a, batch, st);
  return launch_dkdv_t<64, 4, 64>(a, batch, st);
}

}  // namespace slimpipe
