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

#include "kernels.hpp"
#include "tile_common.hpp"

namespace slimpipe {

// ------------------------------------------------------------------------------------ delta
// delta[b,h,r] = sum_d dO[b,r,h,d] * O[b,r,h,d].  One 16-byte chunk per lane, D/8 lanes per row.
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
  if (rh < total && c == 0) a.delta[((int64_t)b * a.n_q_heads + h) * a.s_q + r] = acc;
}

hipError_t launch_delta(const BwdArgs& a, int batch, int head_dim, hipStream_t st) {
  const int64_t lanes = (int64_t)batch * a.s_q * a.n_q_heads * (head_dim / 8);
  dim3 grid((unsigned)((lanes + 255) / 256)), block(256);
  if (head_dim == 128) hipLaunchKernelGGL(attn_delta_kernel<128>, grid, block, 0, st, a, batch);
  else hipLaunchKernelGGL(attn_delta_kernel<64>, grid, block, 0, st, a, batch);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------ dq
template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dq_kernel(const BwdArgs a) {
  constexpr int BM = NW * 32, KS = D / 16, DB = D / 32, KB = BN / 32, T = NW * 64;
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* k_tiles = smem;
  char* v_tiles = smem + 2 * TILE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int qblk = (int)gridDim.x - 1 - (int)blockIdx.x;
  const int h = blockIdx.y, b = blockIdx.z, hk = h / a.group;
  const int m0 = qblk * BM, wrow0 = m0 + wave * 32;
  const int myrow = wrow0 + ql;
  const int myrow_c = myrow < a.s_q ? myrow : a.s_q - 1;
  const int64_t qpos = a.q_offset + myrow;

  bf16x8 qreg[KS], doreg[KS];
  {
    const bf16_t* qp = a.q + (int64_t)b * a.q_stride_b + (int64_t)myrow_c * a.q_stride_s + (int64_t)h * a.q_stride_h;
    const bf16_t* dp = a.d_out + (int64_t)b * a.do_stride_b + (int64_t)myrow_c * a.do_stride_s + (int64_t)h * a.do_stride_h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * g);
      doreg[ks] = *reinterpret_cast<const bf16x8*>(dp + 16 * ks + 8 * g);
    }
  }
  const int64_t stat = ((int64_t)b * a.n_q_heads + h) * a.s_q + myrow_c;
  const float lse_raw = a.lse[stat];
  const float lse2 = (lse_raw == -INFINITY) ? INFINITY : lse_raw * kLog2e;   // empty row -> p = 0
  const float delta = a.delta[stat];

  const int64_t lo = a.kv_begin;
  int64_t hi = a.kv_end;
  if (a.causal) {
    const int last_row = (m0 + BM < a.s_q ? m0 + BM : a.s_q);
    const int64_t lim = a.q_offset + last_row;
    hi = hi < lim ? hi : lim;
  }
  const int nt = hi > lo ? (int)((hi - lo + BN - 1) / BN) : 0;
  const bf16_t* kbase = a.k + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
  const bf16_t* vbase = a.v + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;

  f32x16 dq[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;
  const float c = a.scale_log2e;

  TileStage<D, BN, T> ks_stage, vs_stage;
  if (nt > 0) {
    ks_stage.issue(kbase, a.kv_stride_s, lo, hi - 1, tid);
    vs_stage.issue(vbase, a.kv_stride_s, lo, hi - 1, tid);
    ks_stage.commit(k_tiles, tid);
    vs_stage.commit(v_tiles, tid);
  }
  __syncthreads();

  for (int t = 0; t < nt; ++t) {
    const int64_t key0 = lo + (int64_t)t * BN;
    const char* kt = k_tiles + (t & 1) * TILE_BYTES;
    const char* vt = v_tiles + (t & 1) * TILE_BYTES;
    const bool more = (t + 1 < nt);
    if (more) {
      ks_stage.issue(kbase, a.kv_stride_s, key0 + BN, hi - 1, tid);
      vs_stage.issue(vbase, a.kv_stride_s, key0 + BN, hi - 1, tid);
    }
    const bool skip = a.causal && key0 > a.q_offset + wrow0 + 31;
    if (!skip) {
      f32x16 s[KB], dp[KB];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { s[kb][i] = 0.f; dp[kb][i] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 ka = lds_read_rowpacked<D>(kt, kb * 32 + ql, ks, g);
          s[kb] = mfma32(ka, qreg[ks], s[kb]);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 va = lds_read_rowpacked<D>(vt, kb * 32 + ql, ks, g);
          dp[kb] = mfma32(va, doreg[ks], dp[kb]);
        }
      }
      const bool need_mask = (key0 + BN > a.kv_end) || (a.causal && key0 + BN - 1 > a.q_offset + wrow0);
      if (need_mask) {
        int64_t kmax = a.kv_end - 1;
        if (a.causal && qpos < kmax) kmax = qpos;
        kmax -= key0;
        const int kmax_rel = kmax < -1 ? -1 : (kmax > BN ? BN : (int)kmax);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key_rel = kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
            s[kb][i] = key_rel <= kmax_rel ? s[kb][i] : -INFINITY;     // exp2(-inf) = 0
          }
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = exp2_fast(__builtin_fmaf(s[kb][i], c, -lse2));
          s[kb][i] = p * (dp[kb][i] - delta);        // dS^T
        }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const bf16x8 dsb = pack8(s[kb], 8 * half);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 kta = lds_read_transposed<D>(kt, kb * 32 + 16 * half, db, lane);
            dq[db] = mfma32(kta, dsb, dq[db]);
          }
        }
    }
    if (more) {
      ks_stage.commit(k_tiles + ((t + 1) & 1) * TILE_BYTES, tid);
      vs_stage.commit(v_tiles + ((t + 1) & 1) * TILE_BYTES, tid);
    }
    __syncthreads();
  }

  if (myrow < a.s_q) {
    const int64_t base = (int64_t)b * a.q_stride_b + (int64_t)myrow * a.q_stride_s + (int64_t)h * a.q_stride_h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 32 * db + 8 * i4 + 4 * g;
        f32x4 v4 = {dq[db][4 * i4] * a.scale, dq[db][4 * i4 + 1] * a.scale, dq[db][4 * i4 + 2] * a.scale,
                    dq[db][4 * i4 + 3] * a.scale};
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
  const size_t smem = (size_t)4 * BN * D * 2;
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
// LDS map of the dk/dv kernel: two 2*TILE-byte buffers (Q tile, dO tile), each buffer a power of
// two in size so that switching buffers is one XOR on the lane offsets; row statistics behind them.

// One 32-row query block against the wave's 32 keys: S = Q K^T and dP = dO V^T (row-packed A
// operands from LDS, K/V B operands from registers).  `blk_off` = qb*32 rows in bytes.
template <int D, int TILE_BYTES>
SP_DEV void dkdv_scores(const char* smem, const LaneOffsets<D>& lo, int blk_off,
                        const bf16x8 (&kreg)[D / 16], const bf16x8 (&vreg)[D / 16], f32x16& s, f32x16& dp) {
  bf16x8 qa[D / 16], da[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    qa[ks] = lds_rp<D>(smem, lo, ks, blk_off);
    da[ks] = lds_rp<D>(smem, lo, ks, TILE_BYTES + blk_off);
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    s = mfma32(qa[ks], kreg[ks], s);
    dp = mfma32(da[ks], vreg[ks], dp);
  }
}

// p = exp2(c s - lse2) on visible pairs (in s), dS = p (dP - delta) (in dp).  `masked` is
// wave-uniform: only blocks on the causal diagonal or past the last row take the branch.
SP_DEV void dkdv_softmax(f32x16& s, f32x16& dp, const float* lse_t, const float* del_t, int qb, int g, float c,
                         bool masked, int rmin_rel, int rmax_rel) {
  if (masked) {
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

// dV^T += dO^T P, dK^T += Q^T dS for one 32-row block (transposed A operands from LDS).
template <int D, int TILE_BYTES>
SP_DEV void dkdv_accumulate(const char* smem, const LaneOffsets<D>& lo, int blk_off, const f32x16& p, const f32x16& ds,
                            f32x16 (&dk)[D / 32], f32x16 (&dv)[D / 32]) {
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const bf16x8 pb = pack8(p, 8 * half);
    const bf16x8 dsb = pack8(ds, 8 * half);
    bf16x8 dot[D / 32], qt[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      dot[db] = lds_tr<D>(smem, lo, db, TILE_BYTES + blk_off + half * 16 * D * 2);
      qt[db] = lds_tr<D>(smem, lo, db, blk_off + half * 16 * D * 2);
    }
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      dv[db] = mfma32(dot[db], pb, dv[db]);
      dk[db] = mfma32(qt[db], dsb, dk[db]);
    }
  }
}

// All QB blocks of one staged query tile, software pipelined: the score MFMAs of block qb+1 are
// issued before the softmax of block qb so the matrix pipe has work while the VALU runs.
// rmin_tile = first row of the tile (relative) that sees this lane's key; rows_left = valid rows;
// wave_rmin = the same for the wave's LAST key (wave-uniform): blocks starting at or after it need
// no causal mask.
template <int D, int BMQ>
SP_DEV void dkdv_tile(const char* smem, const LaneOffsets<D>& lo, const float* lse_t, const float* del_t, int lane,
                      const bf16x8 (&kreg)[D / 16], const bf16x8 (&vreg)[D / 16],
                      f32x16 (&dk)[D / 32], f32x16 (&dv)[D / 32], float c, int rmin_tile, int wave_rmin, int rows_left) {
  constexpr int QB = BMQ / 32, TILE_BYTES = BMQ * D * 2, BLK = 32 * D * 2;
  const int g = lane >> 5;
  f32x16 s_cur, dp_cur;
  dkdv_scores<D, TILE_BYTES>(smem, lo, 0, kreg, vreg, s_cur, dp_cur);
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    f32x16 s_nxt, dp_nxt;
    if (qb + 1 < QB) dkdv_scores<D, TILE_BYTES>(smem, lo, (qb + 1) * BLK, kreg, vreg, s_nxt, dp_nxt);
    const bool masked = (wave_rmin > qb * 32) || (rows_left < qb * 32 + 32);
    const int rmin = rmin_tile - qb * 32, left = rows_left - qb * 32;
    const int rmin_rel = rmin < 0 ? 0 : (rmin > 32 ? 32 : rmin);
    const int rmax_rel = left < 0 ? 0 : (left > 32 ? 32 : left);
    dkdv_softmax(s_cur, dp_cur, lse_t, del_t, qb, g, c, masked, rmin_rel, rmax_rel);
    dkdv_accumulate<D, TILE_BYTES>(smem, lo, qb * BLK, s_cur, dp_cur, dk, dv);
    if (qb + 1 < QB) { s_cur = s_nxt; dp_cur = dp_nxt; }
  }
}

template <int D, int NW, int BMQ>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dkdv_kernel(const BwdArgs a) {
  constexpr int BNK = NW * 32, KS = D / 16, DB = D / 32, T = NW * 64;
  constexpr int TILE_BYTES = BMQ * D * 2;
  constexpr int BUF_BYTES = 2 * TILE_BYTES;                    // Q tile, dO tile (power of two)
  static_assert((BUF_BYTES & (BUF_BYTES - 1)) == 0, "buffer toggle is an XOR");
  static_assert(BMQ <= T, "one thread per staged row statistic");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* stats = reinterpret_cast<float*>(smem + 2 * BUF_BYTES);   // [2 buffers][lse2[BMQ], delta[BMQ]]

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

  // query tiles that can see this key tile
  int qt0 = 0;
  if (a.causal && tile_key0 > a.q_offset) {
    const int64_t first = tile_key0 - a.q_offset;            // first row that sees tile_key0
    qt0 = first >= a.s_q ? (a.s_q + BMQ - 1) / BMQ : (int)(first / BMQ);
  }
  const int nqt = (a.s_q + BMQ - 1) / BMQ;
  const int nq = nqt > qt0 ? nqt - qt0 : 0;
  const int total = nq * a.group;
  const float c = a.scale_log2e;
  // first row (absolute, within the slice) that sees this lane's key
  const int64_t rmin_abs = a.causal ? mykey - a.q_offset : 0;
  const int64_t wave_rmin_abs = a.causal ? wkey0 + 31 - a.q_offset : 0;   // same for the wave's last key

  float st_lse = 0.f, st_delta = 0.f;
  auto issue = [&](int it, int buf) {
    const int hh = it / nq, qt = qt0 + it % nq;
    const int h = hk * a.group + hh;
    char* base = smem + buf * BUF_BYTES;
    const bf16_t* qb = a.q + (int64_t)b * a.q_stride_b + (int64_t)h * a.q_stride_h;
    const bf16_t* ob = a.d_out + (int64_t)b * a.do_stride_b + (int64_t)h * a.do_stride_h;
    tile_load_async<D, BMQ, T>(base, qb, a.q_stride_s, (int64_t)qt * BMQ, a.s_q - 1, tid);
    tile_load_async<D, BMQ, T>(base + TILE_BYTES, ob, a.do_stride_s, (int64_t)qt * BMQ, a.s_q - 1, tid);
    if (tid < BMQ) {
      int r = qt * BMQ + tid;
      r = r < a.s_q ? r : a.s_q - 1;
      const int64_t sidx = ((int64_t)b * a.n_q_heads + h) * a.s_q + r;
      const float l = a.lse[sidx];
      st_lse = (l == -INFINITY) ? INFINITY : l * kLog2e;
      st_delta = a.delta[sidx];
    }
  };
  auto commit_stats = [&](int buf) {
    if (tid < BMQ) {
      stats[buf * 2 * BMQ + tid] = st_lse;
      stats[buf * 2 * BMQ + BMQ + tid] = st_delta;
    }
  };

  LaneOffsets<D> lo;
  lo.init(lane, 0);

  if (total > 0) { issue(0, 0); commit_stats(0); }
  wait_async();
  __syncthreads();

  for (int it = 0; it < total; ++it) {
    const int qt = qt0 + it % nq;
    const float* lse_t = stats + (it & 1) * 2 * BMQ;
    const float* del_t = lse_t + BMQ;
    const bool more = (it + 1 < total);
    if (more) issue(it + 1, (it + 1) & 1);

    const int row0 = qt * BMQ;
    {
      // rows of this tile that see the lane's key / the wave's last key, clamped to [0, BMQ]
      const int64_t rl = rmin_abs - row0, rw = wave_rmin_abs - row0;
      const int rmin_tile = rl < 0 ? 0 : (rl > BMQ ? BMQ : (int)rl);
      const int wave_rmin = rw < 0 ? 0 : (rw > BMQ ? BMQ : (int)rw);
      dkdv_tile<D, BMQ>(smem, lo, lse_t, del_t, lane, kreg, vreg, dk, dv, c, rmin_tile, wave_rmin, a.s_q - row0);
    }
    lo.toggle(BUF_BYTES);

    if (more) commit_stats((it + 1) & 1);
    wait_async();
    __syncthreads();
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
  const size_t smem = (size_t)2 * (2 * BMQ * D * 2) + 2 * 2 * BMQ * 4;
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
  static const int variant = [] { const char* e = getenv("SLIMPIPE_DKDV_BMQ"); return e ? atoi(e) : 128; }();
  if (head_dim == 128) {
    if (variant == 64) return launch_dkdv_t<128, 4, 64>(a, batch, st);
    return launch_dkdv_t<128, 4, 128>(a, batch, st);
  }
  if (variant == 64) return launch_dkdv_t<64, 4, 64>(a, batch, st);
  return launch_dkdv_t<64, 4, 128>(a, batch, st);
}

}  // namespace slimpipe
