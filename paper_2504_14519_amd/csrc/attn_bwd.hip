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
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float p = exp2_fast(__builtin_fmaf(s[kb][i], c, -lse2));
          if (need_mask) {
            const int64_t key = key0 + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
            const bool vis = key < a.kv_end && (!a.causal || key <= qpos);
            p = vis ? p : 0.f;
          }
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
template <int D, int NW, int BMQ>
__global__ __launch_bounds__(NW * 64) void attn_bwd_dkdv_kernel(const BwdArgs a) {
  constexpr int BNK = NW * 32, KS = D / 16, DB = D / 32, QB = BMQ / 32, T = NW * 64;
  constexpr int TILE_BYTES = BMQ * D * 2;
  constexpr int BUF_BYTES = 2 * TILE_BYTES + 2 * BMQ * 4;      // Q tile, dO tile, lse2[BMQ], delta[BMQ]
  static_assert(BMQ <= T, "one thread per staged row statistic");
  extern __shared__ __attribute__((aligned(16))) char smem[];

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

  TileStage<D, BMQ, T> q_stage, do_stage;
  float st_lse = 0.f, st_delta = 0.f;

  auto issue = [&](int it) {
    const int hh = it / nq, qt = qt0 + it % nq;
    const int h = hk * a.group + hh;
    const bf16_t* qb = a.q + (int64_t)b * a.q_stride_b + (int64_t)h * a.q_stride_h;
    const bf16_t* ob = a.d_out + (int64_t)b * a.do_stride_b + (int64_t)h * a.do_stride_h;
    q_stage.issue(qb, a.q_stride_s, (int64_t)qt * BMQ, a.s_q - 1, tid);
    do_stage.issue(ob, a.do_stride_s, (int64_t)qt * BMQ, a.s_q - 1, tid);
    if (tid < BMQ) {
      int r = qt * BMQ + tid;
      r = r < a.s_q ? r : a.s_q - 1;
      const int64_t sidx = ((int64_t)b * a.n_q_heads + h) * a.s_q + r;
      const float l = a.lse[sidx];
      st_lse = (l == -INFINITY) ? INFINITY : l * kLog2e;
      st_delta = a.delta[sidx];
    }
  };
  auto commit = [&](int buf) {
    char* base = smem + buf * BUF_BYTES;
    q_stage.commit(base, tid);
    do_stage.commit(base + TILE_BYTES, tid);
    if (tid < BMQ) {
      reinterpret_cast<float*>(base + 2 * TILE_BYTES)[tid] = st_lse;
      reinterpret_cast<float*>(base + 2 * TILE_BYTES + BMQ * 4)[tid] = st_delta;
    }
  };

  if (total > 0) { issue(0); commit(0); }
  __syncthreads();

  for (int it = 0; it < total; ++it) {
    const int qt = qt0 + it % nq;
    const char* base = smem + (it & 1) * BUF_BYTES;
    const char* qtile = base;
    const char* dotile = base + TILE_BYTES;
    const float* lse_t = reinterpret_cast<const float*>(base + 2 * TILE_BYTES);
    const float* del_t = lse_t + BMQ;
    const bool more = (it + 1 < total);
    if (more) issue(it + 1);

#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int row0 = qt * BMQ + qb * 32;                     // first query row of this 32-block
      // rows all before this wave's first key see none of its keys; rows all >= s_q do not exist
      const bool skip = (a.causal && a.q_offset + row0 + 31 < wkey0) || row0 >= a.s_q;
      if (!skip) {
        f32x16 s, dp;
#pragma unroll
        for (int i = 0; i < 16; ++i) { s[i] = 0.f; dp[i] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 qa = lds_read_rowpacked<D>(qtile, qb * 32 + ql, ks, g);
          s = mfma32(qa, kreg[ks], s);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 da = lds_read_rowpacked<D>(dotile, qb * 32 + ql, ks, g);
          dp = mfma32(da, vreg[ks], dp);
        }
        const bool need_mask = (row0 + 32 > a.s_q) || (a.causal && wkey0 + 31 > a.q_offset + row0);
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_t + qb * 32 + 8 * i4 + 4 * g);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(del_t + qb * 32 + 8 * i4 + 4 * g);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int i = 4 * i4 + j;
            float p = exp2_fast(__builtin_fmaf(s[i], c, -l4[j]));
            if (need_mask) {
              const int row = row0 + 8 * i4 + 4 * g + j;
              const bool vis = row < a.s_q && (!a.causal || mykey <= a.q_offset + row);
              p = vis ? p : 0.f;
            }
            s[i] = p;
            dp[i] = p * (dp[i] - d4[j]);                      // dS
          }
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const bf16x8 pb = pack8(s, 8 * half);
          const bf16x8 dsb = pack8(dp, 8 * half);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 dot = lds_read_transposed<D>(dotile, qb * 32 + 16 * half, db, lane);
            dv[db] = mfma32(dot, pb, dv[db]);
            bf16x8 qt_ = lds_read_transposed<D>(qtile, qb * 32 + 16 * half, db, lane);
            dk[db] = mfma32(qt_, dsb, dk[db]);
          }
        }
      }
    }
    if (more) commit((it + 1) & 1);
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
  const size_t smem = (size_t)2 * (2 * BMQ * D * 2 + 2 * BMQ * 4);
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
