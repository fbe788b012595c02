// Forward of slice-wise causal attention over a key range (paper Sec. 4.1.2; partial ranges and
// the normaliser that travels with the output: Sec. 4.2.2, Sec. 5).
//
// One workgroup = NW wavefronts, each owning 32 query rows of one head.  The key range is walked
// in tiles of BN keys staged in LDS (double buffered).  Per tile and wave:
//   S^T = K Q^T        A = K rows from LDS (row-packed), B = Q held in registers
//   online softmax     the C layout gives every lane ONE query column, so the row max / row sum
//                      are in-lane reductions plus one exchange between the two half-waves
//   O^T += V^T P^T     A = V through the transposed LDS read, B = P straight from the C registers
// Scores and probabilities never leave registers.
#include "kernels.hpp"
#include "tile_common.hpp"

namespace slimpipe {

template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64) void attn_fwd_kernel(const FwdArgs a) {
  constexpr int BM = NW * 32, KS = D / 16, DB = D / 32, KB = BN / 32, T = NW * 64;
  constexpr int TILE_BYTES = BN * D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* k_tiles = smem;                       // 2 buffers
  char* v_tiles = smem + 2 * TILE_BYTES;      // 2 buffers

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, ql = lane & 31;
  const int qblk = (int)gridDim.x - 1 - (int)blockIdx.x;   // heaviest (latest) query block first
  const int h = blockIdx.y, b = blockIdx.z, hk = h / a.group;
  const int m0 = qblk * BM, wrow0 = m0 + wave * 32;
  const int myrow = wrow0 + ql;
  const int myrow_c = myrow < a.s_q ? myrow : a.s_q - 1;
  const int64_t qpos = a.q_offset + myrow;

  // Q as B operand: column = my query, k-slots = head_dim 16*ks + 8g ..
  bf16x8 qreg[KS];
  {
    const bf16_t* qp = a.q + (int64_t)b * a.q_stride_b + (int64_t)myrow_c * a.q_stride_s + (int64_t)h * a.q_stride_h;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks + 8 * g);
  }

  // keys this workgroup walks: [lo, hi)
  const int64_t lo = a.kv_begin;
  int64_t hi = a.kv_end;
  if (a.causal) {
    const int last_row = (m0 + BM < a.s_q ? m0 + BM : a.s_q);   // exclusive
    const int64_t lim = a.q_offset + last_row;
    hi = hi < lim ? hi : lim;
  }
  const int nt = hi > lo ? (int)((hi - lo + BN - 1) / BN) : 0;

  const bf16_t* kbase = a.k + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;
  const bf16_t* vbase = a.v + (int64_t)b * a.kv_stride_b + (int64_t)hk * a.kv_stride_h;

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  float m_run = -INFINITY;   // running max of score * c  (log2 domain)
  float l_run = 0.f;         // this lane's share of the running row sum
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

    // whole tile above this wave's causal frontier -> nothing visible
    const bool skip = a.causal && key0 > a.q_offset + wrow0 + 31;
    if (!skip) {
      f32x16 s[KB];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          bf16x8 ka = lds_read_rowpacked<D>(kt, kb * 32 + ql, ks, g);
          s[kb] = mfma32(ka, qreg[ks], s[kb]);
        }
      }
      const bool need_mask = (key0 + BN > a.kv_end) || (a.causal && key0 + BN - 1 > a.q_offset + wrow0);
      if (need_mask) {
        // last visible key of this lane's query, relative to the tile (may be < 0 or >= BN)
        int64_t kmax = a.kv_end - 1;
        if (a.causal && qpos < kmax) kmax = qpos;
        kmax -= key0;
        const int kmax_rel = kmax < -1 ? -1 : (kmax > BN ? BN : (int)kmax);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key_rel = kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
            s[kb][i] = key_rel <= kmax_rel ? s[kb][i] : -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
      mx = xhalf_max(mx);
      const float m_new = fmaxf(m_run, mx * c);
      const float m_eff = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = exp2_fast(m_run - m_eff);     // m_run = -inf -> 0
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = exp2_fast(__builtin_fmaf(s[kb][i], c, -m_eff));
          s[kb][i] = p;
          l_run += p;
        }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const bf16x8 pb = pack8(s[kb], 8 * half);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 va = lds_read_transposed<D>(vt, kb * 32 + 16 * half, db, lane);
            o[db] = mfma32(va, pb, o[db]);
          }
        }
    }
    if (more) {
      ks_stage.commit(k_tiles + ((t + 1) & 1) * TILE_BYTES, tid);
      vs_stage.commit(v_tiles + ((t + 1) & 1) * TILE_BYTES, tid);
    }
    __syncthreads();
  }

  // epilogue
  const float l_tot = xhalf_sum(l_run);
  const bool has = l_tot > 0.f;
  const float inv = has ? 1.0f / l_tot : 0.f;
  if (myrow < a.s_q) {
    if (g == 0) {
      const float lse = has ? (m_run + __builtin_log2f(l_tot)) * kLn2 : -INFINITY;
      a.lse[((int64_t)b * a.n_q_heads + h) * a.s_q + myrow] = lse;
    }
    const int64_t obase = (int64_t)b * a.o_stride_b + (int64_t)myrow * a.o_stride_s + (int64_t)h * a.o_stride_h;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int d = 32 * db + 8 * i4 + 4 * g;
        f32x4 v4 = {o[db][4 * i4] * inv, o[db][4 * i4 + 1] * inv, o[db][4 * i4 + 2] * inv, o[db][4 * i4 + 3] * inv};
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
static hipError_t launch_fwd_t(const FwdArgs& a, int batch, hipStream_t st) {
  constexpr int BM = NW * 32;
  const size_t smem = (size_t)4 * BN * D * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<D, NW, BN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid((a.s_q + BM - 1) / BM, a.n_q_heads, batch), block(NW * 64);
  hipLaunchKernelGGL((attn_fwd_kernel<D, NW, BN>), grid, block, smem, st, a);
  return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs& a, int batch, int head_dim, hipStream_t st) {
  if (head_dim == 128) return launch_fwd_t<128, 8, 64>(a, batch, st);
  return launch_fwd_t<64, 8, 64>(a, batch, st);
}

}  // namespace slimpipe
