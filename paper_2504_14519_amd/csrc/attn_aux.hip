// HBM-bound helpers of the hot path: the online-softmax merge of partial (out, lse) pairs
// (paper Sec. 4.2.2: a remotely computed partial output is folded into the local one; Sec. 5:
// the softmax normaliser travels with it) and the final rounding of fp32 gradient accumulators.
#include "kernels.hpp"
#include "tile_common.hpp"

namespace slimpipe {

// One thread per 8 consecutive head_dim elements of one (row, head).
//   lse = m + ln sum_r exp(lse_r - m),  out = sum_r exp(lse_r - lse) out_r ; parts with lse_r = -inf weigh 0.
__global__ __launch_bounds__(256) void attn_merge_kernel(const MergeArgs a) {
  const int nc = a.head_dim / 8;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t total = a.rows * a.n_q_heads * nc;
  if (gid >= total) return;
  const int c = (int)(gid % nc);
  const int64_t rh = gid / nc;                       // row * Hq + h
  const int h = (int)(rh % a.n_q_heads);
  const int64_t row = rh / a.n_q_heads;              // b * s_q + r
  const int64_t bq = row / a.s_q, r = row % a.s_q;
  const int64_t sidx = (bq * a.n_q_heads + h) * a.s_q + r;

  float m = -INFINITY;
  for (int p = 0; p < a.n_parts; ++p) m = fmaxf(m, a.lses[p][sidx]);
  const bool has = m != -INFINITY;
  float tot = 0.f;
  if (has)
    for (int p = 0; p < a.n_parts; ++p) tot += exp2_fast((a.lses[p][sidx] - m) * kLog2e);
  const float lse = has ? m + __builtin_log2f(tot) * kLn2 : -INFINITY;
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  const int64_t eoff = rh * a.head_dim + c * 8;
  if (has) {
    const float inv = 1.0f / tot;
    for (int p = 0; p < a.n_parts; ++p) {
      const float lp = a.lses[p][sidx];
      if (lp == -INFINITY) continue;          // weight 0: the part's out row is not read (it may be uninitialised)
      const float w = exp2_fast((lp - m) * kLog2e) * inv;
      if (a.part_f32) {
        const f32x4* src = reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(a.outs[p]) + eoff);
        const f32x4 x0 = src[0], x1 = src[1];
#pragma unroll
        for (int j = 0; j < 4; ++j) { acc[j] += w * x0[j]; acc[4 + j] += w * x1[j]; }
      } else {
        const bf16x8 x = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16_t*>(a.outs[p]) + eoff);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += w * (float)x[j];
      }
    }
  }
  const int64_t ooff = bq * a.o_stride_b + r * a.o_stride_s + (int64_t)h * a.o_stride_h + c * 8;
  if (a.out_f32) {
    f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(a.out) + ooff);
    dst[0] = f32x4{acc[0], acc[1], acc[2], acc[3]};
    dst[1] = f32x4{acc[4], acc[5], acc[6], acc[7]};
  } else {
    bf16x8 o;
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
      bf16x2 h2 = __builtin_convertvector(f32x2{acc[j], acc[j + 1]}, bf16x2);
      o[j] = h2[0];
      o[j + 1] = h2[1];
    }
    *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16_t*>(a.out) + ooff) = o;
  }
  if (c == 0) a.lse[sidx] = lse;
}

hipError_t launch_merge(const MergeArgs& a, hipStream_t st) {
  const int64_t total = a.rows * a.n_q_heads * (a.head_dim / 8);
  if (total <= 0) return hipSuccess;
  dim3 grid((unsigned)((total + 255) / 256)), block(256);
  hipLaunchKernelGGL(attn_merge_kernel, grid, block, 0, st, a);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void finalize_bf16_kernel(const float* __restrict__ acc, bf16_t* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += stride) {
    if (i + 4 <= n) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(acc + i);
      *reinterpret_cast<bf16x4*>(dst + i) = __builtin_convertvector(v, bf16x4);
    } else {
      for (int64_t j = i; j < n; ++j) dst[j] = (bf16_t)acc[j];
    }
  }
}

hipError_t launch_finalize(const float* acc, __bf16* dst, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n / 4 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(finalize_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, acc, dst, n);
  return hipGetLastError();
}

// ---- measurement aid: what the matrix pipe sustains on this chip, outside any attention kernel ----
// 8 waves per workgroup, every wave issues nothing but v_mfma_f32_32x32x16_bf16 on four accumulators.
// With `random` operands (every bf16 a different hashed value in [2^-8, 1) with random sign) the chip
// runs into its power limit and clocks down; with constant operands it does not: the two figures
// bracket what "peak" means for a kernel that multiplies real data.
__global__ __launch_bounds__(512) void mfma_rate_kernel(int random, int iters, float* sink) {
  const unsigned tid = threadIdx.x + 512u * blockIdx.x;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      unsigned ha = (tid * 64u + i * 16u + j) * 2654435761u, hb = (tid * 64u + i * 16u + 8u + j) * 2246822519u;
      ha ^= ha >> 15; hb ^= hb >> 13;
      // exponent 0x77..0x7e (2^-8 .. 2^-1), 7 random mantissa bits, random sign
      const unsigned short ba = random ? (unsigned short)(((0x77u + (ha & 7u)) << 7) | ((ha >> 8) & 0x7fu) | ((ha >> 16) & 0x8000u)) : 0x3f00;
      const unsigned short bb = random ? (unsigned short)(((0x77u + (hb & 7u)) << 7) | ((hb >> 8) & 0x7fu) | ((hb >> 16) & 0x8000u)) : 0x3f00;
      a[i][j] = __builtin_bit_cast(bf16_t, ba);
      b[i][j] = __builtin_bit_cast(bf16_t, bb);
    }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
    c0 = mfma32(a[0], b[0], c0);
    c1 = mfma32(a[1], b[1], c1);
    c2 = mfma32(a[2], b[2], c2);
    c3 = mfma32(a[3], b[3], c3);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) t += c0[i] + c1[i] + c2[i] + c3[i];
  if (t == 12345.678f) sink[0] = t;          // keeps the loop alive; practically never true
}

hipError_t launch_mfma_rate(int random, int iters, int workgroups, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(mfma_rate_kernel, dim3((unsigned)workgroups), dim3(512), 0, st, random, iters, sink);
  return hipGetLastError();
}

// ---- measurement aid: how evenly the eight XCDs of the chip run the same work ----
// Every workgroup issues the same number of matrix instructions (random operands) and records when it started and
// ended (constant-rate wall clock) and the XCD it ran on.  Workgroups are handed to the XCDs round-robin whatever
// their speed, so a launch of equal workgroups ends when the slowest XCD ends.
__global__ __launch_bounds__(512) void xcd_rate_kernel(int iters, long long* t_start, long long* t_end, unsigned* xcc) {
  const long long t0 = wall_clock64();
  const unsigned tid = threadIdx.x + 512u * blockIdx.x;
  bf16x8 a[2], b[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      unsigned ha = (tid * 64u + i * 16u + j) * 2654435761u, hb = (tid * 64u + i * 16u + 8u + j) * 2246822519u;
      ha ^= ha >> 15; hb ^= hb >> 13;
      a[i][j] = __builtin_bit_cast(bf16_t, (unsigned short)(((0x77u + (ha & 7u)) << 7) | ((ha >> 8) & 0x7fu) | ((ha >> 16) & 0x8000u)));
      b[i][j] = __builtin_bit_cast(bf16_t, (unsigned short)(((0x77u + (hb & 7u)) << 7) | ((hb >> 8) & 0x7fu) | ((hb >> 16) & 0x8000u)));
    }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
    c0 = mfma32(a[0], b[0], c0);
    c1 = mfma32(a[1], b[1], c1);
    c2 = mfma32(a[0], b[1], c2);
    c3 = mfma32(a[1], b[0], c3);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) t += c0[i] + c1[i] + c2[i] + c3[i];
  if (threadIdx.x == 0) {
    t_start[blockIdx.x] = t0;
    t_end[blockIdx.x] = wall_clock64() + (t == 12345.678f ? 1 : 0);      // (keeps the loop alive)
    xcc[blockIdx.x] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));   // XCC_ID, bits 3:0
  }
}

hipError_t launch_xcd_rate(int iters, int workgroups, long long* t_start, long long* t_end, unsigned* xcc, hipStream_t st) {
  hipLaunchKernelGGL(xcd_rate_kernel, dim3((unsigned)workgroups), dim3(512), 0, st, iters, t_start, t_end, xcc);
  return hipGetLastError();
}

// ---- measurement aid: what float32 atomic adds cost in the access pattern of a fused backward ----
// A backward kernel that computes S and dP once would be key-stationary (dK/dV stay in registers, summed in a
// fixed order) and would have to ADD its dQ contributions into memory: per step a workgroup of 8 waves owning
// 256 keys of one head holds a 32 x 128 (rows_per_step = 32: two partial sums over 128 keys each) or 64 x 128
// (rows_per_step = 64: one sum over 256 keys) block of dQ as eight 32 x 32 MFMA C tiles, lane = head_dim column,
// register = query row, so that one atomic instruction of a wave covers two full 128-byte lines.  This kernel
// issues exactly those atomic adds for `key_tiles` x `heads` workgroups that each walk every query tile of a
// slice of `s_q` rows, optionally with `filler_mfma` matrix instructions per wave and step standing in for the
// five GEMMs (40 per 32 rows), and nothing else.
//   placement 0: consecutive workgroups share a head (every XCD adds into every head's dQ)
//   placement 1: workgroup w works on head w % heads (with 8 heads and round-robin dispatch: one head per XCD)
//   rotate     : start tile of workgroup w shifted by w's key tile (spreads the workgroups over the rows)
__global__ __launch_bounds__(512) void dq_atomic_probe_kernel(float* dq, int s_q, int heads, int key_tiles, int rows_per_step,
                                                              int placement, int rotate, int filler_mfma, int with_atomics,
                                                              unsigned* xcc_mismatch) {
  const int w = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 5, col = lane & 31;
  const int h = placement ? w % heads : w / key_tiles;
  const int kt = placement ? w / heads : w % key_tiles;
  if (placement && threadIdx.x == 0) {
    // XCC_ID (hardware register 20, bits 3:0): which XCD this workgroup runs on
    const unsigned xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));
    if ((int)xcc != (w % 8)) atomicAdd(xcc_mismatch, 1u);
  }
  const int steps = s_q / rows_per_step;
  const int db = wave & 3, half = wave >> 2;
  const int row_in_step = rows_per_step == 64 ? 32 * half : 0;
  bf16x8 a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    unsigned ha = (threadIdx.x * 16u + j) * 2654435761u, hb = (threadIdx.x * 16u + 8u + j) * 2246822519u;
    a[j] = __builtin_bit_cast(bf16_t, (unsigned short)(((0x77u + (ha & 7u)) << 7) | ((ha >> 8) & 0x7fu) | ((ha >> 16) & 0x8000u)));
    b[j] = __builtin_bit_cast(bf16_t, (unsigned short)(((0x77u + (hb & 7u)) << 7) | ((hb >> 8) & 0x7fu) | ((hb >> 16) & 0x8000u)));
  }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  const int t0 = rotate ? (kt * 7) % steps : 0;
  for (int i = 0; i < steps; ++i) {
    int t = t0 + i;
    if (t >= steps) t -= steps;
    for (int m = 0; m < filler_mfma; m += 4) {
      c0 = mfma32(a, b, c0); c1 = mfma32(b, a, c1); c2 = mfma32(a, a, c2); c3 = mfma32(b, b, c3);
    }
    if (with_atomics) {
      float* base = dq + ((int64_t)(t * rows_per_step + row_in_step) * heads + h) * 128 + 32 * db + col;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + 4 * g + (r & 3);
        unsafeAtomicAdd(base + (int64_t)row * heads * 128, 1.0f);
      }
    }
  }
  float tsum = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) tsum += c0[i] + c1[i] + c2[i] + c3[i];
  if (tsum == 12345.678f) dq[0] = tsum;          // keeps the filler alive; practically never true
}

hipError_t launch_dq_atomic_probe(float* dq, int s_q, int heads, int key_tiles, int rows_per_step, int placement, int rotate,
                                  int filler_mfma, int with_atomics, unsigned* xcc_mismatch, hipStream_t st) {
  hipLaunchKernelGGL(dq_atomic_probe_kernel, dim3((unsigned)(key_tiles * heads)), dim3(512), 0, st, dq, s_q, heads, key_tiles,
                     rows_per_step, placement, rotate, filler_mfma, with_atomics, xcc_mismatch);
  return hipGetLastError();
}

}  // namespace slimpipe
