// Whole optimizer step of one small block (m, n <= 128) in a single workgroup.
//
// For blocks this small the step is bound by HBM traffic and launch count, not
// by the matrix cores: run stage by stage, the gradient block is read four
// times, the intermediate Lbar G makes a round trip through HBM, and a bucket
// costs eight launches.  Here one workgroup of 256 threads keeps the gradient
// block in LDS (66 KB of the 160 KB per CU; two workgroups per CU) and runs,
// on a step without root refresh (Sec. 3 complete pseudocode, default
// heuristics):
//   A <- A + G.^2,  s_g = ||G / (sqrt(A) + eps_g)||_F^2                       (Sec. 2.4)
//   L <- beta L + alpha G G^T,  R <- beta R + alpha G^T G                    (Sec. 3.1.1)
//   T = Lbar G (kept in LDS, over G),  P_sh = T Rbar,  s_sh = ||P_sh||_F^2   (Sec. 2.3)
//   P = -sqrt(s_g / s_sh) P_sh [- wd W],  M <- mu M + P,  W <- W + lr M      (Sec. 2.4, 3.1.2, 3.1.3)
// Every tensor is read once and written once.  The matrix products run on
// v_mfma_f32_32x32x2_f32; each wavefront owns a 64 x 64 quadrant as in the
// large-block GEMM, and the factor sums are flushed into float64 registers
// every 16 values of k exactly as there, so both paths give the same factors.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "elementwise.h"
#include "gemm_mfma.h"

namespace shampoo {

constexpr int SB = 128;            // largest block edge handled here
constexpr int SB_LD = SB + 1;      // odd leading dimension: a column walk (32 rows) hits 32 banks
constexpr int SB_SLAB = 16;        // rows of Lbar / Rbar staged per pass
constexpr int SB_XLD = SB + 4;
constexpr int SB_THREADS = 256;

// One block handled by the kernel: where it sits in the caller's tensors and where its state
// sits in the workspace (byte offsets).  Blocks of all small buckets share one launch.
struct SmallBlock {
  BlockDesc d;
  int32_t m, n;
  int64_t off_L, off_R, off_Linv, off_Rinv;   // m x m, n x n float32
  int64_t off_P;                              // m x n: Lbar G Rbar, kept for inspection
  int64_t off_norms;                          // 2 floats
};

struct SmallStepArgs {
  const SmallBlock *blocks;      // one per workgroup, largest first
  unsigned char *ws;
  void *const *w_table;
  const void *const *g_table;
  float *a_state, *m_state;      // m_state nullptr when mu == 0
  double alpha_d, beta_d;        // factor update weights
  float graft_eps, mu, lr, wd_decoupled;
  float a_decay, a_gain, a_bc;   // grafting state A <- a_decay A + a_gain G.^2, root of a_bc A
  int32_t nesterov;
};

// rows [k0, k0 + 16) of a dense dim x dim matrix into Xs[kk][0..128), zero padded
__device__ __forceinline__ void sb_fetch_slab(const float *mat, int dim, int k0, bool vec, int tid, float r[2][4]) {
  const int kk = tid >> 4, c4 = (tid & 15) * 4;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int c = c4 + 64 * h, k = k0 + kk;
    if (vec && k < dim && c + 3 < dim) {
      Elem<float>::load4(mat + (int64_t)k * dim + c, r[h]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) r[h][e] = (k < dim && c + e < dim) ? mat[(int64_t)k * dim + c + e] : 0.f;
    }
  }
}
__device__ __forceinline__ void sb_store_slab(float (*Xs)[SB_XLD], int tid, const float r[2][4]) {
  const int kk = tid >> 4, c4 = (tid & 15) * 4;
#pragma unroll
  for (int h = 0; h < 2; ++h)
    *reinterpret_cast<float4 *>(&Xs[kk][c4 + 64 * h]) = make_float4(r[h][0], r[h][1], r[h][2], r[h][3]);
}

// fixed-order sum over the workgroup; every thread gets the result
__device__ __forceinline__ float sb_reduce(float v, float *red, int tid) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

#define SB_ZERO_ACC()                                         \
  _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)            \
  _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_)            \
  _Pragma("unroll") for (int v_ = 0; v_ < 16; ++v_) acc[i_][j_][v_] = 0.f;

#define SB_MFMA4(a0, a1, b0, b1)                                                   \
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);    \
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);    \
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);    \
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);


// The factor update F <- beta F + alpha S (S = G G^T: WHICH = 0, dim = m, K = n; S = G^T G:
// WHICH = 1, dim = n, K = m) is done per wavefront in two halves of 32 rows x 64 columns.  The
// old values of a half are requested from HBM before the products of the previous half are
// formed, so the read-modify-write latency overlaps the matrix-core work.  float32 MFMA sums
// are added into float64 registers every 16 values of k.
__device__ __forceinline__ void sb_half_prefetch(const float *F, int dim, double beta_d, int row0, int col0,
                                                 int l32, int khalf, float old[32]) {
#pragma unroll
  for (int ni = 0; ni < 2; ++ni)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = row0 + 8 * (v >> 2) + 4 * khalf + (v & 3), j = col0 + ni * 32 + l32;
      old[ni * 16 + v] = (beta_d != 0.0 && i < dim && j < dim) ? F[(int64_t)i * dim + j] : 0.f;
    }
}

template <int WHICH>
__device__ __forceinline__ void sb_half_products(const float *Gs, int K, int row0, int col0, int l32, int khalf,
                                                 double acc64[2][16]) {
  floatx16 acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc[j][v] = 0.f; acc64[j][v] = 0.0; }
  const int Kp = (K + 15) & ~15;
  for (int k0 = 0; k0 < Kp; k0 += 16) {
#pragma unroll
    for (int kk = 0; kk < 16; kk += 2) {
      const int k = k0 + kk + khalf;
      float a, b0, b1;
      if (WHICH == 0) {      // A(i,k) = G[i][k], B(k,j) = G[j][k]
        a = Gs[(row0 + l32) * SB_LD + k];
        b0 = Gs[(col0 + l32) * SB_LD + k]; b1 = Gs[(col0 + 32 + l32) * SB_LD + k];
      } else {               // A(i,k) = G[k][i], B(k,j) = G[k][j]
        a = Gs[k * SB_LD + row0 + l32];
        b0 = Gs[k * SB_LD + col0 + l32]; b1 = Gs[k * SB_LD + col0 + 32 + l32];
      }
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[1], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) { acc64[j][v] += (double)acc[j][v]; acc[j][v] = 0.f; }
  }
}

__device__ __forceinline__ void sb_half_store(float *F, int dim, double alpha_d, double beta_d, int row0, int col0,
                                              int l32, int khalf, const double acc64[2][16], const float old[32]) {
#pragma unroll
  for (int ni = 0; ni < 2; ++ni)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = row0 + 8 * (v >> 2) + 4 * khalf + (v & 3), j = col0 + ni * 32 + l32;
      if (i < dim && j < dim)
        F[(int64_t)i * dim + j] = (float)(alpha_d * acc64[ni][v] + beta_d * (double)old[ni * 16 + v]);
    }
}

// GT: element type of the caller's gradients.  grid: one workgroup per entry of g.blocks.
template <typename GT>
__global__ __launch_bounds__(SB_THREADS, 2) void block_step_small_kernel(const SmallStepArgs g) {
  __shared__ float Gs[SB * SB_LD];                       // G, later T = Lbar G; zero outside m x n
  __shared__ __align__(16) float Xs[SB_SLAB][SB_XLD];    // slab of Lbar / Rbar rows
  __shared__ float red[4];

  const int slot = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, l32 = lane & 31, khalf = lane >> 5;
  const SmallBlock sbk = g.blocks[slot];
  const int m = sbk.m, n = sbk.n;
  const BlockDesc d = sbk.d;
  float *norms = reinterpret_cast<float *>(g.ws + sbk.off_norms);
  const GT *gp = reinterpret_cast<const GT *>(g.g_table[d.param]) + d.offset;
  float *wp = reinterpret_cast<float *>(g.w_table[d.param]) + d.offset;
  float *ap = g.a_state + d.state_offset;
  float *mp = g.m_state ? g.m_state + d.state_offset : nullptr;
  const int ld = d.ld;

  // ---- G -> LDS, grafting state and graft norm on the way (each element once)
  {
    const bool vec = ((ld & 3) == 0) && ((n & 3) == 0) && ((d.offset & 3) == 0) && ((d.state_offset & 3) == 0) &&
                     ((reinterpret_cast<uintptr_t>(g.g_table[d.param]) & 15) == 0);
    float ss = 0.f;
    // 16 float4 of G and of A per thread: every load is issued before the first store, so the
    // whole tile costs one memory round trip
    {
      float gv[16][4], av[16][4];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int idx = tid + SB_THREADS * u;
        const int i = idx >> 5, j = (idx & 31) * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) { gv[u][e] = 0.f; av[u][e] = 0.f; }
        if (i < m && j < n) {
          const int valid = min(4, n - j);
          load_g4<GT>(gp + (int64_t)i * ld + j, vec, valid, gv[u]);
          load_f4(ap + (int64_t)i * ld + j, vec, valid, av[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int idx = tid + SB_THREADS * u;
        const int i = idx >> 5, j = (idx & 31) * 4;
        if (i < m && j < n) {
          const int valid = min(4, n - j);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            av[u][e] = g.a_decay * av[u][e] + g.a_gain * (gv[u][e] * gv[u][e]);
            const float pg = gv[u][e] / (sqrtf(g.a_bc * av[u][e]) + g.graft_eps);
            if (e < valid) ss += pg * pg;
          }
          store_f4(ap + (int64_t)i * ld + j, vec, valid, av[u]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) Gs[i * SB_LD + j + e] = gv[u][e];
      }
    }
    ss = sb_reduce(ss, red, tid);      // also orders the LDS writes before the reads below
    if (tid == 0) norms[0] = ss;
    // (ss = s_g stays in a register of every thread until the update)
    // ---- factor updates (Gs is read-only here, no barriers needed)
    {
      float *Lp = reinterpret_cast<float *>(g.ws + sbk.off_L), *Rp = reinterpret_cast<float *>(g.ws + sbk.off_R);
      const int r0 = wm * 64, c0 = wn * 64;
      // wave-uniform: which 32-row halves of this wavefront's quadrant hold part of a factor
      const bool l0 = r0 < m && c0 < m, l1 = r0 + 32 < m && c0 < m;
      const bool q0 = r0 < n && c0 < n, q1 = r0 + 32 < n && c0 < n;
      float oldA[32], oldB[32];
      double acc64[2][16];
      if (l0) sb_half_prefetch(Lp, m, g.beta_d, r0, c0, l32, khalf, oldA);
      if (l0) sb_half_products<0>(Gs, n, r0, c0, l32, khalf, acc64);
      if (l1) sb_half_prefetch(Lp, m, g.beta_d, r0 + 32, c0, l32, khalf, oldB);
      if (l0) sb_half_store(Lp, m, g.alpha_d, g.beta_d, r0, c0, l32, khalf, acc64, oldA);
      if (l1) sb_half_products<0>(Gs, n, r0 + 32, c0, l32, khalf, acc64);
      if (q0) sb_half_prefetch(Rp, n, g.beta_d, r0, c0, l32, khalf, oldA);
      if (l1) sb_half_store(Lp, m, g.alpha_d, g.beta_d, r0 + 32, c0, l32, khalf, acc64, oldB);
      if (q0) sb_half_products<1>(Gs, m, r0, c0, l32, khalf, acc64);
      if (q1) sb_half_prefetch(Rp, n, g.beta_d, r0 + 32, c0, l32, khalf, oldB);
      if (q0) sb_half_store(Rp, n, g.alpha_d, g.beta_d, r0, c0, l32, khalf, acc64, oldA);
      if (q1) sb_half_products<1>(Gs, m, r0 + 32, c0, l32, khalf, acc64);
      if (q1) sb_half_store(Rp, n, g.alpha_d, g.beta_d, r0 + 32, c0, l32, khalf, acc64, oldB);
    }

    floatx16 acc[2][2];
    const bool active = wm * 64 < m && wn * 64 < n;    // wave-uniform: this quadrant holds part of the block
    // ---- T = Lbar G: Lbar rows through Xs (symmetric: A(i,k) = Lbar[k][i]), B(k,j) = G[k][j]
    float r[2][4];
    float wv[4][16], mv[4][16];
    {
      const float *Li = reinterpret_cast<const float *>(g.ws + sbk.off_Linv);
      const bool vecL = (m & 3) == 0;
      SB_ZERO_ACC();
      sb_fetch_slab(Li, m, 0, vecL, tid, r);
      sb_store_slab(Xs, tid, r);
      __syncthreads();
      for (int k0 = 0; k0 < m; k0 += SB_SLAB) {
        const bool more = k0 + SB_SLAB < m;
        if (more) sb_fetch_slab(Li, m, k0 + SB_SLAB, vecL, tid, r);
        if (active)
#pragma unroll
        for (int kk = 0; kk < SB_SLAB; kk += 2) {
          const int k = kk + khalf;
          const float a0 = Xs[k][wm * 64 + l32], a1 = Xs[k][wm * 64 + 32 + l32];
          const float b0 = Gs[(k0 + k) * SB_LD + wn * 64 + l32], b1 = Gs[(k0 + k) * SB_LD + wn * 64 + 32 + l32];
          SB_MFMA4(a0, a1, b0, b1);
        }
        __syncthreads();
        if (more) sb_store_slab(Xs, tid, r);
        __syncthreads();
      }
      // every wave has finished reading G: overwrite it with T (zero outside m x n by construction)
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              Gs[(wm * 64 + mi * 32 + 8 * q + 4 * khalf + e) * SB_LD + wn * 64 + ni * 32 + l32] = acc[mi][ni][4 * q + e];
    }
    // ---- P_sh = T Rbar: A(i,k) = T[i][k] from LDS, B(k,j) = Rbar[k][j] through Xs
    {
      const float *Ri = reinterpret_cast<const float *>(g.ws + sbk.off_Rinv);
      const bool vecR = (n & 3) == 0;
      SB_ZERO_ACC();
      // W and M of this wavefront's quadrant are requested now and used after the products
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = wm * 64 + (t >> 1) * 32 + 8 * (v >> 2) + 4 * khalf + (v & 3), j = wn * 64 + (t & 1) * 32 + l32;
          const bool in = i < m && j < n;
          wv[t][v] = in ? wp[(int64_t)i * ld + j] : 0.f;
          mv[t][v] = (in && mp) ? mp[(int64_t)i * ld + j] : 0.f;
        }
      sb_fetch_slab(Ri, n, 0, vecR, tid, r);
      sb_store_slab(Xs, tid, r);
      __syncthreads();                 // T and the first slab are in place
      for (int k0 = 0; k0 < n; k0 += SB_SLAB) {
        const bool more = k0 + SB_SLAB < n;
        if (more) sb_fetch_slab(Ri, n, k0 + SB_SLAB, vecR, tid, r);
        if (active)
#pragma unroll
        for (int kk = 0; kk < SB_SLAB; kk += 2) {
          const int k = kk + khalf;
          const float a0 = Gs[(wm * 64 + l32) * SB_LD + k0 + k], a1 = Gs[(wm * 64 + 32 + l32) * SB_LD + k0 + k];
          const float b0 = Xs[k][wn * 64 + l32], b1 = Xs[k][wn * 64 + 32 + l32];
          SB_MFMA4(a0, a1, b0, b1);
        }
        __syncthreads();
        if (more) sb_store_slab(Xs, tid, r);
        __syncthreads();
      }
    }
    // ---- norms, scale, momentum and parameter update straight from the accumulators
    float sp = 0.f;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int j = wn * 64 + ni * 32 + l32;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = wm * 64 + mi * 32 + 8 * q + 4 * khalf + e;
            const float v = acc[mi][ni][4 * q + e];
            if (i < m && j < n) sp += v * v;
          }
      }
    sp = sb_reduce(sp, red, tid);
    if (tid == 0) norms[1] = sp;
    // zero (or non-finite) norms give a zero step for the block instead of NaN
    const bool ok = (ss > 0.f) && (sp > 0.f) && (ss <= 3.0e38f) && (sp <= 3.0e38f);
    const float sc = ok ? (float)(-sqrt((double)ss / (double)sp)) : 0.f;
    float *Pp = reinterpret_cast<float *>(g.ws + sbk.off_P);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int j = wn * 64 + ni * 32 + l32;
        const int t = mi * 2 + ni;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * khalf + (v & 3);
          if (i < m && j < n) {
            const float psh = acc[mi][ni][v];
            Pp[(int64_t)i * n + j] = psh;
            float pv = sc * psh;
            if (g.wd_decoupled != 0.f) pv -= g.wd_decoupled * wv[t][v];
            if (mp) {
              const float mnew = g.mu * mv[t][v] + pv;
              mp[(int64_t)i * ld + j] = mnew;
              pv = g.nesterov ? g.mu * mnew + pv : mnew;
            }
            wp[(int64_t)i * ld + j] = wv[t][v] + g.lr * pv;
          }
        }
      }
  }
}

#undef SB_ZERO_ACC
#undef SB_MFMA4

}  // namespace shampoo
