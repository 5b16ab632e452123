// Coalesced elementwise stages of the step (HBM-bandwidth bound):
//   prep_kernel       G1 = G + wd W (l2 weight decay), Gf <- beta1 Gf + (1-beta1) G1   (Sec. 3.1.1, 3.1.2)
//   graft_kernel      A <- A + G.^2 ; partial sums of ||Gf / (sqrt(A) + eps_g)||_F^2  (Sec. 2.4)
//   scale_kernel      per block: -||P_graft||_F / ||P_shampoo||_F from the partial sums
//   update_kernel     P = scale * P_shampoo (or -P_graft) ; M <- mu M + P ; W <- W + lr M (Sec. 3.1.3)
//   diag_kernel       1-D parameters: diagonal AdaGrad + momentum in one pass (Sec. 4.2.2)
// A block is addressed inside the caller's row-major tensors through its
// BlockDesc; rows of a block are contiguous runs, read as 4-element vectors
// when the block's origin and leading dimension allow it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"

namespace shampoo {

constexpr int EW_THREADS = 256;

struct EwGeom {        // how 256 threads tile a block of m x n
  int32_t lanes_x_log2;   // threads along columns = 1 << lanes_x_log2 (each owns 4 columns per pass)
  int32_t rows_per_wg;
  int32_t chunks;         // workgroups per block = ceil(m / rows_per_wg)
};

struct EwArgs {
  const BlockDesc *desc;
  void *const *w_table;          // parameter pointers (float32)
  const void *const *g_table;    // gradients that feed the grafting state (G, or G + wd W)
  const void *const *gd_table;   // gradients that feed the directions (filtered gradient if beta1 > 0)
  float *a_state;                // grafting state, parameter layout, all parameters concatenated
  float *m_state;                // momentum state, same layout (nullptr when mu == 0)
  const float *p;                // [slot][m][n] Shampoo directions
  float *sg_partial;             // [slot][chunks]
  float *gmax_partial;           // graft_kernel: [slot][chunks] max |G| of the chunk (nullptr: not wanted)
  const float *scale;            // [slot]
  int32_t m, n;
  EwGeom geom;
  float graft_eps, mu, lr;
  float gd_scale;                // direction gradients are multiplied by this (bias correction, 1 = off)
  // grafting state A <- a_decay A + a_gain G.^2 and P_graft = Gf / (sqrt(a_bc A) + eps):
  // (1, 1, 1) AdaGrad; (beta_g, 1 - beta_g, 1) RMSprop; Adam adds a_bc = 1 / (1 - beta_g^(t+1))
  float a_decay, a_gain, a_bc;
  float wd_decoupled;            // update_kernel: P <- P - wd_decoupled * W (0 = off)
  int32_t nesterov;              // update_kernel: step with mu M + P instead of M
  int32_t sgd_graft;             // P_graft = G (no grafting state) instead of AdaGrad
  int32_t same_src;              // g_table and gd_table are the same tensors
  int32_t graft_only;            // update_kernel: use -P_graft instead of scale * P
};

template <typename GT>
__device__ __forceinline__ void load_g4(const GT *g, bool vec, int valid, float v[4]) {
  if (vec) { Elem<GT>::load4(g, v); return; }
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = e < valid ? Elem<GT>::load1(g + e) : 0.f;
}
// 16 bytes that this step touches once: marked as streaming, so that they do not displace what
// the next kernel wants to find in the caches
typedef float ew_floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_load4(const float *p) {
  const ew_floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const ew_floatx4 *>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void nt_store4(float *p, const float4 &v) {
  const ew_floatx4 x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<ew_floatx4 *>(p));
}
__device__ __forceinline__ void load_f4(const float *p, bool vec, int valid, float v[4]) {
  if (vec) { Elem<float>::load4(p, v); return; }
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = e < valid ? p[e] : 0.f;
}
__device__ __forceinline__ void store_f4(float *p, bool vec, int valid, const float v[4]) {
  if (vec) { *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]); return; }
#pragma unroll
  for (int e = 0; e < 4; ++e) if (e < valid) p[e] = v[e];
}

// grid: chunks * (blocks of the bucket) workgroups, chunk index fastest.
// GS / GD: element types of the state-source and direction-source gradients.
template <typename GS, typename GD>
__global__ __launch_bounds__(EW_THREADS) void graft_kernel(const EwArgs g) {
  __shared__ float red[EW_THREADS / 64];
  const int slot = blockIdx.x / g.geom.chunks, chunk = blockIdx.x - slot * g.geom.chunks, tid = threadIdx.x;
  const BlockDesc d = g.desc[slot];
  const GS *gp = reinterpret_cast<const GS *>(g.g_table[d.param]) + d.offset;
  const GD *dp = reinterpret_cast<const GD *>(g.gd_table[d.param]) + d.offset;
  float *ap = g.a_state + d.state_offset;
  const int ld = d.ld, n = g.n;
  const bool vec = ((ld & 3) == 0) && ((n & 3) == 0) && ((d.offset & 3) == 0) && ((d.state_offset & 3) == 0) &&
                   ((reinterpret_cast<uintptr_t>(g.g_table[d.param]) & 15) == 0) &&
                   ((reinterpret_cast<uintptr_t>(g.gd_table[d.param]) & 15) == 0);
  const int lx = g.geom.lanes_x_log2;
  const int tx = tid & ((1 << lx) - 1), ty = tid >> lx, ny = EW_THREADS >> lx;
  const int r0 = chunk * g.geom.rows_per_wg;
  const int r1 = min(r0 + g.geom.rows_per_wg, g.m);
  float ss = 0.f, gmax = 0.f;
  if (vec && g.same_src && !g.sgd_graft) {
    // The common case, four column passes at a time, every load requested before the first store.
    constexpr int U = 4;
    const int step = 4 << lx;
    for (int i = r0 + ty; i < r1; i += ny)
      for (int j0 = tx * 4; j0 < n; j0 += U * step) {
        float gq[U][4];
        float4 av[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = j0 + u * step;
          if (j < n) {
            Elem<GD>::load4(dp + (int64_t)i * ld + j, gq[u]);
            av[u] = nt_load4(ap + (int64_t)i * ld + j);
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = j0 + u * step;
          if (j < n) {
            float a4[4] = {av[u].x, av[u].y, av[u].z, av[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float gv = gq[u][e];
              gmax = fmaxf(gmax, fabsf(gv));
              a4[e] = g.a_decay * a4[e] + g.a_gain * (gv * gv);
              const float pg = (gv * g.gd_scale) / (sqrtf(g.a_bc * a4[e]) + g.graft_eps);
              ss += pg * pg;
            }
            nt_store4(ap + (int64_t)i * ld + j, make_float4(a4[0], a4[1], a4[2], a4[3]));
          }
        }
      }
  } else
  for (int i = r0 + ty; i < r1; i += ny)
    for (int j = tx * 4; j < n; j += 4 << lx) {
      const int valid = min(4, n - j);
      float gv[4], dv[4], av[4];
      load_g4<GD>(dp + (int64_t)i * ld + j, vec, valid, dv);
      gmax = fmaxf(fmaxf(gmax, fmaxf(fabsf(dv[0]), fabsf(dv[1]))), fmaxf(fabsf(dv[2]), fabsf(dv[3])));
      if (g.same_src) {
#pragma unroll
        for (int e = 0; e < 4; ++e) gv[e] = dv[e];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) dv[e] *= g.gd_scale;
      if (g.sgd_graft) {
#pragma unroll
        for (int e = 0; e < 4; ++e) if (e < valid) ss += dv[e] * dv[e];
        continue;
      }
      if (!g.same_src) load_g4<GS>(gp + (int64_t)i * ld + j, vec, valid, gv);
      load_f4(ap + (int64_t)i * ld + j, vec, valid, av);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        av[e] = g.a_decay * av[e] + g.a_gain * (gv[e] * gv[e]);
        const float pg = dv[e] / (sqrtf(g.a_bc * av[e]) + g.graft_eps);
        if (e < valid) ss += pg * pg;
      }
      store_f4(ap + (int64_t)i * ld + j, vec, valid, av);
    }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  if (tid == 0) g.sg_partial[(int64_t)slot * g.geom.chunks + chunk] = (red[0] + red[1]) + (red[2] + red[3]);
  if (g.gmax_partial) {       // uniform
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) gmax = fmaxf(gmax, __shfl_xor(gmax, off, 64));
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = gmax;
    __syncthreads();
    if (tid == 0) g.gmax_partial[(int64_t)slot * g.geom.chunks + chunk] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  }
}

struct ScaleArgs {
  const float *sg_partial; int32_t sg_count;   // per block
  const float *ssh_partial; int32_t ssh_count; // per block
  float *scale;    // [blocks]
  float *norms;    // [blocks][2]
};

// One wavefront per block; fixed summation order, so results are reproducible.
__global__ __launch_bounds__(64) void scale_kernel(const ScaleArgs g) {
  const int b = blockIdx.x, lane = threadIdx.x;
  double sg = 0.0, ssh = 0.0;
  for (int i = lane; i < g.sg_count; i += 64) sg += (double)g.sg_partial[(int64_t)b * g.sg_count + i];
  for (int i = lane; i < g.ssh_count; i += 64) ssh += (double)g.ssh_partial[(int64_t)b * g.ssh_count + i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    sg += __shfl_xor(sg, off, 64);
    ssh += __shfl_xor(ssh, off, 64);
  }
  if (lane == 0) {
    // zero (or non-finite) norms give a zero step for the block instead of NaN
    const bool ok = (sg > 0.0) && (ssh > 0.0) && (sg <= 1.0e300) && (ssh <= 1.0e300);
    g.scale[b] = ok ? (float)(-sqrt(sg / ssh)) : 0.f;
    g.norms[2 * b] = (float)sg;
    g.norms[2 * b + 1] = (float)ssh;
  }
}

// GD: element type of the direction-source gradients (read only in the grafting-only phase).
template <typename GD>
__global__ __launch_bounds__(EW_THREADS) void update_kernel(const EwArgs g) {
  const int slot = blockIdx.x / g.geom.chunks, chunk = blockIdx.x - slot * g.geom.chunks, tid = threadIdx.x;
  const BlockDesc d = g.desc[slot];
  float *wp = reinterpret_cast<float *>(g.w_table[d.param]) + d.offset;
  const GD *gp = reinterpret_cast<const GD *>(g.gd_table[d.param]) + d.offset;
  float *ap = g.a_state + d.state_offset;
  float *mp = g.m_state ? g.m_state + d.state_offset : nullptr;
  const int ld = d.ld, n = g.n;
  const float *pp = g.p + (int64_t)slot * g.m * n;
  const bool vec = ((ld & 3) == 0) && ((n & 3) == 0) && ((d.offset & 3) == 0) && ((d.state_offset & 3) == 0) &&
                   ((reinterpret_cast<uintptr_t>(g.w_table[d.param]) & 15) == 0) &&
                   ((reinterpret_cast<uintptr_t>(g.gd_table[d.param]) & 15) == 0);
  const int lx = g.geom.lanes_x_log2;
  const int tx = tid & ((1 << lx) - 1), ty = tid >> lx, ny = EW_THREADS >> lx;
  const int r0 = chunk * g.geom.rows_per_wg;
  const int r1 = min(r0 + g.geom.rows_per_wg, g.m);
  const float sc = g.graft_only ? 0.f : g.scale[slot];
  if (vec && !g.graft_only && mp) {
    // The common case, four column passes at a time: all twelve 16-byte loads of a thread are
    // requested before the first store (a store between two loads would make the second one
    // wait: the compiler cannot tell that M, W and P do not overlap).
    constexpr int U = 4;
    const int step = 4 << lx;
    for (int i = r0 + ty; i < r1; i += ny)
      for (int j0 = tx * 4; j0 < n; j0 += U * step) {
        float4 pv[U], wv[U], mv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = j0 + u * step;
          if (j < n) {
            pv[u] = nt_load4(pp + (int64_t)i * n + j);
            wv[u] = nt_load4(wp + (int64_t)i * ld + j);
            mv[u] = nt_load4(mp + (int64_t)i * ld + j);
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = j0 + u * step;
          if (j < n) {
            float p4[4] = {pv[u].x * sc, pv[u].y * sc, pv[u].z * sc, pv[u].w * sc};
            float w4[4] = {wv[u].x, wv[u].y, wv[u].z, wv[u].w};
            float m4[4] = {mv[u].x, mv[u].y, mv[u].z, mv[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (g.wd_decoupled != 0.f) p4[e] -= g.wd_decoupled * w4[e];
              m4[e] = g.mu * m4[e] + p4[e];
              w4[e] += g.lr * (g.nesterov ? g.mu * m4[e] + p4[e] : m4[e]);
            }
            nt_store4(mp + (int64_t)i * ld + j, make_float4(m4[0], m4[1], m4[2], m4[3]));
            nt_store4(wp + (int64_t)i * ld + j, make_float4(w4[0], w4[1], w4[2], w4[3]));
          }
        }
      }
    return;
  }
  for (int i = r0 + ty; i < r1; i += ny)
    for (int j = tx * 4; j < n; j += 4 << lx) {
      const int valid = min(4, n - j);
      float pv[4], wv[4], mv[4];
      if (g.graft_only) {
        float gv[4], av[4];
        load_g4<GD>(gp + (int64_t)i * ld + j, vec, valid, gv);
#pragma unroll
        for (int e = 0; e < 4; ++e) gv[e] *= g.gd_scale;
        if (g.sgd_graft) {
#pragma unroll
          for (int e = 0; e < 4; ++e) pv[e] = -gv[e];
        } else {
          load_f4(ap + (int64_t)i * ld + j, vec, valid, av);
#pragma unroll
          for (int e = 0; e < 4; ++e) pv[e] = -gv[e] / (sqrtf(g.a_bc * av[e]) + g.graft_eps);
        }
      } else {
        load_f4(pp + (int64_t)i * n + j, vec, valid, pv);
#pragma unroll
        for (int e = 0; e < 4; ++e) pv[e] *= sc;
      }
      load_f4(wp + (int64_t)i * ld + j, vec, valid, wv);
      if (g.wd_decoupled != 0.f) {
#pragma unroll
        for (int e = 0; e < 4; ++e) pv[e] -= g.wd_decoupled * wv[e];
      }
      if (mp) {
        load_f4(mp + (int64_t)i * ld + j, vec, valid, mv);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          mv[e] = g.mu * mv[e] + pv[e];
          wv[e] += g.lr * (g.nesterov ? g.mu * mv[e] + pv[e] : mv[e]);
        }
        store_f4(mp + (int64_t)i * ld + j, vec, valid, mv);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) wv[e] += g.lr * pv[e];
      }
      store_f4(wp + (int64_t)i * ld + j, vec, valid, wv);
    }
}

// 1-D parameters, cut into chunks of at most DIAG_CHUNK elements.
constexpr int DIAG_CHUNK = 4096;
struct DiagChunk {
  int32_t param;
  int32_t len;
  int64_t start;         // first element inside the parameter
  int64_t state_offset;  // offset of that element in the A / M state arrays
};
struct DiagArgs {
  const DiagChunk *chunks;
  void *const *w_table;
  const void *const *g_table;
  float *a_state, *m_state, *gf_state;   // gf_state: filtered gradient (nullptr when beta1 == 0)
  float graft_eps, mu, lr;
  float beta1, wd_l2, wd_decoupled;
  float gd_scale;        // bias correction of the filtered gradient (1 = off)
  float a_decay, a_gain, a_bc;   // as in EwArgs
  int32_t nesterov;
};

template <typename GT>
__global__ __launch_bounds__(EW_THREADS) void diag_kernel(const DiagArgs g) {
  const DiagChunk c = g.chunks[blockIdx.x];
  float *w = reinterpret_cast<float *>(g.w_table[c.param]) + c.start;
  const GT *gp = reinterpret_cast<const GT *>(g.g_table[c.param]) + c.start;
  float *a = g.a_state + c.state_offset;
  float *m = g.m_state ? g.m_state + c.state_offset : nullptr;
  float *gf = g.gf_state ? g.gf_state + c.state_offset : nullptr;
  for (int i = threadIdx.x; i < c.len; i += EW_THREADS) {
    float wv = w[i];
    float gv = Elem<GT>::load1(gp + i);
    if (g.wd_l2 != 0.f) gv += g.wd_l2 * wv;
    const float av = g.a_decay * a[i] + g.a_gain * (gv * gv);
    a[i] = av;
    float dv = gv;
    if (gf) { dv = g.beta1 * gf[i] + (1.f - g.beta1) * gv; gf[i] = dv; }
    float p = -(g.gd_scale * dv) / (sqrtf(g.a_bc * av) + g.graft_eps);
    if (g.wd_decoupled != 0.f) p -= g.wd_decoupled * wv;
    if (m) {
      const float mv = g.mu * m[i] + p;
      m[i] = mv;
      p = g.nesterov ? g.mu * mv + p : mv;
    }
    w[i] = wv + g.lr * p;
  }
}

// 2-D parameters, flat chunks: G1 = G + wd W (if g1 != nullptr) and
// Gf <- beta1 Gf + (1 - beta1) G1 (if gf != nullptr); both in the A / M state layout.
struct PrepArgs {
  const DiagChunk *chunks;
  void *const *w_table;
  const void *const *g_table;
  float *g1, *gf;
  float wd_l2, beta1;
};

template <typename GT>
__global__ __launch_bounds__(EW_THREADS) void prep_kernel(const PrepArgs g) {
  const DiagChunk c = g.chunks[blockIdx.x];
  const float *w = reinterpret_cast<const float *>(g.w_table[c.param]) + c.start;
  const GT *gp = reinterpret_cast<const GT *>(g.g_table[c.param]) + c.start;
  for (int i = threadIdx.x; i < c.len; i += EW_THREADS) {
    float gv = Elem<GT>::load1(gp + i);
    if (g.g1) { gv += g.wd_l2 * w[i]; g.g1[c.state_offset + i] = gv; }
    if (g.gf) {
      const float f = g.beta1 * g.gf[c.state_offset + i] + (1.f - g.beta1) * gv;
      g.gf[c.state_offset + i] = f;
    }
  }
}

__global__ __launch_bounds__(256) void fill_kernel(float *p, float v, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// roots start as the identity: count matrices of n x n
__global__ __launch_bounds__(256) void eye_kernel(float *p, int32_t n, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int64_t e = i % ((int64_t)n * n);
  p[i] = (e / n == e % n) ? 1.f : 0.f;
}

}  // namespace shampoo
