// Diagonal Shampoo (Sec. 4.2.3 of the paper): a parameter with a dimension above the block
// size is kept whole and the Kronecker factor of every such dimension is replaced by its
// diagonal,
//   l_i <- beta2 l_i + (1 - beta2) sum_j G_ij^2      (= diag(G G^T))
//   r_j <- beta2 r_j + (1 - beta2) sum_i G_ij^2      (= diag(G^T G))
// whose root inverse is elementwise (the framed box of Sec. 3.2.1 applied to a diagonal
// matrix, whose eigenvalues are its entries).  A dimension within the block size keeps its
// full factor and goes through the SYRK / eigensolver / GEMM kernels; these kernels cover
// the diagonal sides: the two reductions, the elementwise root, and the row / column scaling
// that stands in for the matrix product.  All are single passes bound by HBM.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "elementwise.h"

namespace shampoo {

struct DiagFactorArgs {
  const BlockDesc *desc;
  const void *const *g_table;
  float *vec;            // [slot][m] (rows) or [slot][n] (columns)
  double a, b;           // vec <- a vec + b sums
  int32_t m, n;
  float *partial;        // columns only: [slot][segs][n]
  int32_t segs, rows_per_seg;
};

// Row sums of squares.  grid (ceil(m / 4), batch), 256 threads: one wavefront per row.
template <typename GS>
__global__ __launch_bounds__(256) void diag_row_kernel(const DiagFactorArgs g) {
  const int slot = blockIdx.y, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= g.m) return;
  const BlockDesc d = g.desc[slot];
  const GS *gp = reinterpret_cast<const GS *>(g.g_table[d.param]) + d.offset + (int64_t)i * d.ld;
  double ss = 0.0;
  for (int j = lane; j < g.n; j += 64) {
    const double v = (double)Elem<GS>::load1(gp + j);
    ss += v * v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if (lane == 0) {
    float *v = g.vec + (int64_t)slot * g.m + i;
    *v = (float)(g.a * (double)*v + g.b * ss);
  }
}

// Column sums of squares, first pass: rows are cut into `segs` segments so that a tall
// parameter still fills the GPU.  grid (ceil(n / 256), segs, batch): thread = column.
template <typename GS>
__global__ __launch_bounds__(256) void diag_col_partial_kernel(const DiagFactorArgs g) {
  const int slot = blockIdx.z, seg = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= g.n) return;
  const BlockDesc d = g.desc[slot];
  const GS *gp = reinterpret_cast<const GS *>(g.g_table[d.param]) + d.offset + j;
  const int i0 = seg * g.rows_per_seg, i1 = min(i0 + g.rows_per_seg, g.m);
  double ss = 0.0;
  for (int i = i0; i < i1; ++i) {
    const double v = (double)Elem<GS>::load1(gp + (int64_t)i * d.ld);
    ss += v * v;
  }
  g.partial[((int64_t)slot * g.segs + seg) * g.n + j] = (float)ss;
}

// Second pass: fixed-order sum of the segments, then the moving average.  grid (ceil(n / 256), batch).
__global__ __launch_bounds__(256) void diag_col_reduce_kernel(const DiagFactorArgs g) {
  const int slot = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= g.n) return;
  double ss = 0.0;
  for (int seg = 0; seg < g.segs; ++seg) ss += (double)g.partial[((int64_t)slot * g.segs + seg) * g.n + j];
  float *v = g.vec + (int64_t)slot * g.n + j;
  *v = (float)(g.a * (double)*v + g.b * ss);
}

struct DiagRootArgs {
  const float *vec;      // [batch][dim]
  float *out;            // [batch][dim]
  int32_t dim;
  float epsilon, r, scale;
  unsigned long long *fail_count;
};

// out_i = (scale v_i - min(min_i scale v_i, 0) + eps)^-r.  One workgroup per factor; a factor
// with a non-finite entry or root keeps its previous root and is counted (Sec. 3.2.3).
__global__ __launch_bounds__(256) void diag_root_kernel(const DiagRootArgs g) {
  __shared__ double redd[4];
  __shared__ int redi[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float *v = g.vec + (int64_t)b * g.dim;
  float *out = g.out + (int64_t)b * g.dim;
  int bad = 0;
  double lmin = 1.0e300;
  for (int i = tid; i < g.dim; i += 256) {
    const float x = v[i];
    if (!(fabsf(x) <= 3.0e38f)) bad = 1;
    lmin = fmin(lmin, (double)g.scale * (double)x);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { bad |= __shfl_xor(bad, off, 64); lmin = fmin(lmin, __shfl_xor(lmin, off, 64)); }
  if (lane == 0) { redd[wave] = lmin; redi[wave] = bad; }
  __syncthreads();
  lmin = fmin(fmin(redd[0], redd[1]), fmin(redd[2], redd[3]));
  bad = redi[0] | redi[1] | redi[2] | redi[3];
  const double shift = fmin(lmin, 0.0);
  // first the check, then the writes: a failed factor must be left untouched
  if (!bad)
    for (int i = tid; i < g.dim; i += 256) {
      const float f = (float)pow((double)g.scale * (double)v[i] - shift + (double)g.epsilon, -(double)g.r);
      if (!(f <= 3.0e38f) || !(f >= 0.f)) bad = 1;
    }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) bad |= __shfl_xor(bad, off, 64);
  __syncthreads();
  if (lane == 0) redi[wave] = bad;
  __syncthreads();
  bad = redi[0] | redi[1] | redi[2] | redi[3];
  if (bad) {
    if (tid == 0 && g.fail_count) atomicAdd(g.fail_count, 1ull);
    return;
  }
  for (int i = tid; i < g.dim; i += 256)
    out[i] = (float)pow((double)g.scale * (double)v[i] - shift + (double)g.epsilon, -(double)g.r);
}

struct DiagScaleArgs {
  const BlockDesc *desc;
  const void *const *g_table;   // source when src == nullptr: the gradient block
  const float *src;             // or a dense [slot][m][n] float32 array
  const float *dl, *dr;         // [slot][m], [slot][n]; nullptr = no scaling on that side
  float *out;                   // [slot][m][n]
  float *norm_partial;          // [slot][chunks] sums of squares of the output, or nullptr
  float alpha;
  int32_t m, n;
  EwGeom geom;
};

// out_ij = alpha dl_i src_ij dr_j.  grid: chunks * batch workgroups, chunk index fastest.
template <typename GD>
__global__ __launch_bounds__(EW_THREADS) void diag_scale_kernel(const DiagScaleArgs g) {
  __shared__ float red[EW_THREADS / 64];
  const int slot = blockIdx.x / g.geom.chunks, chunk = blockIdx.x - slot * g.geom.chunks, tid = threadIdx.x;
  const int n = g.n;
  const BlockDesc d = g.desc[slot];
  const GD *gp = g.src ? nullptr : reinterpret_cast<const GD *>(g.g_table[d.param]) + d.offset;
  const float *sp = g.src ? g.src + (int64_t)slot * g.m * n : nullptr;
  const int ld = g.src ? n : d.ld;
  const bool vec_in = g.src ? ((n & 3) == 0)
                            : (((d.ld & 3) == 0) && ((d.offset & 3) == 0) &&
                               ((reinterpret_cast<uintptr_t>(g.g_table[d.param]) & 15) == 0) && ((n & 3) == 0));
  const bool vec_out = (n & 3) == 0;
  float *op = g.out + (int64_t)slot * g.m * n;
  const float *dl = g.dl ? g.dl + (int64_t)slot * g.m : nullptr;
  const float *dr = g.dr ? g.dr + (int64_t)slot * n : nullptr;
  const int lx = g.geom.lanes_x_log2;
  const int tx = tid & ((1 << lx) - 1), ty = tid >> lx, ny = EW_THREADS >> lx;
  const int r0 = chunk * g.geom.rows_per_wg;
  const int r1 = min(r0 + g.geom.rows_per_wg, g.m);
  float ss = 0.f;
  for (int i = r0 + ty; i < r1; i += ny) {
    const float li = g.alpha * (dl ? dl[i] : 1.f);
    for (int j = tx * 4; j < n; j += 4 << lx) {
      const int valid = min(4, n - j);
      float v[4];
      if (sp) load_f4(sp + (int64_t)i * ld + j, vec_in, valid, v);
      else load_g4<GD>(gp + (int64_t)i * ld + j, vec_in, valid, v);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] *= li * ((dr && e < valid) ? dr[j + e] : 1.f);
        if (e < valid) ss += v[e] * v[e];
      }
      store_f4(op + (int64_t)i * n + j, vec_out, valid, v);
    }
  }
  if (g.norm_partial) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    if (tid == 0) g.norm_partial[(int64_t)slot * g.geom.chunks + chunk] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

}  // namespace shampoo
