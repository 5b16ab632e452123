// Blocks of tensor parameters (Sec. 2.3 of the paper: Shampoo for a tensor of order w keeps one
// factor per dimension and preconditions by mode products; Sec. 4.2.1: merging and blocking).
//
// A block d1 x d2 x d3 (x d4) of a D1 x D2 x D3 (x D4) parameter is strided two or three times
// inside the caller's tensor.  The step therefore works on a block-contiguous copy of the gradient and of the
// parameter (blocks back to back, in row-major order of their block indices), in which
//   * the unfolding along the first dimension is the plain d1 x (d2 d3 ...) matrix,
//   * the unfolding along the last dimension is the plain (d1 d2 ...) x d_last matrix read
//     "rows along k",
//   * the unfolding along a middle dimension k becomes plain once the block, seen as
//     pre x d_k x post, has its first two indices swapped (permute_12_kernel): d_k x (pre post),
// so every factor update and mode product is one of the batched SYRK / GEMM launches of the
// matrix case, and the elementwise kernels see the block as a d1 x (d2 d3) matrix.  The kernels
// here only move data: gather / scatter between the caller's tensor and the copy, and the swap.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"

namespace shampoo {

struct TensorCopyArgs {
  const void *tensor_in;   // gather: the caller's D1 x D2 x D3 tensor (row-major)
  void *tensor_out;        // scatter: the same
  const void *copy_in;     // scatter: the block-contiguous copy
  void *copy_out;          // gather: the same
  int64_t D1, D2, D3, D4;  // unused trailing dimensions are 1
  int32_t b;               // block size
  int32_t k2n, k3n, k4n;   // pieces along the second, third and fourth dimension
};

// grid (blocks, chunks): block index = ((k1 * k2n + k2) * k3n + k3) * k4n + k4.  All pieces
// before the last one of a dimension are full, so the offset of a block inside the copy is
// s1 D2 D3 D4 + d1 s2 D3 D4 + d1 d2 s3 D4 + d1 d2 d3 s4.
template <typename T, bool SCATTER>
__global__ __launch_bounds__(256) void tensor_block_copy_kernel(const TensorCopyArgs g) {
  int64_t blk = blockIdx.x;
  const int64_t k4 = blk % g.k4n; blk /= g.k4n;
  const int64_t k3 = blk % g.k3n; blk /= g.k3n;
  const int64_t k2 = blk % g.k2n, k1 = blk / g.k2n;
  const int64_t s1 = k1 * g.b, s2 = k2 * g.b, s3 = k3 * g.b, s4 = k4 * g.b;
  const int64_t d1 = min((int64_t)g.b, g.D1 - s1), d2 = min((int64_t)g.b, g.D2 - s2), d3 = min((int64_t)g.b, g.D3 - s3),
                d4 = min((int64_t)g.b, g.D4 - s4);
  const int64_t voff = s1 * g.D2 * g.D3 * g.D4 + d1 * (s2 * g.D3 * g.D4) + d1 * d2 * (s3 * g.D4) + d1 * d2 * d3 * s4;
  const int64_t n = d1 * d2 * d3 * d4;
  const T *tin = static_cast<const T *>(g.tensor_in);
  T *tout = static_cast<T *>(g.tensor_out);
  const T *cin = static_cast<const T *>(g.copy_in);
  T *cout = static_cast<T *>(g.copy_out);
  for (int64_t e = (int64_t)blockIdx.y * 256 + threadIdx.x; e < n; e += (int64_t)gridDim.y * 256) {
    int64_t r = e;
    const int64_t i4 = r % d4; r /= d4;
    const int64_t i3 = r % d3; r /= d3;
    const int64_t i2 = r % d2, i1 = r / d2;
    const int64_t at = (((s1 + i1) * g.D2 + (s2 + i2)) * g.D3 + (s3 + i3)) * g.D4 + s4 + i4;
    if (SCATTER) tout[at] = cin[voff + e];
    else cout[voff + e] = tin[at];
  }
}

struct PermuteArgs {
  const BlockDesc *desc;        // input through the pointer table (blocks of the copy) ...
  const void *const *table;
  const float *src;             // ... or a dense float32 array [slot][d1][d2][d3]
  float *dst;                   // [slot][d2][d1][d3]
  int32_t d1, d2, d3;
};

// dst[slot][i2][i1][i3] = in[slot][i1][i2][i3].  grid (chunks, slots).
template <typename T>
__global__ __launch_bounds__(256) void permute_12_kernel(const PermuteArgs g) {
  const int slot = blockIdx.y;
  const int64_t n = (int64_t)g.d1 * g.d2 * g.d3;
  const T *tin = nullptr;
  if (!g.src) {
    const BlockDesc d = g.desc[slot];
    tin = reinterpret_cast<const T *>(g.table[d.param]) + d.offset;
  }
  const float *fin = g.src ? g.src + (int64_t)slot * n : nullptr;
  float *out = g.dst + (int64_t)slot * n;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (int64_t)gridDim.x * 256) {
    const int64_t i3 = e % g.d3, i2 = (e / g.d3) % g.d2, i1 = e / ((int64_t)g.d3 * g.d2);
    const float v = fin ? fin[e] : Elem<T>::load1(tin + e);
    out[(i2 * g.d1 + i1) * g.d3 + i3] = v;
  }
}

struct GramReduceArgs {
  const float *partial;   // [slot][splits][d][d]
  float *factor;          // [slot][d][d]
  int32_t d, splits;
  double alpha, beta;
};

// factor <- beta factor + alpha sum_s partial_s, in float64, fixed order.  The factor of the
// last dimension of a tensor block is a d3 x d3 Gram matrix over d1 d2 rows (d3 = 9 for a
// 3 x 3 convolution, 16384 rows at block size 128): its rows are split into `splits` ranges
// whose Gram matrices are separate batch entries of the SYRK launch.  grid (ceil(d d / 256), slots).
__global__ __launch_bounds__(256) void gram_reduce_kernel(const GramReduceArgs g) {
  const int slot = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int dd = g.d * g.d;
  if (e >= dd) return;
  const float *p = g.partial + (int64_t)slot * g.splits * dd + e;
  double acc = 0.0;
  for (int s = 0; s < g.splits; ++s) acc += (double)p[(int64_t)s * dd];
  float *f = g.factor + (int64_t)slot * dd + e;
  *f = (float)(g.beta * (double)*f + g.alpha * acc);
}

}  // namespace shampoo
