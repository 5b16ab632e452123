// Coupled inverse Newton iteration for the root inverse (Sec. 3.2.1, item 2 of the paper):
//   A = scale * L + eps I,  c^p = 2 ||A||_F / (p + 1),  X_0 = I / c,  M_0 = A / c^p,
//   T_k = ((p + 1) I - M_k) / p,  X_{k+1} = X_k T_k,  M_{k+1} = T_k^p M_k,
// until ||M_k - I||_inf < tol.  Every iterate is a polynomial in A, hence symmetric, and all
// of them commute: each product is formed on its lower-triangular tiles only and mirrored
// (the SYRK epilogue of the GEMM kernel), 36 of 64 tiles at n = 1024.  The kernels here are
// the small elementwise / reduction steps around those products; convergence is tracked per
// matrix on the device (`done` flags, which the GEMM launches take as their skip list), so
// a refresh needs no host synchronisation.
//
// Arithmetic is float32 (MFMA with float32 accumulation).  ||M_k - I||_inf cannot fall below
// about n * 2^-24 * (a few) in that arithmetic, so besides the paper's test the iteration of
// a matrix also ends when the norm, once below 0.1 (quadratic regime), fails to halve.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace shampoo {

struct NewtonArgs {
  const float *a;        // [batch][n][n] input matrices
  int64_t a_stride;
  float *M, *X, *T;      // [batch][n][n] work matrices
  double *rowpart;       // [batch][n] row sums of squares of A
  float *err;            // [batch] ||M - I||_inf of the current iterate (atomic max, cleared by check)
  float *prev;           // [batch] the norm one iteration earlier
  int32_t *done;         // [batch] iteration finished (converged, stalled, capped or failed)
  int32_t *failed;       // [batch] not finite: the caller keeps the previous root
  int32_t *iters;        // [batch] number of iterations taken
  int32_t n, p, k, max_iter;
  float epsilon, scale, tol;
};

// grid (n, batch): row i of A = scale * sym(L) + eps I: sum of squares, non-finite check.
__global__ __launch_bounds__(256) void newton_rownorm_kernel(const NewtonArgs g) {
  __shared__ double red[4];
  const int i = blockIdx.x, b = blockIdx.y, n = g.n, tid = threadIdx.x;
  const float *a = g.a + (int64_t)b * g.a_stride;
  double ss = 0.0;
  int bad = 0;
  for (int j = tid; j < n; j += 256) {
    const float lo = a[(int64_t)i * n + j], up = a[(int64_t)j * n + i];
    if (!(fabsf(lo) <= 3.0e38f) || !(fabsf(up) <= 3.0e38f)) bad = 1;
    double v = (double)g.scale * 0.5 * ((double)lo + (double)up);
    if (i == j) v += (double)g.epsilon;
    ss += v * v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { ss += __shfl_xor(ss, off, 64); bad |= __shfl_xor(bad, off, 64); }
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  if (bad && (tid & 63) == 0) atomicOr(&g.failed[b], 1);
  __syncthreads();
  if (tid == 0) g.rowpart[(int64_t)b * n + i] = (red[0] + red[1]) + (red[2] + red[3]);
}

// grid (n, batch): row i of M_0 = A / c^p and X_0 = I / c; the Frobenius norm is summed from
// the row parts in a fixed order by every workgroup.
__global__ __launch_bounds__(256) void newton_init_kernel(const NewtonArgs g) {
  __shared__ double red[4];
  const int i = blockIdx.x, b = blockIdx.y, n = g.n, tid = threadIdx.x;
  if (g.failed[b]) {
    if (i == 0 && tid == 0) { g.done[b] = 1; g.iters[b] = 0; }
    return;
  }
  double ss = 0.0;
  for (int j = tid; j < n; j += 256) ss += g.rowpart[(int64_t)b * n + j];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const double fro = sqrt((red[0] + red[1]) + (red[2] + red[3]));
  const double cp = 2.0 * fro / ((double)g.p + 1.0);           // c^p
  const bool ok = cp > 0.0 && cp <= 1.0e300;
  const double inv_cp = ok ? 1.0 / cp : 0.0;
  const float inv_c = ok ? (float)pow(cp, -1.0 / (double)g.p) : 0.f;
  const float *a = g.a + (int64_t)b * g.a_stride;
  float *M = g.M + (int64_t)b * n * n, *X = g.X + (int64_t)b * n * n;
  for (int j = tid; j < n; j += 256) {
    double v = (double)g.scale * 0.5 * ((double)a[(int64_t)i * n + j] + (double)a[(int64_t)j * n + i]);
    if (i == j) v += (double)g.epsilon;
    M[(int64_t)i * n + j] = (float)(v * inv_cp);
    X[(int64_t)i * n + j] = (i == j) ? inv_c : 0.f;
  }
  if (i == 0 && tid == 0) {
    g.done[b] = ok ? 0 : 1;
    if (!ok) g.failed[b] = 1;      // zero or non-finite norm
    g.iters[b] = 0; g.err[b] = 0.f; g.prev[b] = 3.0e38f;
  }
}

// grid (n, batch): row i of T = ((p + 1) I - M) / p and of ||M - I||_inf.
__global__ __launch_bounds__(256) void newton_prep_kernel(const NewtonArgs g) {
  __shared__ float red[4];
  const int i = blockIdx.x, b = blockIdx.y, n = g.n, tid = threadIdx.x;
  if (g.done[b]) return;
  const float *M = g.M + (int64_t)b * n * n + (int64_t)i * n;
  float *T = g.T + (int64_t)b * n * n + (int64_t)i * n;
  const float pp = (float)g.p, inv_p = 1.f / pp;
  float rs = 0.f;
  for (int j = tid; j < n; j += 256) {
    const float mv = M[j], id = (i == j) ? 1.f : 0.f;
    rs += fabsf(mv - id);
    T[j] = ((pp + 1.f) * id - mv) * inv_p;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) rs += __shfl_xor(rs, off, 64);
  if ((tid & 63) == 0) red[tid >> 6] = rs;
  __syncthreads();
  if (tid == 0) {
    float r = (red[0] + red[1]) + (red[2] + red[3]);
    if (!(r <= 3.0e38f)) r = __int_as_float(0x7f800000);   // NaN / inf -> +inf, which orders above everything
    atomicMax(reinterpret_cast<int *>(g.err + b), __float_as_int(r));   // r >= 0: int order = float order
  }
}

// one thread per matrix: the termination test on M_k (k = g.k)
__global__ __launch_bounds__(256) void newton_check_kernel(const NewtonArgs g, int batch) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= batch || g.done[b]) return;
  const float e = g.err[b], pv = g.prev[b];
  int stop = 0;
  if (!(e <= 3.0e38f)) { g.failed[b] = 1; stop = 1; }
  else if (e < g.tol) stop = 1;                               // the paper's criterion
  else if (g.k >= g.max_iter) stop = 1;                       // iteration cap
  else if (pv < 0.1f && e > 0.5f * pv) stop = 1;              // float32 floor reached
  if (stop) { g.done[b] = 1; g.iters[b] = g.k; }
  g.prev[b] = e;
  g.err[b] = 0.f;
}

struct NewtonFinishArgs {
  const float *X; float *x; int64_t x_stride;
  const int32_t *done, *failed; int32_t *failed_out; unsigned long long *fail_count;
  const int32_t *iters; int32_t *iters_out;
  int32_t n, k;
};

// grid (n, batch), launched after the test on M_k: a matrix whose iteration ended at exactly
// this k copies row i of X_k into the output (unless it failed) and reports its status.
__global__ __launch_bounds__(256) void newton_finish_kernel(const NewtonFinishArgs g) {
  const int i = blockIdx.x, b = blockIdx.y, n = g.n, tid = threadIdx.x;
  if (!g.done[b] || g.iters[b] != g.k) return;
  const int bad = g.failed[b];
  if (i == 0 && tid == 0) {
    if (g.failed_out) g.failed_out[b] = bad;
    if (g.iters_out) g.iters_out[b] = g.iters[b];
    if (bad && g.fail_count) atomicAdd(g.fail_count, 1ull);
  }
  if (bad) return;
  const float *X = g.X + (int64_t)b * n * n + (int64_t)i * n;
  float *x = g.x + (int64_t)b * g.x_stride + (int64_t)i * n;
  for (int j = tid; j < n; j += 256) x[j] = X[j];
}

}  // namespace shampoo
