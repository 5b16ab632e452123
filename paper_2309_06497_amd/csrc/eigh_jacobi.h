// Batched symmetric eigensolver for the root-inverse refresh (framed box of
// Sec. 3.2.1 of the paper: lambda, Q = eigh(L); lambda' = lambda - min(lambda_min, 0)
// + eps; return Q diag(lambda'^-r) Q^T).  The paper calls a library eigh; this is
// a Jacobi solver laid out for CDNA4:
//
//  * n <= 128: one workgroup per matrix, the matrix A (float64, packed lower
//    triangle) and the accumulated rotations J (float32) both resident in LDS
//    (132 KB at n = 128).  Rounds of n/2 disjoint rotations
//    (round-robin tournament ordering); in a round every thread updates whole
//    2 x 2 blocks  R_k^T [a b; c d] R_l  so rows and columns are rotated in one
//    pass with no intermediate barrier.  The root inverse is formed in the
//    same kernel from LDS.
//  * n > 128: two-sided block Jacobi.  The matrix (padded to a multiple of 64)
//    is cut into 32-wide block columns; a round pairs them up, each 64 x 64
//    pivot is diagonalised by the LDS solver above, and the 64 x 64 rotation
//    blocks are applied to A (both sides, A_kl <- J_k^T A_kl J_l, float64 MFMA)
//    and to Q^T (rows, float32 MFMA).  The reconstruction Q f(Lambda) Q^T reuses
//    the batched SYRK kernel.
//
// Rotations are applied in the form x' = x - s (y + tau x), y' = y + s (x - tau y)
// with tau = s / (1 + c): for small angles the cosine rounds to 1 and the plain
// form c x - s y would let the columns of Q grow by t^2 per rotation.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"

namespace shampoo {

constexpr int JAC_THREADS = 256;
constexpr int JAC_NB = 32;            // block-column width of the block solver
constexpr int JAC_PIV = 2 * JAC_NB;   // pivot size
constexpr int JAC_SMALL_MAX = 128;    // largest n solved entirely in LDS
constexpr int JAC_SMALL_SWEEPS = 20;
constexpr int JAC_OUTER_SWEEPS = 16;
constexpr int JAC_INNER_SWEEPS = 2;
// rotation thresholds |a_pq| > rel * sqrt(|a_pp a_qq|) and > abs * max|diag(input)|
constexpr double JAC_SMALL_TOL_REL = 1e-11;   // LDS solver on a float64 copy of the factor
constexpr double JAC_SMALL_TOL_ABS = 1e-15;

struct JacScratch {      // small per-workgroup LDS arrays
  double s[JAC_SMALL_MAX / 2];
  double t[JAC_SMALL_MAX / 2];
  int p[JAC_SMALL_MAX / 2];
  int q[JAC_SMALL_MAX / 2];
  int flag;
};

// Pair k of round r of a round-robin tournament over `cnt` (even) players.
__device__ __host__ __forceinline__ void rr_pair(int cnt, int r, int k, int &p, int &q) {
  const int m1 = cnt - 1;
  if (k == 0) { p = m1; q = r; }
  else {
    p = r + k; if (p >= m1) p -= m1;
    q = r - k; if (q < 0) q += m1;
  }
  if (p > q) { const int t = p; p = q; q = t; }
}

// index of element (i, j) of a symmetric matrix stored as its packed lower triangle
__device__ __forceinline__ int tri(int i, int j) {
  return i >= j ? i * (i + 1) / 2 + j : j * (j + 1) / 2 + i;
}

// Up to max_sweeps sweeps of parallel two-sided Jacobi on the s x s (s even)
// symmetric matrix At (float64, packed lower triangle), accumulating the
// rotations into the float32 matrix J <- J R (row stride LD, odd).  Keeping A in
// float64 makes the small eigenvalues of an ill-conditioned factor (a single
// G G^T at the first refresh) as accurate as the stored factor allows; the
// rotations themselves only need float32.  Because A is symmetric only the
// 2 x 2 blocks (rows of pair k, columns of pair l) with l <= k are updated.
// Returns nonzero if any rotation was applied.  All threads must call it.
__device__ int jacobi_sweeps(double *At, float *Js, int s, const int LD, int max_sweeps, double tol_rel,
                             double tol_abs, JacScratch *sc) {
  const int tid = threadIdx.x;
  const int half = s >> 1;
  int any = 0;
  for (int sw = 0; sw < max_sweeps; ++sw) {
    if (tid == 0) sc->flag = 0;
    __syncthreads();
    for (int r = 0; r < s - 1; ++r) {
      if (tid < half) {
        int p, q;
        rr_pair(s, r, tid, p, q);   // p < q
        const double app = At[tri(p, p)], aqq = At[tri(q, q)], apq = At[tri(q, p)];
        double sn = 0.0, tp = 0.0;
        const double aa = fabs(apq);
        if (aa > tol_abs && aa > tol_rel * sqrt(fabs(app * aqq))) {
          const double tau = (aqq - app) / (2.0 * apq);
          const double t = copysign(1.0, tau) / (fabs(tau) + sqrt(1.0 + tau * tau));
          const double c = 1.0 / sqrt(1.0 + t * t);
          sn = t * c;
          tp = sn / (1.0 + c);
          if (sn != 0.0) sc->flag = 1;
        }
        sc->s[tid] = sn; sc->t[tid] = tp; sc->p[tid] = p; sc->q[tid] = q;
      }
      __syncthreads();
      // A <- R^T A R on the blocks with l <= k
      for (int k = tid >> 5; k < half; k += JAC_THREADS / 32) {
        const int pk = sc->p[k], qk = sc->q[k];
        const double sk = sc->s[k], tk = sc->t[k];
        for (int l = tid & 31; l <= k; l += 32) {
          const int pl = sc->p[l], ql = sc->q[l];
          const double sl = sc->s[l], tl = sc->t[l];
          if (sk == 0.0 && sl == 0.0) continue;
          const int ia = tri(pk, pl), ib = tri(pk, ql), ic = tri(qk, pl), id = tri(qk, ql);
          double a = At[ia], b = At[ib], c = At[ic], d = At[id];
          // rows: (a, c) and (b, d) are (x, y) pairs of rotation k
          const double a1 = a - sk * (c + tk * a), c1 = c + sk * (a - tk * c);
          const double b1 = b - sk * (d + tk * b), d1 = d + sk * (b - tk * d);
          // columns: (a1, b1) and (c1, d1) are (x, y) pairs of rotation l
          a = a1 - sl * (b1 + tl * a1); b = b1 + sl * (a1 - tl * b1);
          c = c1 - sl * (d1 + tl * c1); d = d1 + sl * (c1 - tl * d1);
          if (k == l) {   // pivot block: ib == ic is the annihilated element
            At[ia] = a; At[ib] = 0.0; At[id] = d;
          } else {
            At[ia] = a; At[ib] = b; At[ic] = c; At[id] = d;
          }
        }
      }
      // J <- J R (columns)
      for (int i = tid >> 5; i < s; i += JAC_THREADS / 32) {
        for (int l = tid & 31; l < half; l += 32) {
          const float sl = (float)sc->s[l];
          if (sl == 0.f) continue;
          const float tl = (float)sc->t[l];
          const int pl = sc->p[l], ql = sc->q[l];
          const float x = Js[i * LD + pl], y = Js[i * LD + ql];
          Js[i * LD + pl] = x - sl * (y + tl * x);
          Js[i * LD + ql] = y + sl * (x - tl * y);
        }
      }
      __syncthreads();
    }
    if (sc->flag == 0) break;
    any = 1;
    __syncthreads();   // everyone has read flag before thread 0 clears it again
  }
  return any;
}

// ---------------------------------------------------------------------------
// n <= 128: whole root inverse in one workgroup.
// ---------------------------------------------------------------------------
struct SmallRootArgs {
  const float *a;        // batch matrices, dense n x n, stride a_stride
  int64_t a_stride;
  float *x;              // outputs, dense n x n, stride x_stride
  int64_t x_stride;
  float *lambda;         // optional [batch][n]
  int32_t *failed;       // optional [batch]
  unsigned long long *fail_count;  // optional global counter
  int32_t n;
  float epsilon, r;
};

__global__ __launch_bounds__(JAC_THREADS) void rootinv_small_kernel(const SmallRootArgs g) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ float redf[JAC_THREADS / 64];
  __shared__ int redi[JAC_THREADS / 64];
  __shared__ JacScratch scratch;
  JacScratch *sc = &scratch;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  const int n = g.n;
  const int s = (n + 1) & ~1;
  const int LD = s + 1;
  double *At = reinterpret_cast<double *>(smem);            // s (s + 1) / 2
  float *Js = reinterpret_cast<float *>(At + s * (s + 1) / 2);
  float *fv = Js + s * LD;                                  // [s]
  const float *a = g.a + (int64_t)b * g.a_stride;

  // load (symmetrising: a no-op for exactly symmetric input), padding decoupled zeros
  int bad = 0;
  float dmax = 0.f;
  for (int i = tid >> 6; i < s; i += JAC_THREADS / 64)
    for (int j = lane; j < s; j += 64) {
      if (j <= i) {
        double v = 0.0;
        if (i < n) {
          const float lo = a[(int64_t)i * n + j], up = a[(int64_t)j * n + i];
          if (!(fabsf(lo) <= 3.0e38f) || !(fabsf(up) <= 3.0e38f)) bad = 1;
          v = 0.5 * ((double)lo + (double)up);
          if (i == j) dmax = fmaxf(dmax, fabsf(lo));
        }
        At[i * (i + 1) / 2 + j] = v;
      }
      Js[i * LD + j] = (i == j) ? 1.f : 0.f;
    }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    dmax = fmaxf(dmax, __shfl_xor(dmax, off, 64));
    bad |= __shfl_xor(bad, off, 64);
  }
  if (lane == 0) { redf[wave] = dmax; redi[wave] = bad; }
  __syncthreads();
  dmax = fmaxf(fmaxf(redf[0], redf[1]), fmaxf(redf[2], redf[3]));
  bad = redi[0] | redi[1] | redi[2] | redi[3];
  if (bad) {   // uniform: Sec. 3.2.3, keep the previous root
    if (tid == 0) {
      if (g.failed) g.failed[b] = 1;
      if (g.fail_count) atomicAdd(g.fail_count, 1ull);
    }
    return;
  }

  jacobi_sweeps(At, Js, s, LD, JAC_SMALL_SWEEPS, JAC_SMALL_TOL_REL, JAC_SMALL_TOL_ABS * (double)dmax, sc);
  __syncthreads();

  // lambda_min over the true eigenvalues, then f = (lambda - min(lambda_min, 0) + eps)^-r
  double lmin = 1.0e300;
  for (int i = tid; i < n; i += JAC_THREADS) lmin = fmin(lmin, At[i * (i + 1) / 2 + i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) lmin = fmin(lmin, __shfl_xor(lmin, off, 64));
  __syncthreads();
  if (lane == 0) reinterpret_cast<double *>(sc->s)[wave] = lmin;   // rotation scratch is free now
  __syncthreads();
  lmin = fmin(fmin(sc->s[0], sc->s[1]), fmin(sc->s[2], sc->s[3]));
  const double shift = fmin(lmin, 0.0);
  int badf = 0;
  for (int i = tid; i < s; i += JAC_THREADS) {
    float f = 0.f;
    if (i < n) {
      const double lam = At[i * (i + 1) / 2 + i];
      f = (float)pow(lam - shift + (double)g.epsilon, -(double)g.r);
      if (!(f <= 3.0e38f) || !(f >= 0.f)) badf = 1;
      if (g.lambda) g.lambda[(int64_t)b * n + i] = (float)lam;
    }
    fv[i] = sqrtf(f);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) badf |= __shfl_xor(badf, off, 64);
  if (lane == 0) redi[wave] = badf;
  __syncthreads();
  badf = redi[0] | redi[1] | redi[2] | redi[3];
  if (tid == 0 && g.failed) g.failed[b] = badf ? 1 : 0;
  if (badf) {
    if (tid == 0 && g.fail_count) atomicAdd(g.fail_count, 1ull);
    return;
  }
  // J <- J diag(sqrt f); X = J J^T, lower triangle computed and mirrored
  for (int i = tid >> 6; i < n; i += JAC_THREADS / 64)
    for (int k = lane; k < s; k += 64) Js[i * LD + k] *= fv[k];
  __syncthreads();
  float *x = g.x + (int64_t)b * g.x_stride;
  for (int i = tid >> 6; i < n; i += JAC_THREADS / 64)
    for (int j = lane; j <= i; j += 64) {
      float acc = 0.f;
      for (int k = 0; k < n; ++k) acc += Js[i * LD + k] * Js[j * LD + k];
      x[(int64_t)i * n + j] = acc;
      x[(int64_t)j * n + i] = acc;
    }
}

inline size_t rootinv_small_lds_bytes(int n) {
  const int s = (n + 1) & ~1;
  return (size_t)(s * (s + 1) / 2) * sizeof(double) + (size_t)(s * (s + 1) + s) * sizeof(float);
}

// ---------------------------------------------------------------------------
// n > 128: block Jacobi.  Work arrays per matrix (np = n rounded up to 64):
//   W  [np][np] float64  the matrix being diagonalised (padding: zero, decoupled);
//                        kept exactly symmetric (mirrored writes)
//   Qt [np][np] float32  accumulated rotations, transposed (rows are eigenvectors)
//   J  [np/64][64][64] float32 rotation blocks of the current round
// W is float64 for the same reason as in the LDS solver: the update
// A_kl <- J_k^T A_kl J_l runs on the float64 matrix cores (v_mfma_f64_16x16x4_f64),
// so eigenvalues far below 2^-24 lambda_max survive the ~400 updates of a solve.
// J is only orthogonal to float32 accuracy; applied as a congruence this moves
// every eigenvalue by a *relative* 1e-7 per round, which is harmless.
// ---------------------------------------------------------------------------
typedef double doublex4 __attribute__((ext_vector_type(4)));

struct BlockJacArgs {
  double *w;
  float *qt;
  float *jbuf;
  int32_t *ident;        // [batch][np/64]: pivot of the current round needed no rotation
  int32_t *rot;          // [batch][JAC_OUTER_SWEEPS]: pivots that rotated, per outer sweep
  const float *dmax;     // [batch]
  const int32_t *failed; // [batch]
  int32_t np;            // padded size
  int32_t round, sweep;
};

struct BlockInitArgs {
  const float *a; int64_t a_stride; int32_t n;
  double *w; float *qt; int32_t np;
  float *dmax; int32_t *failed; int32_t *rot;
};

// W = pad(sym(A)), Qt = I, dmax, failed, rot = 0.  grid (np, batch), 256 threads.
__global__ __launch_bounds__(256) void blockjac_init_kernel(const BlockInitArgs g) {
  const int b = blockIdx.y, i = blockIdx.x, np = g.np, n = g.n;
  double *w = g.w + (int64_t)b * np * np + (int64_t)i * np;
  float *qt = g.qt + (int64_t)b * np * np + (int64_t)i * np;
  const float *a = g.a + (int64_t)b * g.a_stride;
  int bad = 0;
  for (int j = threadIdx.x; j < np; j += 256) {
    double v = 0.0;
    if (i < n && j < n) {
      const float lo = a[(int64_t)i * n + j], up = a[(int64_t)j * n + i];
      if (!(fabsf(lo) <= 3.0e38f) || !(fabsf(up) <= 3.0e38f)) bad = 1;
      v = 0.5 * ((double)lo + (double)up);
    }
    w[j] = v;
    qt[j] = (i == j) ? 1.f : 0.f;
  }
  if (bad) g.failed[b] = 1;
  if (i < n && threadIdx.x == 0) {
    const float d = fabsf(a[(int64_t)i * n + i]);
    if (d <= 3.0e38f) atomicMax(reinterpret_cast<int *>(g.dmax + b), __float_as_int(d));  // d >= 0: int order = float order
  }
  if (i == 0 && threadIdx.x < JAC_OUTER_SWEEPS) g.rot[b * JAC_OUTER_SWEEPS + threadIdx.x] = 0;
}

constexpr int PIV_LD = JAC_PIV + 1;

// One workgroup per (pair, matrix): diagonalise the 64 x 64 pivot.
__global__ __launch_bounds__(JAC_THREADS) void blockjac_pivot_kernel(const BlockJacArgs g) {
  __shared__ double At[JAC_PIV * (JAC_PIV + 1) / 2];
  __shared__ float Js[JAC_PIV * PIV_LD];
  __shared__ JacScratch sc;
  const int b = blockIdx.y, pair = blockIdx.x;
  if (g.failed[b]) return;
  if (g.sweep > 0 && g.rot[b * JAC_OUTER_SWEEPS + g.sweep - 1] == 0) return;   // converged
  const int np = g.np, nblk = np / JAC_NB;
  int pb, qb;
  rr_pair(nblk, g.round, pair, pb, qb);
  const double *w = g.w + (int64_t)b * np * np;
  const int tid = threadIdx.x;
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64) {
    const int j = tid & 63;
    const int gi = (i < JAC_NB ? pb * JAC_NB + i : qb * JAC_NB + i - JAC_NB);
    const int gj = (j < JAC_NB ? pb * JAC_NB + j : qb * JAC_NB + j - JAC_NB);
    if (j <= i) At[i * (i + 1) / 2 + j] = w[(int64_t)gi * np + gj];
    Js[i * PIV_LD + j] = (i == j) ? 1.f : 0.f;
  }
  __syncthreads();
  const double dm = (double)g.dmax[b];
  const int any = jacobi_sweeps(At, Js, JAC_PIV, PIV_LD, JAC_INNER_SWEEPS, JAC_SMALL_TOL_REL, JAC_SMALL_TOL_ABS * dm, &sc);
  __syncthreads();
  if (tid == 0) {
    g.ident[b * (nblk / 2) + pair] = any ? 0 : 1;
    if (any) atomicAdd(&g.rot[b * JAC_OUTER_SWEEPS + g.sweep], 1);
  }
  if (!any) return;
  float *jout = g.jbuf + ((int64_t)b * (nblk / 2) + pair) * JAC_PIV * JAC_PIV;
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64) jout[i * JAC_PIV + (tid & 63)] = Js[i * PIV_LD + (tid & 63)];
}

constexpr int APP_LD = JAC_PIV + 4;

// Loads rotation block `idx` of this matrix into LDS (identity if that pivot did not rotate).
__device__ __forceinline__ void load_rotation(float *dst, const float *jb, int idx, bool ident, int tid) {
  const int c = tid & 63;
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64)
    dst[i * APP_LD + c] = ident ? (i == c ? 1.f : 0.f) : jb[((int64_t)idx * JAC_PIV + i) * JAC_PIV + c];
}

// W_kl <- J_k^T W_kl J_l for the pair-blocks l <= k of one matrix, in float64 on the
// matrix cores; the transposed result is written to W_lk.  grid (hp (hp + 1) / 2, batch).
// Wavefront (wi, wj) owns the 32 x 32 quadrant as 2 x 2 tiles of 16 x 16; a 16x16x4
// MFMA takes A(i, k) from lane (i = lane % 16, k = lane / 16), B(k, j) likewise, and
// leaves D(4 (lane / 16) + v, lane % 16) in element v of the lane's result.
__global__ __launch_bounds__(JAC_THREADS, 2) void blockjac_apply_w_kernel(const BlockJacArgs g) {
  __shared__ __align__(16) float Jk[JAC_PIV * APP_LD];
  __shared__ __align__(16) float Jl[JAC_PIV * APP_LD];
  __shared__ __align__(32) double X[JAC_PIV * APP_LD];   // W_kl, then (J_k^T W_kl)^T
  const int b = blockIdx.y;
  if (g.failed[b]) return;
  if (g.sweep > 0 && g.rot[b * JAC_OUTER_SWEEPS + g.sweep - 1] == 0) return;
  const int np = g.np, nblk = np / JAC_NB, hp = nblk / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int32_t *ident = g.ident + b * hp;
  const float *jb = g.jbuf + (int64_t)b * hp * JAC_PIV * JAC_PIV;
  // lower-triangular pair-block index: blockIdx.x = k (k + 1) / 2 + l, l <= k
  int k = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
  while ((k + 1) * (k + 2) / 2 <= (int)blockIdx.x) ++k;
  while (k * (k + 1) / 2 > (int)blockIdx.x) --k;
  const int l = blockIdx.x - k * (k + 1) / 2;
  if (ident[k] && ident[l]) return;
  double *w = g.w + (int64_t)b * np * np;
  int pk, qk, pl, ql;
  rr_pair(nblk, g.round, k, pk, qk);
  rr_pair(nblk, g.round, l, pl, ql);

  const int c = tid & 63;
  const int gcol = (c < JAC_NB ? pl * JAC_NB + c : ql * JAC_NB + c - JAC_NB);
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64) {
    const int grow = (i < JAC_NB ? pk * JAC_NB + i : qk * JAC_NB + i - JAC_NB);
    X[i * APP_LD + c] = w[(int64_t)grow * np + gcol];
  }
  load_rotation(Jk, jb, k, ident[k] != 0, tid);
  load_rotation(Jl, jb, l, ident[l] != 0, tid);
  __syncthreads();

  const int li = lane & 15, lk = lane >> 4;
  doublex4 acc[2][2];
  // T = J_k^T X :  A(i, kk) = Jk[kk][i], B(kk, j) = X[kk][j]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 2; ++e) acc[a][e] = (doublex4){0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
  for (int kk = 0; kk < JAC_PIV; kk += 4) {
    const int row = (kk + lk) * APP_LD;
    const double a0 = (double)Jk[row + wi * 32 + li], a1 = (double)Jk[row + wi * 32 + 16 + li];
    const double b0 = X[row + wj * 32 + li], b1 = X[row + wj * 32 + 16 + li];
    acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
  }
  __syncthreads();   // all reads of X done
  // X <- T^T : lane holds T(i0 .. i0+3, j)
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int i0 = wi * 32 + a * 16 + 4 * lk, j = wj * 32 + e * 16 + li;
      *reinterpret_cast<doublex4 *>(&X[j * APP_LD + i0]) = acc[a][e];
    }
  __syncthreads();
  // C = T J_l :  A(i, kk) = X[kk][i] (= T[i][kk]), B(kk, j) = Jl[kk][j]
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 2; ++e) acc[a][e] = (doublex4){0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
  for (int kk = 0; kk < JAC_PIV; kk += 4) {
    const int row = (kk + lk) * APP_LD;
    const double a0 = X[row + wi * 32 + li], a1 = X[row + wi * 32 + 16 + li];
    const double b0 = (double)Jl[row + wj * 32 + li], b1 = (double)Jl[row + wj * 32 + 16 + li];
    acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
  }
  // write C to block (k, l) and C^T to block (l, k); on the diagonal (k == l) only the
  // lower half is kept and mirrored, so W stays exactly symmetric
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int j = wj * 32 + e * 16 + li;
      const int gc = (j < JAC_NB ? pl * JAC_NB + j : ql * JAC_NB + j - JAC_NB);
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int i = wi * 32 + a * 16 + 4 * lk + v;
        const int gr = (i < JAC_NB ? pk * JAC_NB + i : qk * JAC_NB + i - JAC_NB);
        if (k != l || j <= i) {
          const double val = (k == l && i == j) ? acc[a][e][v] : acc[a][e][v];
          w[(int64_t)gr * np + gc] = val;
          if (gr != gc) w[(int64_t)gc * np + gr] = val;
        }
      }
    }
}

// 64 x 64 x 64 float32 product on one workgroup: wavefront (wi, wj) computes the 32 x 32
// tile  C[i][j] = sum_k At[k][i] * B[k][j]  from LDS (both operands k-major).
__device__ __forceinline__ floatx16 mfma_64(const float *At, const float *B, int wi, int wj, int lane) {
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int i = wi * 32 + (lane & 31), j = wj * 32 + (lane & 31), kh = lane >> 5;
#pragma unroll 8
  for (int k = 0; k < JAC_PIV; k += 2)
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(At[(k + kh) * APP_LD + i], B[(k + kh) * APP_LD + j], acc, 0, 0, 0);
  return acc;
}

// Qt rows of pair k <- J_k^T (those rows), one 64-column tile per workgroup, float32 MFMA.
// grid (hp * np / 64, batch).
__global__ __launch_bounds__(JAC_THREADS, 2) void blockjac_apply_q_kernel(const BlockJacArgs g) {
  __shared__ __align__(16) float Jk[JAC_PIV * APP_LD];
  __shared__ __align__(16) float X[JAC_PIV * APP_LD];
  const int b = blockIdx.y;
  if (g.failed[b]) return;
  if (g.sweep > 0 && g.rot[b * JAC_OUTER_SWEEPS + g.sweep - 1] == 0) return;
  const int np = g.np, nblk = np / JAC_NB, hp = nblk / 2, ctiles = np / JAC_PIV;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int k = blockIdx.x / ctiles, ctile = blockIdx.x - k * ctiles;
  if (g.ident[b * hp + k]) return;
  float *qt = g.qt + (int64_t)b * np * np;
  int pk, qk;
  rr_pair(nblk, g.round, k, pk, qk);
  const int c = tid & 63;
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64) {
    const int grow = (i < JAC_NB ? pk * JAC_NB + i : qk * JAC_NB + i - JAC_NB);
    X[i * APP_LD + c] = qt[(int64_t)grow * np + ctile * JAC_PIV + c];
  }
  load_rotation(Jk, g.jbuf + (int64_t)b * hp * JAC_PIV * JAC_PIV, k, false, tid);
  __syncthreads();
  const floatx16 acc = mfma_64(Jk, X, wi, wj, lane);
  const int gc = ctile * JAC_PIV + wj * 32 + (lane & 31);
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = wi * 32 + 8 * q + 4 * (lane >> 5) + e;
      const int grow = (i < JAC_NB ? pk * JAC_NB + i : qk * JAC_NB + i - JAC_NB);
      qt[(int64_t)grow * np + gc] = acc[4 * q + e];
    }
}

struct BlockFinalArgs {
  const double *w; int32_t np; int32_t n;
  float epsilon, r;
  float *fvals;          // [batch][np]: lambda'^-r (0 on padding)
  float *lambda;         // optional [batch][n]
  int32_t *failed;       // [batch] in/out
  int32_t *failed_out;   // optional user-visible copy
  unsigned long long *fail_count;
};

// One workgroup per matrix: eigenvalues = diag(W); shift; f(lambda).
__global__ __launch_bounds__(256) void blockjac_final_kernel(const BlockFinalArgs g) {
  __shared__ double redf[4];
  __shared__ int redi[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int np = g.np, n = g.n;
  const double *w = g.w + (int64_t)b * np * np;
  float *fv = g.fvals + (int64_t)b * np;
  const int bad = g.failed[b];
  double lmin = 1.0e300;
  if (!bad)
    for (int i = tid; i < n; i += 256) lmin = fmin(lmin, w[(int64_t)i * np + i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) lmin = fmin(lmin, __shfl_xor(lmin, off, 64));
  if (lane == 0) redf[wave] = lmin;
  __syncthreads();
  lmin = fmin(fmin(redf[0], redf[1]), fmin(redf[2], redf[3]));
  const double shift = fmin(lmin, 0.0);
  int badf = bad;
  for (int i = tid; i < np; i += 256) {
    float f = 0.f;
    if (i < n && !bad) {
      const double lam = w[(int64_t)i * np + i];
      f = (float)pow(lam - shift + (double)g.epsilon, -(double)g.r);
      if (!(f <= 3.0e38f) || !(f >= 0.f)) badf = 1;
      if (g.lambda) g.lambda[(int64_t)b * n + i] = (float)lam;
    }
    fv[i] = f;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) badf |= __shfl_xor(badf, off, 64);
  if (lane == 0) redi[wave] = badf;
  __syncthreads();
  badf = redi[0] | redi[1] | redi[2] | redi[3];
  if (tid == 0) {
    g.failed[b] = badf;
    if (g.failed_out) g.failed_out[b] = badf;
    if (badf && g.fail_count) atomicAdd(g.fail_count, 1ull);
  }
}

}  // namespace shampoo
