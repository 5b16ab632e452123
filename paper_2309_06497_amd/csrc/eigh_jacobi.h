// Batched symmetric eigensolver for the root-inverse refresh (framed box of
// Sec. 3.2.1 of the paper: lambda, Q = eigh(L); lambda' = lambda - min(lambda_min, 0)
// + eps; return Q diag(lambda'^-r) Q^T).  The paper calls a library eigh; this is
// a Jacobi solver laid out for CDNA4:
//
//  * n <= 128: one workgroup per matrix, the matrix A and the accumulated
//    rotations J both resident in LDS.  Rounds of n/2 disjoint rotations
//    (round-robin tournament ordering); in a round every thread updates whole
//    2 x 2 blocks  R_k^T [a b; c d] R_l  so rows and columns are rotated in one
//    pass with no intermediate barrier.  The root inverse is formed in the
//    same kernel from LDS.
//  * n > 128: two-sided block Jacobi.  The matrix (padded to a multiple of 64)
//    is cut into 32-wide block columns; a round pairs them up, each 64 x 64
//    pivot is diagonalised by the LDS solver above, and the 64 x 64 rotation
//    blocks are applied to A (both sides, A_kl <- J_k^T A_kl J_l) and to Q^T
//    (rows) with fp32 MFMA.  The reconstruction Q f(Lambda) Q^T reuses the
//    batched SYRK kernel.
//
// Rotations are applied in the form x' = x - s (y + tau x), y' = y + s (x - tau y)
// with tau = s / (1 + c): for small angles the float32 cosine rounds to 1 and
// the plain form c x - s y would let the columns of Q grow by t^2 per rotation.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"

namespace shampoo {

constexpr int JAC_THREADS = 256;
constexpr int JAC_NB = 32;            // block-column width of the block solver
constexpr int JAC_PIV = 2 * JAC_NB;   // pivot size
constexpr int JAC_SMALL_MAX = 128;    // largest n solved entirely in LDS
constexpr int JAC_SMALL_SWEEPS = 16;
constexpr int JAC_OUTER_SWEEPS = 12;
constexpr int JAC_INNER_SWEEPS = 2;
constexpr float JAC_TOL_REL = 5.9604645e-8f;   // 2^-24
constexpr float JAC_TOL_ABS = 9.3132257e-10f;  // 2^-30, times the largest |diagonal| of the input

struct JacScratch {      // small per-workgroup LDS arrays
  float s[JAC_SMALL_MAX / 2];
  float t[JAC_SMALL_MAX / 2];
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

// Up to max_sweeps sweeps of parallel two-sided Jacobi on the s x s (s even)
// symmetric matrix As, accumulating J <- J R.  LD = LDS row stride (odd, so that
// column walks are bank-conflict free).  Returns nonzero if any rotation was
// applied.  All threads must call it.
__device__ int jacobi_sweeps(float *As, float *Js, int s, const int LD, int max_sweeps, float tol_abs, JacScratch *sc) {
  const int tid = threadIdx.x;
  const int half = s >> 1;
  int any = 0;
  for (int sw = 0; sw < max_sweeps; ++sw) {
    if (tid == 0) sc->flag = 0;
    __syncthreads();
    for (int r = 0; r < s - 1; ++r) {
      if (tid < half) {
        int p, q;
        rr_pair(s, r, tid, p, q);
        const float app = As[p * LD + p], aqq = As[q * LD + q], apq = As[p * LD + q];
        float sn = 0.f, tp = 0.f;
        const float aa = fabsf(apq);
        if (aa > tol_abs && aa > JAC_TOL_REL * sqrtf(fabsf(app * aqq))) {
          const float tau = (aqq - app) / (2.f * apq);
          const float t = copysignf(1.f, tau) / (fabsf(tau) + sqrtf(1.f + tau * tau));
          const float c = 1.f / sqrtf(1.f + t * t);
          sn = t * c;
          tp = sn / (1.f + c);
          if (sn != 0.f) sc->flag = 1;
        }
        sc->s[tid] = sn; sc->t[tid] = tp; sc->p[tid] = p; sc->q[tid] = q;
      }
      __syncthreads();
      // A <- R^T A R, one 2 x 2 block (rows of pair k, columns of pair l) per step
      for (int k = tid >> 5; k < half; k += JAC_THREADS / 32) {
        const int pk = sc->p[k], qk = sc->q[k];
        const float sk = sc->s[k], tk = sc->t[k];
        for (int l = tid & 31; l < half; l += 32) {
          const int pl = sc->p[l], ql = sc->q[l];
          const float sl = sc->s[l], tl = sc->t[l];
          if (sk == 0.f && sl == 0.f) continue;
          float a = As[pk * LD + pl], b = As[pk * LD + ql];
          float c = As[qk * LD + pl], d = As[qk * LD + ql];
          // rows: (a, c) and (b, d) are (x, y) pairs of rotation k
          float a1 = a - sk * (c + tk * a), c1 = c + sk * (a - tk * c);
          float b1 = b - sk * (d + tk * b), d1 = d + sk * (b - tk * d);
          // columns: (a1, b1) and (c1, d1) are (x, y) pairs of rotation l
          a = a1 - sl * (b1 + tl * a1); b = b1 + sl * (a1 - tl * b1);
          c = c1 - sl * (d1 + tl * c1); d = d1 + sl * (c1 - tl * d1);
          if (k == l) { b = 0.f; c = 0.f; }   // the annihilated pivot element
          As[pk * LD + pl] = a; As[pk * LD + ql] = b;
          As[qk * LD + pl] = c; As[qk * LD + ql] = d;
        }
      }
      // J <- J R (columns)
      for (int i = tid >> 5; i < s; i += JAC_THREADS / 32) {
        for (int l = tid & 31; l < half; l += 32) {
          const float sl = sc->s[l];
          if (sl == 0.f) continue;
          const float tl = sc->t[l];
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
  const int SMALL_LD = s + 1;
  float *As = reinterpret_cast<float *>(smem);
  float *Js = As + s * SMALL_LD;
  float *fv = Js + s * SMALL_LD;            // [s]
  const float *a = g.a + (int64_t)b * g.a_stride;

  int bad = 0;
  float dmax = 0.f;
  for (int i = tid >> 6; i < s; i += JAC_THREADS / 64)
    for (int j = lane; j < s; j += 64) {
      float v = 0.f;
      if (i < n && j < n) {
        v = a[(int64_t)i * n + j];
        if (!(fabsf(v) <= 3.0e38f)) bad = 1;
        if (i == j) dmax = fmaxf(dmax, fabsf(v));
      }
      As[i * SMALL_LD + j] = v;
      Js[i * SMALL_LD + j] = (i == j) ? 1.f : 0.f;
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
  // symmetrise (a no-op for exactly symmetric input)
  for (int i = tid >> 6; i < s; i += JAC_THREADS / 64)
    for (int j = lane; j < i; j += 64) {
      const float v = 0.5f * (As[i * SMALL_LD + j] + As[j * SMALL_LD + i]);
      As[i * SMALL_LD + j] = v;
      As[j * SMALL_LD + i] = v;
    }
  __syncthreads();

  jacobi_sweeps(As, Js, s, SMALL_LD, JAC_SMALL_SWEEPS, JAC_TOL_ABS * dmax, sc);
  __syncthreads();

  // lambda_min over the true eigenvalues, then f = (lambda - min(lambda_min, 0) + eps)^-r
  float lmin = 3.0e38f;
  for (int i = tid; i < n; i += JAC_THREADS) lmin = fminf(lmin, As[i * SMALL_LD + i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) lmin = fminf(lmin, __shfl_xor(lmin, off, 64));
  if (lane == 0) redf[wave] = lmin;
  __syncthreads();
  lmin = fminf(fminf(redf[0], redf[1]), fminf(redf[2], redf[3]));
  const float shift = fminf(lmin, 0.f);
  int badf = 0;
  for (int i = tid; i < s; i += JAC_THREADS) {
    float f = 0.f;
    if (i < n) {
      const float lam = As[i * SMALL_LD + i];
      const double ln = (double)(lam - shift) + (double)g.epsilon;
      f = (float)pow(ln, -(double)g.r);
      if (!(f <= 3.0e38f) || !(f >= 0.f)) badf = 1;
      if (g.lambda) g.lambda[(int64_t)b * n + i] = lam;
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
    for (int k = lane; k < s; k += 64) Js[i * SMALL_LD + k] *= fv[k];
  __syncthreads();
  float *x = g.x + (int64_t)b * g.x_stride;
  for (int i = tid >> 6; i < n; i += JAC_THREADS / 64)
    for (int j = lane; j <= i; j += 64) {
      float acc = 0.f;
      for (int k = 0; k < n; ++k) acc += Js[i * SMALL_LD + k] * Js[j * SMALL_LD + k];
      x[(int64_t)i * n + j] = acc;
      x[(int64_t)j * n + i] = acc;
    }
}

inline size_t rootinv_small_lds_bytes(int n) {
  const int s = (n + 1) & ~1;
  return (size_t)(2 * s * (s + 1) + s) * sizeof(float);
}

// ---------------------------------------------------------------------------
// n > 128: block Jacobi.  Work arrays per matrix (np = n rounded up to 64):
//   W  [np][np]  the matrix being diagonalised (padding: zero, decoupled)
//   Qt [np][np]  accumulated rotations, transposed (rows are eigenvectors)
//   J  [np/64][64][64] rotation blocks of the current round
// ---------------------------------------------------------------------------
struct BlockJacArgs {
  float *w;
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
  float *w; float *qt; int32_t np;
  float *dmax; int32_t *failed; int32_t *rot;
};

// W = pad(A), Qt = I, dmax, failed, rot = 0.  grid (np, batch), 256 threads.
__global__ __launch_bounds__(256) void blockjac_init_kernel(const BlockInitArgs g) {
  const int b = blockIdx.y, i = blockIdx.x, np = g.np, n = g.n;
  float *w = g.w + (int64_t)b * np * np + (int64_t)i * np;
  float *qt = g.qt + (int64_t)b * np * np + (int64_t)i * np;
  const float *a = g.a + (int64_t)b * g.a_stride + (int64_t)i * n;
  int bad = 0;
  for (int j = threadIdx.x; j < np; j += 256) {
    float v = 0.f;
    if (i < n && j < n) {
      v = a[j];
      if (!(fabsf(v) <= 3.0e38f)) bad = 1;
    }
    w[j] = v;
    qt[j] = (i == j) ? 1.f : 0.f;
  }
  if (bad) g.failed[b] = 1;
  if (i < n && threadIdx.x == 0) {
    const float d = fabsf(a[i]);
    if (d <= 3.0e38f) atomicMax(reinterpret_cast<int *>(g.dmax + b), __float_as_int(d));  // d >= 0: int order = float order
  }
  if (i == 0 && threadIdx.x < JAC_OUTER_SWEEPS) g.rot[b * JAC_OUTER_SWEEPS + threadIdx.x] = 0;
}

constexpr int PIV_LD = JAC_PIV + 1;

// One workgroup per (pair, matrix): diagonalise the 64 x 64 pivot.
__global__ __launch_bounds__(JAC_THREADS) void blockjac_pivot_kernel(const BlockJacArgs g) {
  __shared__ float As[JAC_PIV * PIV_LD];
  __shared__ float Js[JAC_PIV * PIV_LD];
  __shared__ JacScratch sc;
  const int b = blockIdx.y, pair = blockIdx.x;
  if (g.failed[b]) return;
  if (g.sweep > 0 && g.rot[b * JAC_OUTER_SWEEPS + g.sweep - 1] == 0) return;   // converged
  const int np = g.np, nblk = np / JAC_NB;
  int pb, qb;
  rr_pair(nblk, g.round, pair, pb, qb);
  const float *w = g.w + (int64_t)b * np * np;
  const int tid = threadIdx.x;
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64) {
    const int j = tid & 63;
    const int gi = (i < JAC_NB ? pb * JAC_NB + i : qb * JAC_NB + i - JAC_NB);
    const int gj = (j < JAC_NB ? pb * JAC_NB + j : qb * JAC_NB + j - JAC_NB);
    As[i * PIV_LD + j] = w[(int64_t)gi * np + gj];
    Js[i * PIV_LD + j] = (i == j) ? 1.f : 0.f;
  }
  __syncthreads();
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64) {
    const int j = tid & 63;
    if (j < i) {
      const float v = 0.5f * (As[i * PIV_LD + j] + As[j * PIV_LD + i]);
      As[i * PIV_LD + j] = v;
      As[j * PIV_LD + i] = v;
    }
  }
  __syncthreads();
  const int any = jacobi_sweeps(As, Js, JAC_PIV, PIV_LD, JAC_INNER_SWEEPS, JAC_TOL_ABS * g.dmax[b], &sc);
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

// 64 x 64 x 64 product on one workgroup: wavefront (wi, wj) computes the 32 x 32
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

// Applies the round's rotations.  blockIdx.x < hp*hp: A_kl <- J_k^T A_kl J_l for
// the pair-block (k, l); otherwise Qt rows of pair k, one 64-column tile.
__global__ __launch_bounds__(JAC_THREADS, 2) void blockjac_apply_kernel(const BlockJacArgs g) {
  __shared__ __align__(16) float Jk[JAC_PIV * APP_LD];
  __shared__ __align__(16) float Jl[JAC_PIV * APP_LD];
  __shared__ __align__(16) float X[JAC_PIV * APP_LD];
  __shared__ __align__(16) float Tt[JAC_PIV * APP_LD];
  const int b = blockIdx.y;
  if (g.failed[b]) return;
  if (g.sweep > 0 && g.rot[b * JAC_OUTER_SWEEPS + g.sweep - 1] == 0) return;
  const int np = g.np, nblk = np / JAC_NB, hp = nblk / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int32_t *ident = g.ident + b * hp;
  const float *jb = g.jbuf + (int64_t)b * hp * JAC_PIV * JAC_PIV;

  const bool two_sided = (int)blockIdx.x < hp * hp;
  int k, l = 0, ctile = 0;
  float *mat;
  if (two_sided) {
    k = blockIdx.x / hp; l = blockIdx.x - k * hp;
    if (ident[k] && ident[l]) return;
    mat = g.w + (int64_t)b * np * np;
  } else {
    const int rest = blockIdx.x - hp * hp;
    const int ctiles = np / JAC_PIV;
    k = rest / ctiles; ctile = rest - k * ctiles;
    if (ident[k]) return;
    mat = g.qt + (int64_t)b * np * np;
  }
  int pk, qk, pl = 0, ql = 0;
  rr_pair(nblk, g.round, k, pk, qk);
  if (two_sided) rr_pair(nblk, g.round, l, pl, ql);

  // global row / column of local index (one 64-float row per 64 consecutive threads)
  const int c = tid & 63;
  const int gcol = two_sided ? (c < JAC_NB ? pl * JAC_NB + c : ql * JAC_NB + c - JAC_NB) : ctile * JAC_PIV + c;
  const bool idk = ident[k] != 0;
  const bool idl = two_sided ? (ident[l] != 0) : true;
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_THREADS / 64) {
    const int grow = (i < JAC_NB ? pk * JAC_NB + i : qk * JAC_NB + i - JAC_NB);
    X[i * APP_LD + c] = mat[(int64_t)grow * np + gcol];
    Jk[i * APP_LD + c] = idk ? (i == c ? 1.f : 0.f) : jb[((int64_t)k * JAC_PIV + i) * JAC_PIV + c];
    if (two_sided) Jl[i * APP_LD + c] = idl ? (i == c ? 1.f : 0.f) : jb[((int64_t)l * JAC_PIV + i) * JAC_PIV + c];
  }
  __syncthreads();
  // T = J_k^T X
  floatx16 acc = mfma_64(Jk, X, wi, wj, lane);
  const int j = wj * 32 + (lane & 31);
  if (two_sided) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i0 = wi * 32 + 8 * q + 4 * (lane >> 5);
      *reinterpret_cast<float4 *>(&Tt[j * APP_LD + i0]) =
          make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    }
    __syncthreads();
    // C = T J_l   (A-operand (i, k) = Tt[k][i])
    acc = mfma_64(Tt, Jl, wi, wj, lane);
  }
  const int gc = two_sided ? (j < JAC_NB ? pl * JAC_NB + j : ql * JAC_NB + j - JAC_NB) : ctile * JAC_PIV + j;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = wi * 32 + 8 * q + 4 * (lane >> 5) + e;
      const int grow = (i < JAC_NB ? pk * JAC_NB + i : qk * JAC_NB + i - JAC_NB);
      mat[(int64_t)grow * np + gc] = acc[4 * q + e];
    }
}

struct BlockFinalArgs {
  const float *w; int32_t np; int32_t n;
  float epsilon, r;
  float *fvals;          // [batch][np]: lambda'^-r (0 on padding)
  float *lambda;         // optional [batch][n]
  int32_t *failed;       // [batch] in/out
  int32_t *failed_out;   // optional user-visible copy
  unsigned long long *fail_count;
};

// One workgroup per matrix: eigenvalues = diag(W); shift; f(lambda).
__global__ __launch_bounds__(256) void blockjac_final_kernel(const BlockFinalArgs g) {
  __shared__ float redf[4];
  __shared__ int redi[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int np = g.np, n = g.n;
  const float *w = g.w + (int64_t)b * np * np;
  float *fv = g.fvals + (int64_t)b * np;
  int bad = g.failed[b];
  float lmin = 3.0e38f;
  if (!bad)
    for (int i = tid; i < n; i += 256) lmin = fminf(lmin, w[(int64_t)i * np + i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) lmin = fminf(lmin, __shfl_xor(lmin, off, 64));
  if (lane == 0) redf[wave] = lmin;
  __syncthreads();
  lmin = fminf(fminf(redf[0], redf[1]), fminf(redf[2], redf[3]));
  const float shift = fminf(lmin, 0.f);
  int badf = bad;
  for (int i = tid; i < np; i += 256) {
    float f = 0.f;
    if (i < n && !bad) {
      const float lam = w[(int64_t)i * np + i];
      const double ln = (double)(lam - shift) + (double)g.epsilon;
      f = (float)pow(ln, -(double)g.r);
      if (!(f <= 3.0e38f) || !(f >= 0.f)) badf = 1;
      if (g.lambda) g.lambda[(int64_t)b * n + i] = lam;
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
