// W = Q^T A Q in float64 from float32 operands, between the float32 and the float64 sweeps of
// the blocked eigensolver and (rounded to float32 at the end) for its warm start (Sec. 3.2.1: the root inverse by symmetric eigendecomposition is recomputed every
// precondition_frequency steps from a factor that has changed little; the eigenvectors of the
// previous refresh then nearly diagonalise the new factor).  With Qt = Q^T (rows are the
// previous eigenvectors, float32) and the new factor A (float32):
//     T = A Qt^T   (float64, a panel of columns at a time)
//     W = Qt T     (float64; only what the solver keeps: the 32 x 32 sub-blocks on and below
//                   the diagonal, the diagonal ones completed to exact symmetry)
// Products of two float32 values are exact in float64, so W is the exact congruence of A by
// the float32 matrix Qt up to the rounding of the float64 sums: whatever Qt lacks in
// orthogonality (1e-6 after a solve) moves every eigenvalue of A by that relative amount only.
//
// One kernel does both products: C (float64) = A (float32, k contiguous) * B, where B is either
// float32 given by rows along k (B(k, j) = b[j * ldb + k]: the rows of Qt) or float64 given by
// rows along j (B(k, j) = b[k * ldb + j]: the panel T).  Tile 128 x 128 per workgroup of four
// wavefronts; wavefront w owns rows 32 w .. 32 w + 31 as 2 x 8 tiles of v_mfma_f64_16x16x4_f64
// (lane l supplies A(l % 16, l / 16) and B(l / 16, l % 16); element v of the result is
// D(l / 16 + 4 v, l % 16)).  Operands go through LDS in slabs of 16 k (float32 operands are
// kept as float32 there and widened when read); the next slab is fetched into registers while
// the current one is multiplied.  Shapes are arbitrary: loads are scalar with zero fill.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "eigh_jacobi.h"      // w32_index: where the float32 copy of W keeps element (i, j)

namespace shampoo {

typedef double cg_doublex4 __attribute__((ext_vector_type(4)));

constexpr int CG_TILE = 128;
constexpr int CG_KS = 16;              // k per slab
constexpr int CG_THREADS = 256;
constexpr int CG_LDF = CG_KS + 1;      // float32 operand rows in LDS: [row][k], odd stride
constexpr int CG_LDD = CG_TILE + 2;    // float64 B slab: [k][j]

struct CongruenceArgs {
  const float *a; int64_t a_batch; int32_t lda;     // A operand: M x K, element (i, k) at a[i * lda + k]
  const void *b; int64_t b_batch; int32_t ldb;      // B operand, see BF64
  double *c; int64_t c_batch; int32_t ldc;          // C: M x N, row-major
  int32_t M, N, K;
  int32_t col0;             // LOWER: column of C (and of W) at which this panel starts
  const int32_t *skip;      // optional [batch]: nonzero entries are left alone
};

// BF64: B is float64 [K][N] (rows along j); else float32 [N][K] (rows along k).
// LOWER: C is the solver's W: only tiles that reach the diagonal or lie below it are computed,
// elements above the diagonal are not stored, except inside the 32 x 32 sub-blocks on the diagonal,
// which receive the mirror image of their lower half (exactly symmetric).
// OUT32 (with LOWER): the result is rounded to float32 and goes into the solver's float32 copy of
// W (c is that array, c_batch counts floats, ldc = np), sub-blocks contiguous.
template <bool BF64, bool LOWER, bool OUT32 = false>
__global__ __launch_bounds__(CG_THREADS, 1) void congruence_gemm_kernel(const CongruenceArgs g) {
  __shared__ float As[CG_TILE * CG_LDF];
  __shared__ __align__(16) unsigned char Bs_raw[BF64 ? CG_KS * CG_LDD * 8 : CG_TILE * CG_LDF * 4];
  float *Bf = reinterpret_cast<float *>(Bs_raw);
  double *Bd = reinterpret_cast<double *>(Bs_raw);
  const int bz = blockIdx.z;
  if (g.skip && g.skip[bz]) return;
  const int row0 = blockIdx.y * CG_TILE, colt = blockIdx.x * CG_TILE;   // tile origin inside C
  if (LOWER && row0 + CG_TILE <= g.col0 + colt) return;                 // entirely above the diagonal
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const float *a = g.a + (int64_t)bz * g.a_batch;
  const float *bf = reinterpret_cast<const float *>(g.b) + (int64_t)bz * g.b_batch;
  const double *bd = reinterpret_cast<const double *>(g.b) + (int64_t)bz * g.b_batch;
  double *c = g.c + (int64_t)bz * g.c_batch;

  cg_doublex4 acc[2][8];
#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[r][t] = (cg_doublex4){0.0, 0.0, 0.0, 0.0};

  // slab fetch: thread -> (row = tid / 2 + 0, k half = tid % 2): 8 consecutive k of one row, for A
  // and for a float32 B alike; a float64 B slab is [16][128]: thread -> (k = tid / 16, 8 columns)
  const int fr = tid >> 1, fk = (tid & 1) * 8;
  float pa[8], pbf[8];
  double pbd[8];
  auto fetch = [&](int k0) {
    const int i = row0 + fr;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = k0 + fk + e;
      pa[e] = (i < g.M && k < g.K) ? a[(int64_t)i * g.lda + k] : 0.f;
    }
    if (BF64) {
      const int k = k0 + (tid >> 4), j0 = colt + (tid & 15) * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) pbd[e] = (k < g.K && j0 + e < g.N) ? bd[(int64_t)k * g.ldb + j0 + e] : 0.0;
    } else {
      const int j = colt + fr;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int k = k0 + fk + e;
        pbf[e] = (j < g.N && k < g.K) ? bf[(int64_t)j * g.ldb + k] : 0.f;
      }
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int e = 0; e < 8; ++e) As[fr * CG_LDF + fk + e] = pa[e];
    if (BF64) {
#pragma unroll
      for (int e = 0; e < 8; ++e) Bd[(tid >> 4) * CG_LDD + (tid & 15) * 8 + e] = pbd[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) Bf[fr * CG_LDF + fk + e] = pbf[e];
    }
  };

  fetch(0);
  for (int k0 = 0; k0 < g.K; k0 += CG_KS) {
    __syncthreads();                 // everyone is done with the slab before
    stash();
    __syncthreads();
    if (k0 + CG_KS < g.K) fetch(k0 + CG_KS);
#pragma unroll
    for (int s = 0; s < CG_KS / 4; ++s) {
      const double a0 = (double)As[(32 * wave + li) * CG_LDF + 4 * s + lg];
      const double a1 = (double)As[(32 * wave + 16 + li) * CG_LDF + 4 * s + lg];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        double bv;
        if (BF64) bv = Bd[(4 * s + lg) * CG_LDD + 16 * t + li];
        else bv = (double)Bf[(16 * t + li) * CG_LDF + 4 * s + lg];
        acc[0][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, bv, acc[0][t], 0, 0, 0);
        acc[1][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, bv, acc[1][t], 0, 0, 0);
      }
    }
  }

#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int i = row0 + 32 * wave + 16 * r + lg + 4 * v;
        const int jl = colt + 16 * t + li;          // column inside the panel
        if (i >= g.M || jl >= g.N) continue;
        const double x = acc[r][t][v];
        if (!LOWER) { c[(int64_t)i * g.ldc + jl] = x; continue; }
        const int j = g.col0 + jl;                  // column inside W
        if (j > i) continue;
        if (OUT32) {
          float *cf = reinterpret_cast<float *>(g.c) + (int64_t)bz * g.c_batch;
          const int nblk = g.ldc / JAC_NB;
          cf[w32_index(i, j, nblk)] = (float)x;
          if ((i >> 5) == (j >> 5) && j < i) cf[w32_index(j, i, nblk)] = (float)x;
          continue;
        }
        c[(int64_t)i * g.ldc + j] = x;
        if ((i >> 5) == (j >> 5) && j < i) c[(int64_t)j * g.ldc + i] = x;
      }
}

}  // namespace shampoo
