// Factor update for bf16 gradients on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// The product of two bf16 values is exact in float32, so G G^T of a bf16 gradient
// loses nothing on the bf16 MFMA path (16x the float32 MFMA rate) provided the
// accumulation is as careful as on the float32 path: here two chained MFMAs (32
// values of k) are accumulated in float32 and then added into float64 registers,
// and beta2 L + (1 - beta2) S is evaluated in float64 before the single rounding
// to float32.  R = G^T G runs through the same kernel on a bf16 transpose of the
// block (transpose_bf16_kernel), so both operands are always read along k.
//
// Tile 128 x 128 per workgroup of 4 wavefronts (64 x 64 each, 2 x 2 MFMA tiles);
// operand tiles are staged in LDS as [row][k] with 32 values of k per slab (rows
// padded to 80 bytes), double-buffered.  An MFMA operand is 8 consecutive k of one
// row per lane: lane = row % 32 + 32 * (k / 8).  Only lower-triangular tiles are
// computed; the mirror image is written with the same bits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"

namespace shampoo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

#ifndef SHAMPOO_SYRK_CHAIN
#define SHAMPOO_SYRK_CHAIN 2
#endif
constexpr int SCH = SHAMPOO_SYRK_CHAIN;   // MFMAs (16 k each) chained in float32 before the float64 flush
constexpr int SBK = 16 * SCH;             // k per slab
constexpr int SLD = SBK + 8;     // LDS row stride, bf16 elements

struct SyrkBf16Args {
  Operand a;                 // bf16 matrix X (rows x K, k contiguous); C = beta C + alpha X X^T
  const BlockDesc *desc;
  const void *const *ptr_table;
  float *c; int64_t c_batch_stride; int32_t ldc;
  int32_t M, K;              // C is M x M
  double alpha, beta;
  int32_t tiles;             // lower-triangular tile count per batch entry
  int32_t batch;
};

// Requires: operand base 16-byte aligned, ld % 8 == 0 (checked by the host).
__global__ __launch_bounds__(GEMM_THREADS, 2) void syrk_bf16_kernel(const SyrkBf16Args g) {
  // one LDS region: the operand slabs during the k loop, then the tile on its way to the
  // mirrored (transposed) position
  constexpr int SYRK_TLD = BM + 1;
  constexpr int SLAB_BYTES = 2 * BM * SLD * 2;
  constexpr int LDS_BYTES = BN * SYRK_TLD * 4 > 2 * SLAB_BYTES ? BN * SYRK_TLD * 4 : 2 * SLAB_BYTES;
  __shared__ __align__(16) unsigned char smem[LDS_BYTES];
  uint16_t (*As)[BM][SLD] = reinterpret_cast<uint16_t (*)[BM][SLD]>(smem);
  uint16_t (*Bs)[BN][SLD] = reinterpret_cast<uint16_t (*)[BN][SLD]>(smem + SLAB_BYTES);
  float *Ts = reinterpret_cast<float *>(smem);
  const int total = g.tiles * g.batch;
  const int logical = xcd_remap(blockIdx.x, total);
  if (logical >= total) return;
  const int b = logical / g.tiles;
  const int tile = logical - b * g.tiles;
  int ti = (int)((sqrtf(8.f * (float)tile + 1.f) - 1.f) * 0.5f);
  while ((ti + 1) * (ti + 2) / 2 <= tile) ++ti;
  while (ti * (ti + 1) / 2 > tile) --ti;
  const int tj = tile - ti * (ti + 1) / 2;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = ti * BM, col0 = tj * BN;
  int ld;
  const uint16_t *x = operand_ptr<uint16_t>(g.a, g.desc, g.ptr_table, b, ld);
  const uint16_t *xa = x + (int64_t)row0 * ld;
  const uint16_t *xb = x + (int64_t)col0 * ld;
  const int rows_a = g.M - row0, rows_b = g.M - col0;

  // thread (r, kc): rows r + SRPP * h, 8 consecutive k starting at kc
  constexpr int SCPR = SBK / 8, SRPP = GEMM_THREADS / SCPR, SPASS = BM / SRPP;
  const int r = tid / SCPR, kc = (tid % SCPR) * 8;
  uint4 ra[SPASS], rb[SPASS];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int h = 0; h < SPASS; ++h) {
      const int rr = r + SRPP * h;
      const bool kin = k0 + kc < g.K;     // K % 8 == 0: a chunk is entirely in or out
      ra[h] = (rr < rows_a && kin) ? *reinterpret_cast<const uint4 *>(xa + (int64_t)rr * ld + k0 + kc) : make_uint4(0, 0, 0, 0);
      rb[h] = (rr < rows_b && kin) ? *reinterpret_cast<const uint4 *>(xb + (int64_t)rr * ld + k0 + kc) : make_uint4(0, 0, 0, 0);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int h = 0; h < SPASS; ++h) {
      *reinterpret_cast<uint4 *>(&As[buf][r + SRPP * h][kc]) = ra[h];
      *reinterpret_cast<uint4 *>(&Bs[buf][r + SRPP * h][kc]) = rb[h];
    }
  };

  double acc64[2][2][16];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc64[i][j][v] = 0.0;
  floatx16 zero;
#pragma unroll
  for (int v = 0; v < 16; ++v) zero[v] = 0.f;

  const int nk = (g.K + SBK - 1) / SBK;
  fetch(0);
  stash(0);
  __syncthreads();
  const int fi = lane & 31, fk = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) fetch((kt + 1) * SBK);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        floatx16 acc = zero;
#pragma unroll
        for (int s = 0; s < SCH; ++s) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&As[cur][wm * 64 + i * 32 + fi][s * 16 + fk]));
          const bf16x8 bb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&Bs[cur][wn * 64 + j * 32 + fi][s * 16 + fk]));
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc64[i][j][v] += (double)acc[v];
      }
    if (kt + 1 < nk) stash(cur ^ 1);
    __syncthreads();
  }

  // Epilogue.  The lower-triangular tile is stored from the accumulators (rows of 32
  // consecutive floats per half wavefront).  Its mirror image would be a scatter of single
  // floats, so the tile goes through LDS transposed and is stored along rows as well; a
  // diagonal tile is completed to the full symmetric tile in LDS and stored once.  Both
  // copies carry the same bits, so the factor stays exactly symmetric.
  float *c = g.c + (int64_t)b * g.c_batch_stride;
  const int ldc = g.ldc;
  const bool diag = ti == tj;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int jl = wn * 64 + ni * 32 + (lane & 31), j = col0 + jl;
      float old[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = row0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        old[v] = (g.beta != 0.0 && i < g.M && j <= i) ? c[(int64_t)i * ldc + j] : 0.f;
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int il = wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), i = row0 + il;
        const float x = (float)(g.alpha * acc64[mi][ni][v] + g.beta * (double)old[v]);
        if (diag) {
          if (jl <= il) { Ts[il * SYRK_TLD + jl] = x; Ts[jl * SYRK_TLD + il] = x; }
        } else {
          Ts[jl * SYRK_TLD + il] = x;
          if (i < g.M && j < g.M) c[(int64_t)i * ldc + j] = x;
        }
      }
    }
  __syncthreads();
  {
    // rows of the LDS tile -> rows of C at (col0, row0) (or (row0, row0) for a diagonal tile)
    const int rbase = diag ? row0 : col0, cbase = row0;
    const int cx = (tid & 31) * 4;
    const bool vec = (ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(c) & 15) == 0;
    for (int rr = tid >> 5; rr < BM; rr += GEMM_THREADS / 32) {
      const int gi = rbase + rr, gj = cbase + cx;
      if (gi >= g.M || gj >= g.M) continue;
      const float *src = Ts + rr * SYRK_TLD + cx;
      if (vec && gj + 3 < g.M) {
        *reinterpret_cast<float4 *>(c + (int64_t)gi * ldc + gj) = make_float4(src[0], src[1], src[2], src[3]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) if (gj + e < g.M) c[(int64_t)gi * ldc + gj + e] = src[e];
      }
    }
  }
}

struct TransposeArgs {
  const BlockDesc *desc;
  const void *const *g_table;
  uint16_t *out;             // [slot][n][m]
  int32_t m, n;
};

// out[slot][j][i] = G_block[i][j] (bf16 bits).  grid (ceil(n/64), ceil(m/64), blocks), 256 threads.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const TransposeArgs g) {
  __shared__ uint16_t tile[64][66];
  const BlockDesc d = g.desc[blockIdx.z];
  const uint16_t *src = reinterpret_cast<const uint16_t *>(g.g_table[d.param]) + d.offset;
  uint16_t *dst = g.out + (int64_t)blockIdx.z * g.m * g.n;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int ii = ty; ii < 64; ii += 4) {
    const int i = i0 + ii, j = j0 + tx;
    tile[ii][tx] = (i < g.m && j < g.n) ? src[(int64_t)i * d.ld + j] : (uint16_t)0;
  }
  __syncthreads();
  for (int jj = ty; jj < 64; jj += 4) {
    const int j = j0 + jj, i = i0 + tx;
    if (j < g.n && i < g.m) dst[(int64_t)j * g.m + i] = tile[tx][jj];
  }
}

}  // namespace shampoo
