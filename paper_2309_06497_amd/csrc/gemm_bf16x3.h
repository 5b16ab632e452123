// float32-accurate batched GEMM on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// A float32 value x splits exactly into three bf16 values, x = h + m + l with
// h = bf16(x), m = bf16(x - h), l = bf16(x - h - m) (8 significant bits each; the
// subtractions are exact).  The product of two bf16 values is exact in float32, so
//   a b = ah bh + (ah bm + am bh) + (ah bl + al bh + am bm) + O(2^-24 |a b|)
// and a float32 GEMM becomes six bf16 MFMA products accumulated in float32: what is
// dropped is below the rounding of a single float32 product.  An operand that is
// already bf16 (the gradient) is one exact term, which leaves three products.  The
// bf16 matrix cores run 16x faster than the float32 ones, so six products cost 3/8 of
// the float32-MFMA time (three: 3/16), with the same float32 accumulation as there.
//
// Operands are kept split in memory, as three (or one) bf16 planes, so the split is paid
// once per value and not once per tile that reads it: the roots are split after each
// refresh (split3_kernel), and the first product of the preconditioning step writes its
// result T directly as three planes.  C[i][j] = alpha * sum_k A[i][k] * B[j][k]: both
// operands are read along k (row-major A; B given transposed, or symmetric).  The two
// products of Sec. 2.3 of the paper have that form:
//   T = Lbar G       A = Lbar (three planes)   B = G^T (the bf16 transpose of the block, one plane)
//   P = T Rbar       A = T (three planes)      B = Rbar (symmetric, three planes)
// Tile 128 x 128 per workgroup of 4 wavefronts (64 x 64 each, 2 x 2 MFMA tiles); operand
// slabs of 32 values of k (64 for the first product) are staged in LDS as [plane][row][k]
// (rows padded by 16 bytes; 60 KB for 3 + 3 planes, two workgroups per CU); the global loads
// of the next slab are in flight while the current one is multiplied.  An MFMA operand is 8 consecutive k of one row per lane:
// lane = row % 32 + 32 * (k / 8).
// Requires K % 8 == 0, leading dimensions % 8 == 0 and 16-byte aligned operands (the host
// checks, and otherwise uses the float32-MFMA kernel).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"
#include "syrk_bf16.h"

namespace shampoo {

#ifndef SHAMPOO_X3_BK1
#define SHAMPOO_X3_BK1 64
#endif
#ifndef SHAMPOO_X3_BK2
#define SHAMPOO_X3_BK2 32
#endif
constexpr int X3_BK_FIRST = SHAMPOO_X3_BK1;    // k per slab of T = Lbar G (3 + 1 planes)
constexpr int X3_BK_SECOND = SHAMPOO_X3_BK2;   // k per slab of P = T Rbar (3 + 3 planes)

enum { X3_STORE_NORM = 0, X3_STORE_SPLIT = 1 };

struct GemmX3Args {
  const uint16_t *a; int64_t a_plane_stride, a_batch_stride; int32_t lda;   // [plane][batch][M][K]
  const uint16_t *b; int64_t b_plane_stride, b_batch_stride; int32_t ldb;   // [plane][batch][N][K]
  float *c;                // X3_STORE_NORM: [batch][M][N] float32
  uint16_t *c3;            // X3_STORE_SPLIT: [plane][batch][M][N] bf16
  int64_t c3_plane_stride;
  int64_t c_batch_stride; int32_t ldc;
  int32_t M, N, K;
  float alpha;
  float *norm_partial;     // X3_STORE_NORM: [batch][tiles] sums of squares of the stored tile
  int32_t tiles_m, tiles_n, batch;
};

// round-to-nearest-even float32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// x = h + m + l exactly (up to underflow), each a bf16
__device__ __forceinline__ void split3(float x, uint32_t &h, uint32_t &m, uint32_t &l) {
  h = f32_to_bf16_rne(x);
  const float r1 = x - __uint_as_float(h << 16);
  m = f32_to_bf16_rne(r1);
  const float r2 = r1 - __uint_as_float(m << 16);
  l = f32_to_bf16_rne(r2);
}

// out[plane][i] = the three bf16 terms of in[i]
__global__ __launch_bounds__(256) void split3_kernel(const float *in, uint16_t *out, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  uint32_t h, m, l;
  split3(in[i], h, m, l);
  out[i] = (uint16_t)h; out[count + i] = (uint16_t)m; out[2 * count + i] = (uint16_t)l;
}

// XBK: k per slab (16, 32 or 64)
template <int NA, int NB, int EPI, int XBK>
__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_bf16x3_kernel(const GemmX3Args g) {
  constexpr int XLD = XBK + 8;                // LDS row stride, bf16 elements (an odd number of 16-byte units)
  constexpr int XCPR = XBK / 8;               // 16-byte chunks per row of a slab
  constexpr int XRPP = GEMM_THREADS / XCPR;   // rows per pass of the loader
  constexpr int XPASS = BM / XRPP;
  __shared__ __align__(16) uint16_t As[NA][BM][XLD];
  __shared__ __align__(16) uint16_t Bs[NB][BN][XLD];
  __shared__ float red[4];
  const int tiles = g.tiles_m * g.tiles_n;
  const int total = tiles * g.batch;
  const int logical = xcd_remap(blockIdx.x, total);
  if (logical >= total) return;
  const int b = logical / tiles;
  const int tile = logical - b * tiles;
  const int ti = tile / g.tiles_n, tj = tile - ti * g.tiles_n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = ti * BM, col0 = tj * BN;
  // thread (r, kc): rows r + XRPP * h of the tile, 8 consecutive k starting at kc, every plane
  const int r = tid / XCPR, kc = (tid % XCPR) * 8;
  const uint16_t *pa = g.a + (int64_t)b * g.a_batch_stride + (int64_t)(row0 + r) * g.lda + kc;
  const uint16_t *pb = g.b + (int64_t)b * g.b_batch_stride + (int64_t)(col0 + r) * g.ldb + kc;
  // The slab after the one being multiplied is already on its way into registers; it is
  // written to LDS once every wavefront has finished reading the current one.  (Measured on
  // the 1024-blocks, both products together: slabs of 32 in one LDS buffer 20.3 ms; slabs of
  // 16 double-buffered 25.4; slabs of 32 double-buffered, one workgroup per CU, 28.9; loads
  // two slabs ahead 21.9; 8 wavefronts of which 4 only move operands and 4 only multiply,
  // double-buffered, 25.5; the same with the LDS reads of the next 16 k issued ahead of the
  // MFMAs, 26.9.  With real roots instead of identities every variant is ~25 % slower: the
  // same instruction stream on denser data, i.e. the clocks give way.)
  uint4 ra[XPASS][NA], rb[XPASS][NB];
  auto fetch = [&](int k0) {
    const bool kin = k0 + kc < g.K;     // K % 8 == 0: a chunk is entirely in or out
#pragma unroll
    for (int h = 0; h < XPASS; ++h) {
      const bool a_in = row0 + r + XRPP * h < g.M && kin, b_in = col0 + r + XRPP * h < g.N && kin;
#pragma unroll
      for (int s = 0; s < NA; ++s)
        ra[h][s] = a_in ? *reinterpret_cast<const uint4 *>(pa + s * g.a_plane_stride + (int64_t)XRPP * h * g.lda + k0)
                        : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int s = 0; s < NB; ++s)
        rb[h][s] = b_in ? *reinterpret_cast<const uint4 *>(pb + s * g.b_plane_stride + (int64_t)XRPP * h * g.ldb + k0)
                        : make_uint4(0, 0, 0, 0);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int h = 0; h < XPASS; ++h) {
#pragma unroll
      for (int s = 0; s < NA; ++s) *reinterpret_cast<uint4 *>(&As[s][r + XRPP * h][kc]) = ra[h][s];
#pragma unroll
      for (int s = 0; s < NB; ++s) *reinterpret_cast<uint4 *>(&Bs[s][r + XRPP * h][kc]) = rb[h][s];
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = (g.K + XBK - 1) / XBK;
  fetch(0);
  stash();
  __syncthreads();
  const int fi = lane & 31, fk = (lane >> 5) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) fetch((kt + 1) * XBK);
#pragma unroll
    for (int ks = 0; ks < XBK; ks += 16) {
      bf16x8 a[NA][2], bb[NB][2];   // [plane][tile]
#pragma unroll
      for (int s = 0; s < NA; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          a[s][t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&As[s][wm * 64 + t * 32 + fi][ks + fk]));
#pragma unroll
      for (int s = 0; s < NB; ++s)
#pragma unroll
        for (int t = 0; t < 2; ++t)
          bb[s][t] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(&Bs[s][wn * 64 + t * 32 + fi][ks + fk]));
      // plane pairs (s, u) with s + u <= 2, smallest contributions first
#pragma unroll
      for (int order = 2; order >= 0; --order)
#pragma unroll
        for (int s = 0; s < NA; ++s) {
          const int u = order - s;
          if (u < 0 || u >= NB) continue;
#pragma unroll
          for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s][i], bb[u][j], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();   // every wavefront has read the slab before it is overwritten
    if (kt + 1 < nk) stash();
    __syncthreads();
  }

  // epilogue: accumulator element v of MFMA tile (mi, ni) is
  // row = wm*64 + mi*32 + 8*(v/4) + 4*(lane/32) + v%4, col = wn*64 + ni*32 + lane%32
  float ss = 0.f;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int j = col0 + wn * 64 + ni * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = row0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (i < g.M && j < g.N) {
          const float x = g.alpha * acc[mi][ni][v];
          const int64_t at = (int64_t)b * g.c_batch_stride + (int64_t)i * g.ldc + j;
          if (EPI == X3_STORE_SPLIT) {
            uint32_t h, m, l;
            split3(x, h, m, l);
            g.c3[at] = (uint16_t)h; g.c3[g.c3_plane_stride + at] = (uint16_t)m; g.c3[2 * g.c3_plane_stride + at] = (uint16_t)l;
          } else {
            g.c[at] = x;
            ss += x * x;
          }
        }
      }
    }
  if (EPI == X3_STORE_NORM) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (tid == 0) g.norm_partial[(int64_t)b * tiles + tile] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

}  // namespace shampoo
