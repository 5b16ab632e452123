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
// Tile 128 x 256 per workgroup of 4 wavefronts (64 x 128 each, 2 x 4 MFMA tiles), one
// workgroup per CU.  With six (three) MFMA products per pair of operand values the kernel is
// bound by the matrix cores only if the operands arrive fast enough; measured on this part,
// L2-resident panels reach LDS at ~16 TB/s (all CUs together) when each row piece is at least
// 64 bytes, and a 128 x 128 tile of the six-product kernel would need more than that at the
// rate the matrix cores sustain.  Hence the larger tile, and operand slabs of 32 values of k
// (64-byte rows) that never pass through registers: global_load_lds_dwordx4 writes 16 bytes
// per lane straight into LDS, the next slab (the next two for the three-product kernel, whose
// stages are smaller) in flight while the current one is multiplied.  LDS rows are unpadded
// (the 64 lanes of such a load fill consecutive addresses); the 16-byte chunk c of row r sits
// at chunk position c ^ ((r >> 1) & 3), which keeps the operand reads free of bank conflicts.
// An MFMA operand is 8 consecutive k of one row per lane: lane = row % 32 + 32 * (k / 8).
//
// One wavefront per SIMD leaves nobody to cover a stall, so the LDS reads are scheduled by
// hand (inline assembly, with the s_waitcnt that belongs to each): the registers of an
// operand plane are refilled for the next 16 k as soon as the last MFMA group that reads
// them has been issued, two or more groups (512 cycles) before they are needed again.
// Requires K % 8 == 0, leading dimensions % 8 == 0 and 16-byte aligned operands (the host
// checks, and otherwise uses the float32-MFMA kernel).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"
#include "lds_dma.h"

namespace shampoo {

constexpr int X3_TM = 128, X3_TN = 256;        // workgroup tile
constexpr int X3_BK = 32;                      // k per slab (64-byte rows)
constexpr int X3_A_SLAB = X3_TM * X3_BK * 2;   // bytes of one plane of the A slab
constexpr int X3_B_SLAB = X3_TN * X3_BK * 2;

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

#define X3_DS_READ(dst, addr, imm) LDS_DS_READ_B128(dst, addr, imm)
#define X3_SB() LDS_SCHED_BARRIER()
// the two 32-row tiles of plane S of the A slab / the four of plane U of the B slab, at the k step of (LA, LB)
#define X3_RD_A(S, LA) { X3_DS_READ(a[S][0], LA, (S) * X3_A_SLAB); X3_DS_READ(a[S][1], LA, (S) * X3_A_SLAB + 2048); }
#define X3_RD_B(DST, U, LB) { X3_DS_READ(DST[0], LB, (U) * X3_B_SLAB); X3_DS_READ(DST[1], LB, (U) * X3_B_SLAB + 2048); \
                              X3_DS_READ(DST[2], LB, (U) * X3_B_SLAB + 4096); X3_DS_READ(DST[3], LB, (U) * X3_B_SLAB + 6144); }
// wait until at most N LDS reads are outstanding; the named registers are valid afterwards
#define X3_WAIT_A(N, S) asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(a[S][0]), "+v"(a[S][1]) :: "memory")
#define X3_WAIT_B(N, B_) asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(B_[0]), "+v"(B_[1]), "+v"(B_[2]), "+v"(B_[3]) :: "memory")
#define X3_WAIT_AB(N, S, B_) asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(a[S][0]), "+v"(a[S][1]), "+v"(B_[0]), "+v"(B_[1]), "+v"(B_[2]), "+v"(B_[3]) :: "memory")
// eight MFMAs: plane S of A against the four tiles B_ of a plane of B
#define X3_GROUP(S, B_)                                                                                   \
  {                                                                                                       \
    _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                                      \
      _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_)                                                    \
        acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[S][i_]),       \
                                                              __builtin_bit_cast(bf16x8, B_[j_]), acc[i_][j_], 0, 0, 0); \
  }

template <int NA, int NB, int EPI>
__global__ __launch_bounds__(GEMM_THREADS, 1) void gemm_bf16x3_kernel(const GemmX3Args g) {
  static_assert(NA == 3 && (NB == 3 || NB == 1), "plane counts of the two products of the preconditioning step");
  constexpr int STAGE = NA * X3_A_SLAB + NB * X3_B_SLAB;     // 72 KB (3 + 3 planes) or 40 KB (3 + 1)
  constexpr int NST = NB == 3 ? 2 : 3;
  constexpr int PW = 2 * NA + 4 * NB;                        // loads per wavefront per slab
  __shared__ __align__(128) unsigned char smem[NST * STAGE];
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
  const int row0 = ti * X3_TM, col0 = tj * X3_TN;
  const uint16_t *pa = g.a + (int64_t)b * g.a_batch_stride + (int64_t)row0 * g.lda;
  const uint16_t *pb = g.b + (int64_t)b * g.b_batch_stride + (int64_t)col0 * g.ldb;
  const int rows_a = g.M - row0, rows_b = g.N - col0;

  // Chunk position p = 64 q + lane of a plane slab: LDS row p / 4, position p % 4 within it.
  // Rows past the end of the matrix read its last row instead: they only reach elements of
  // the tile that are never stored.
  const int uw = __builtin_amdgcn_readfirstlane(wave);
  uint32_t offa[2], offb[4];
  int chunk_a[2], chunk_b[4];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int p = (wave * 2 + t) * 64 + lane, row = p >> 2, ch = (p & 3) ^ ((row >> 1) & 3);
    chunk_a[t] = ch * 8;
    offa[t] = (uint32_t)(min(row, rows_a - 1) * g.lda + ch * 8) * 2u;
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int p = (wave * 4 + t) * 64 + lane, row = p >> 2, ch = (p & 3) ^ ((row >> 1) & 3);
    chunk_b[t] = ch * 8;
    offb[t] = (uint32_t)(min(row, rows_b - 1) * g.ldb + ch * 8) * 2u;
  }
  auto issue = [&](int stage, int k0) {
    unsigned char *st = smem + stage * STAGE;
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      const char *ga = uniform_ptr(pa + s * g.a_plane_stride + k0);
#pragma unroll
      for (int t = 0; t < 2; ++t)
        __builtin_amdgcn_global_load_lds((glb_void *)(ga + offa[t]), (lds_void *)(st + s * X3_A_SLAB + (uw * 2 + t) * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const char *gb = uniform_ptr(pb + u * g.b_plane_stride + k0);
#pragma unroll
      for (int t = 0; t < 4; ++t)
        __builtin_amdgcn_global_load_lds((glb_void *)(gb + offb[t]), (lds_void *)(st + NA * X3_A_SLAB + u * X3_B_SLAB + (uw * 4 + t) * 1024), 16, 0, 0);
    }
  };

  // LDS byte addresses of this lane's operand rows in stage 0, k step 0 (k step 1: ^ 32)
  const int fi = lane & 31, fq = lane >> 5;
  const uint32_t lbase = (uint32_t)(uintptr_t)(lds_void *)smem;
  const uint32_t la0 = lbase + (wm * 64 + fi) * 64 + ((fq ^ ((fi >> 1) & 3)) * 16);
  const uint32_t lb0 = lbase + NA * X3_A_SLAB + (wn * 128 + fi) * 64 + ((fq ^ ((fi >> 1) & 3)) * 16);

  floatx16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  u32x4 a[3][2];          // [plane][tile]
  u32x4 b0[4], b1[4], b2[4];   // NB == 3: the planes of B; NB == 1: b0 / b1 hold the plane at even / odd k steps

  // One 1 KiB piece of the next slab: the loads are spread between the MFMA groups, one or two
  // after each, so that the wavefront (the only one on its SIMD) never queues more than the
  // texture path takes at once: a wavefront stalled on issuing loads issues no MFMAs either.
#define X3_DMA_A(S, T) __builtin_amdgcn_global_load_lds((glb_void *)(ga[S] + offa[T]), (lds_void *)(st_in + (S) * X3_A_SLAB + (uw * 2 + (T)) * 1024), 16, 0, 0)
#define X3_DMA_B(U, T) __builtin_amdgcn_global_load_lds((glb_void *)(gb[U] + offb[T]), (lds_void *)(st_in + NA * X3_A_SLAB + (U) * X3_B_SLAB + (uw * 4 + (T)) * 1024), 16, 0, 0)
  // The products of one slab (two k steps of 16) in the stage at byte offset `so`, and, if
  // `feed`, the loads of the slab at k0 into the stage at `st_in`.
  auto slab_product = [&](uint32_t so, bool feed, unsigned char *st_in, int k0) {
    const uint32_t la = la0 + so, lb = lb0 + so, la1 = la ^ 32, lb1 = lb ^ 32;
    const char *ga[NA], *gb[NB];
#pragma unroll
    for (int s = 0; s < NA; ++s) ga[s] = uniform_ptr(pa + s * g.a_plane_stride + k0);
#pragma unroll
    for (int u = 0; u < NB; ++u) gb[u] = uniform_ptr(pb + u * g.b_plane_stride + k0);
    if constexpr (NB == 3) {
      // plane pairs (s, u) with s + u <= 2, in an order that frees every plane's registers two
      // or more groups before the next k step needs them: (0,2) (0,0) (2,0) (0,1) (1,0) (1,1)
      X3_RD_A(0, la); X3_RD_B(b2, 2, lb); X3_RD_B(b0, 0, lb); X3_RD_A(2, la); X3_RD_B(b1, 1, lb); X3_RD_A(1, la);
      X3_SB();
      X3_WAIT_AB(12, 0, b2); X3_SB();                   // outstanding after a0, b2: b0 a2 b1 a1 = 12
      X3_GROUP(0, b2); X3_RD_B(b2, 2, lb1); if (feed) { X3_DMA_A(0, 0); X3_DMA_A(0, 1); } X3_SB();
      X3_WAIT_B(12, b0); X3_SB();                       // a2 b1 a1 b2' = 12
      X3_GROUP(0, b0); if (feed) { X3_DMA_A(1, 0); X3_DMA_A(1, 1); } X3_SB();
      X3_WAIT_A(10, 2); X3_SB();                        // b1 a1 b2' = 10
      X3_GROUP(2, b0); X3_RD_A(2, la1); if (feed) { X3_DMA_A(2, 0); X3_DMA_A(2, 1); } X3_SB();
      X3_WAIT_B(8, b1); X3_SB();                        // a1 b2' a2' = 8
      X3_GROUP(0, b1); X3_RD_A(0, la1); if (feed) { X3_DMA_B(0, 0); X3_DMA_B(0, 1); } X3_SB();
      X3_WAIT_A(8, 1); X3_SB();                         // b2' a2' a0' = 8
      X3_GROUP(1, b0); X3_RD_B(b0, 0, lb1); if (feed) { X3_DMA_B(0, 2); X3_DMA_B(0, 3); } X3_SB();
      X3_GROUP(1, b1); X3_RD_A(1, la1); X3_RD_B(b1, 1, lb1); if (feed) { X3_DMA_B(1, 0); X3_DMA_B(1, 1); } X3_SB();
      // second k step; issue order of its reads: b2 a2 a0 b0 a1 b1
      X3_WAIT_AB(10, 0, b2); X3_SB();                   // b0 a1 b1 = 10
      X3_GROUP(0, b2); if (feed) { X3_DMA_B(1, 2); X3_DMA_B(1, 3); } X3_SB();
      X3_WAIT_B(6, b0); X3_SB();                        // a1 b1 = 6
      X3_GROUP(0, b0); if (feed) { X3_DMA_B(2, 0); X3_DMA_B(2, 1); } X3_SB();
      X3_WAIT_A(6, 2); X3_SB();
      X3_GROUP(2, b0); if (feed) { X3_DMA_B(2, 2); X3_DMA_B(2, 3); } X3_SB();
      X3_WAIT_AB(0, 1, b1); X3_SB();
      X3_GROUP(0, b1); X3_SB();
      X3_GROUP(1, b0); X3_SB();
      X3_GROUP(1, b1); X3_SB();
    } else {
      X3_RD_A(0, la); X3_RD_B(b0, 0, lb); X3_RD_A(1, la); X3_RD_A(2, la);
      X3_SB();
      X3_WAIT_AB(4, 0, b0); X3_SB();                    // a1 a2 = 4
      X3_GROUP(0, b0); X3_RD_A(0, la1); X3_RD_B(b1, 0, lb1); if (feed) { X3_DMA_A(0, 0); X3_DMA_A(0, 1); } X3_SB();
      X3_WAIT_A(8, 1); X3_SB();                         // a2 a0' b' = 8
      X3_GROUP(1, b0); X3_RD_A(1, la1); if (feed) { X3_DMA_A(1, 0); X3_DMA_A(1, 1); } X3_SB();
      X3_WAIT_A(8, 2); X3_SB();                         // a0' b' a1' = 8
      X3_GROUP(2, b0); X3_RD_A(2, la1); if (feed) { X3_DMA_A(2, 0); X3_DMA_A(2, 1); } X3_SB();
      X3_WAIT_AB(4, 0, b1); X3_SB();                    // a1' a2' = 4
      X3_GROUP(0, b1); if (feed) { X3_DMA_B(0, 0); X3_DMA_B(0, 1); } X3_SB();
      X3_WAIT_A(2, 1); X3_SB();
      X3_GROUP(1, b1); if (feed) { X3_DMA_B(0, 2); X3_DMA_B(0, 3); } X3_SB();
      X3_WAIT_A(0, 2); X3_SB();
      X3_GROUP(2, b1); X3_SB();
    }
  };

  const int nk = g.K / X3_BK;                    // full slabs; K % 32 values of k remain
#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < nk) issue(s, s * X3_BK);
  if (g.K % X3_BK) {
    // The ragged end of k goes first, through registers with zero fill, into the last stage,
    // while the first full slabs are on their way.
    const int k0 = nk * X3_BK;
    unsigned char *st = smem + (NST - 1) * STAGE;
#pragma unroll
    for (int s = 0; s < NA; ++s)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bool kin = k0 + chunk_a[t] < g.K;    // K % 8 == 0: a chunk is entirely in or out
        const uint4 v = kin ? *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(pa + s * g.a_plane_stride + k0) + offa[t])
                            : make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4 *>(st + s * X3_A_SLAB + (wave * 2 + t) * 1024 + lane * 16) = v;
      }
#pragma unroll
    for (int u = 0; u < NB; ++u)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bool kin = k0 + chunk_b[t] < g.K;
        const uint4 v = kin ? *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(pb + u * g.b_plane_stride + k0) + offb[t])
                            : make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4 *>(st + NA * X3_A_SLAB + u * X3_B_SLAB + (wave * 4 + t) * 1024 + lane * 16) = v;
      }
    __syncthreads();
    slab_product((NST - 1) * STAGE, false, smem, 0);
  }
  // Slab kt is multiplied while the next NST - 1 slabs are on their way.
  int stage = 0, stage_in = NST - 1;
  for (int kt = 0; kt < nk; ++kt) {
    // outstanding: slab kt, and slab kt + 1 if there are three stages and it exists
    if (NST == 3 && kt + 1 < nk) { LDS_DMA_WAIT_VM(PW); } else { LDS_DMA_WAIT_VM(0); }
    __builtin_amdgcn_s_barrier();
    const int kin = kt + NST - 1;
    slab_product((uint32_t)(stage * STAGE), kin < nk, smem + stage_in * STAGE, min(kin, nk - 1) * X3_BK);
    stage = stage + 1 == NST ? 0 : stage + 1;
    stage_in = stage_in + 1 == NST ? 0 : stage_in + 1;
  }
  LDS_DMA_WAIT_VM(0);

  // epilogue: accumulator element v of MFMA tile (mi, ni) is
  // row = wm*64 + mi*32 + 8*(v/4) + 4*(lane/32) + v%4, col = wn*128 + ni*32 + lane%32
  float ss = 0.f;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int j = col0 + wn * 128 + ni * 32 + (lane & 31);
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
