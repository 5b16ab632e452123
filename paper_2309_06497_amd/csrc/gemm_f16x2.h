// float32-accurate batched GEMM on the fp16 matrix cores (v_mfma_f32_32x32x16_f16).
//
// A float32 value x, scaled by a power of two s so that |s x| stays inside the fp16 range,
// splits into two fp16 values, s x = h + l up to 2^-24 |s x|, with h = fp16(s x) and
// l = fp16(s x - h) (11 significant bits each; the subtraction is exact).  The product of two
// fp16 values is exact in float32, so
//   a b = (ah bh + ah bl + al bh) / (sa sb) + O(2^-22 |a b|)
// and a float32 GEMM becomes three fp16 MFMA products accumulated in float32: what is dropped
// (al bl, and the 2^-24 tails of the splits) is at the level of the rounding of a single
// float32 product.  A bf16 operand (the gradient) is one exact fp16 term after scaling, which
// leaves two products.  The fp16 matrix cores run 16x faster than the float32 ones, so three
// products cost 3/16 of the float32-MFMA time (two: 1/8), with the same float32 accumulation.
// (Three bf16 terms per value would need no scaling, but six products and half as many more
// operand bytes; this kernel is bound by operand delivery, so bytes decide.)
//
// Scaling.  Each matrix has one scale, chosen from a bound on its largest element so that the
// scaled values stay below 2^14 (pow2_scale_f16): elements down to 2^-16 of the bound keep both
// terms normal, smaller ones lose relative but not absolute accuracy (error <= 2^-39 of the
// bound).  Roots get their scale when they are split, after each refresh (matrix_stats_kernel,
// split2h_kernel); the gradient block from max |G| found by the grafting pass of the same step;
// T = c1 Lbar G from the bound c1 ||Lbar||_inf max |G| (x2_scales_kernel).  All scales are
// powers of two, so undoing them is exact.
//
// Operands are kept split in memory, as two (or one) fp16 planes, so the split is paid once
// per value and not once per tile that reads it; the first product of the preconditioning
// step writes its result T directly as two planes.  C[i][j] = alpha * sum_k A[i][k] * B[j][k]:
// both operands are read along k (row-major A; B given transposed, or symmetric).  The two
// products of Sec. 2.3 of the paper have that form:
//   T = Lbar G       A = Lbar (two planes)   B = G^T (the scaled fp16 transpose of the block, one plane)
//   P = T Rbar       A = T (two planes)      B = Rbar (symmetric, two planes)
//
// Tile TM x 256 per workgroup of 4 wavefronts, one workgroup per CU: TM = 256 with 128 x 128 per
// wavefront (4 x 4 MFMA tiles, 256 accumulator registers), or TM = 128 with 64 x 128 per
// wavefront; 8 wavefronts of 64 x 128 on the 256-row tile (two per SIMD) measured the same.
// Operand slabs of 32 values of k (64-byte rows) never pass through registers:
// global_load_lds_dwordx4 writes 16 bytes per lane straight into LDS, the next slab (the next
// two where three stages fit) in flight while the current one is multiplied.  LDS rows are
// unpadded (the 64 lanes of such a load fill consecutive addresses); the 16-byte chunk c of row
// r sits at chunk position c ^ ((r >> 2) & 3): a 16-byte read is served 16 lanes at a time from
// 64 banks of 4 bytes, the 16 rows of such a group start at banks 16 (r % 4), and rows with
// equal r % 4 take different chunk positions, so the group covers every bank once
// (SQ_LDS_BANK_CONFLICT reads 0).
// An MFMA operand is 8 consecutive k of one row per lane: lane = row % 32 + 32 * (k / 8).
//
// The LDS reads are scheduled by hand (inline assembly, with the s_waitcnt that belongs to
// each): the operands of the second k step of a slab are read while the first is multiplied.
// Requires K % 8 == 0, leading dimensions % 8 == 0 and 16-byte aligned operands (the host
// checks, and otherwise uses the float32-MFMA kernel).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"
#include "lds_dma.h"

namespace shampoo {

constexpr int X2_TN = 256;                     // workgroup tile: TM x 256
constexpr int X2_BK = 32;                      // k per slab (64-byte rows)
constexpr int X2_B_SLAB = X2_TN * X2_BK * 2;   // bytes of one plane of the B slab; A: A_SLAB = TM * 64 inside the kernel

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// X2_STORE_NORM: float32 result and per-tile sums of squares; X2_STORE_SPLIT: the result as
// two fp16 planes
enum { X2_STORE_NORM = 0, X2_STORE_SPLIT = 1 };

struct GemmX2Args {
  const uint16_t *a; int64_t a_plane_stride, a_batch_stride; int32_t lda;   // [plane][batch][M][K] fp16
  const uint16_t *b; int64_t b_plane_stride, b_batch_stride; int32_t ldb;   // [plane][batch][N][K] fp16
  float *c;                // X2_STORE_NORM: [batch][M][N] float32
  uint16_t *c2;            // X2_STORE_SPLIT: [plane][batch][M][N] fp16
  int64_t c2_plane_stride;
  int64_t c_batch_stride; int32_t ldc;
  int32_t M, N, K;
  float alpha;
  const float *out_scale;  // [batch] further factor on the result (a power of two; nullptr: none)
  float *norm_partial;     // X2_STORE_NORM: [batch][tiles] sums of squares of the stored tile
  int32_t tiles_m, tiles_n, batch;
};

// The power of two s that puts a bound on |x| just below 2^14 (s * bound in [2^13, 2^14)):
// fp16 values s x then stay finite with a factor 4 to spare, and their low-order terms
// stay normal down to 2^-16 of the bound.  1 for a bound that is zero or not finite.
__device__ __forceinline__ float pow2_scale_f16(float bound) {
  if (!(bound > 0.f) || !(bound < 3.0e38f)) return 1.f;
  int e;
  (void)frexpf(bound, &e);               // bound = f 2^e with f in [0.5, 1)
  return ldexpf(1.f, min(max(14 - e, -126), 100));
}

// x = h + l up to 2^-24 |x| (11 significant bits each), both fp16; |x| must be below 65504
__device__ __forceinline__ void split2h(float x, uint16_t &h, uint16_t &l) {
  const _Float16 hh = (_Float16)x;
  const _Float16 ll = (_Float16)(x - (float)hh);
  h = __builtin_bit_cast(uint16_t, hh);
  l = __builtin_bit_cast(uint16_t, ll);
}

// stats[2 b] = max |x_ij|, stats[2 b + 1] = max_i sum_j |x_ij| of the n x n matrix b.
// grid (batch), 256 threads.
__global__ __launch_bounds__(256) void matrix_stats_kernel(const float *x, float *stats, int n) {
  __shared__ float red[8];
  const float *p = x + (int64_t)blockIdx.x * n * n;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float mx = 0.f, rs = 0.f;
  for (int i = wave; i < n; i += 4) {
    float sum = 0.f;
    for (int j = lane; j < n; j += 64) {
      const float v = fabsf(p[(int64_t)i * n + j]);
      sum += v;
      mx = fmaxf(mx, v);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    rs = fmaxf(rs, sum);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  if (lane == 0) { red[wave] = mx; red[4 + wave] = rs; }
  __syncthreads();
  if (threadIdx.x == 0) {
    stats[2 * blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    stats[2 * blockIdx.x + 1] = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
  }
}

// out[plane][i] = the two fp16 terms of s_b in[i], s_b = pow2_scale_f16(stats[2 b]) for the
// matrix b = i / per that element i belongs to
__global__ __launch_bounds__(256) void split2h_kernel(const float *in, const float *stats, uint16_t *out, int64_t per, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const float sc = pow2_scale_f16(stats[2 * (i / per)]);
  uint16_t h, l;
  split2h(in[i] * sc, h, l);
  out[i] = h; out[count + i] = l;
}

// Scales of the fp16 operands of one bucket and step, all powers of two.  The gradient block
// goes to the matrix cores as fp16(s_G G) with s_G from max |G|; T = c1 Lbar G is bounded by
// c1 ||Lbar||_inf max |G| and kept as the planes of s_T T; the roots are kept as the planes
// of s_L Lbar and s_R Rbar (from their largest elements).  So
//   G^T G      = acc / s_G^2
//   s_T T      = c1 acc s_T / (s_L s_G)
//   P = T Rbar = acc / (s_T s_R)
// One wavefront per block.
struct X2ScaleArgs {
  const float *gmax_partial; int32_t parts;   // [batch][parts] max |G| per piece of the block
  const float *stat_l, *stat_r;               // matrix_stats_kernel of Lbar, Rbar
  float c1;
  float *s_g, *inv_g2, *t_scale, *inv_ts;     // [batch] s_G, 1 / s_G^2, s_T / (s_L s_G), 1 / (s_T s_R)
};
__global__ __launch_bounds__(64) void x2_scales_kernel(const X2ScaleArgs g) {
  const int b = blockIdx.x, lane = threadIdx.x;
  float gm = 0.f;
  for (int i = lane; i < g.parts; i += 64) gm = fmaxf(gm, g.gmax_partial[(int64_t)b * g.parts + i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) gm = fmaxf(gm, __shfl_xor(gm, off, 64));
  if (lane == 0) {
    const float sg = pow2_scale_f16(gm);
    const float st = pow2_scale_f16(fabsf(g.c1) * g.stat_l[2 * b + 1] * gm);
    const float sl = pow2_scale_f16(g.stat_l[2 * b]);
    const float sr = pow2_scale_f16(g.stat_r[2 * b]);
    g.s_g[b] = sg;
    g.inv_g2[b] = (1.f / sg) * (1.f / sg);
    g.t_scale[b] = (st / sl) / sg;
    g.inv_ts[b] = (1.f / st) * (1.f / sr);
  }
}

#define X2_DS_READ(dst, addr, imm) LDS_DS_READ_B128(dst, addr, imm)
#define X2_SB() LDS_SCHED_BARRIER()
// the MI 32-row tiles of plane S of the A slab into ARR[I] / the four of plane U of the B slab
// into DST, at the k step of (LA, LB)
#define X2_RD_A(ARR, I, S, LA) { X2_DS_READ(ARR[I][0], LA, (S) * A_SLAB); X2_DS_READ(ARR[I][1], LA, (S) * A_SLAB + 2048); \
                                 if constexpr (MI == 4) { X2_DS_READ(ARR[I][MI - 2], LA, (S) * A_SLAB + 4096); X2_DS_READ(ARR[I][MI - 1], LA, (S) * A_SLAB + 6144); } }
#define X2_RD_B(DST, U, LB) { X2_DS_READ(DST[0], LB, (U) * X2_B_SLAB); X2_DS_READ(DST[1], LB, (U) * X2_B_SLAB + 2048); \
                              X2_DS_READ(DST[2], LB, (U) * X2_B_SLAB + 4096); X2_DS_READ(DST[3], LB, (U) * X2_B_SLAB + 6144); }
// wait until at most N2 (MI = 2) or N4 (MI = 4) LDS reads are outstanding; the named registers
// are valid afterwards
#define X2_WAIT_A(N2, N4, ARR, I) { if constexpr (MI == 2) asm volatile("s_waitcnt lgkmcnt(" #N2 ")" : "+v"(ARR[I][0]), "+v"(ARR[I][1]) :: "memory"); \
    else asm volatile("s_waitcnt lgkmcnt(" #N4 ")" : "+v"(ARR[I][0]), "+v"(ARR[I][1]), "+v"(ARR[I][MI - 2]), "+v"(ARR[I][MI - 1]) :: "memory"); }
#define X2_WAIT_B(N2, N4, B_) { if constexpr (MI == 2) asm volatile("s_waitcnt lgkmcnt(" #N2 ")" : "+v"(B_[0]), "+v"(B_[1]), "+v"(B_[2]), "+v"(B_[3]) :: "memory"); \
    else asm volatile("s_waitcnt lgkmcnt(" #N4 ")" : "+v"(B_[0]), "+v"(B_[1]), "+v"(B_[2]), "+v"(B_[3]) :: "memory"); }
#define X2_WAIT_AB(N2, N4, ARR, I, B_) { if constexpr (MI == 2) asm volatile("s_waitcnt lgkmcnt(" #N2 ")" : "+v"(ARR[I][0]), "+v"(ARR[I][1]), "+v"(B_[0]), "+v"(B_[1]), "+v"(B_[2]), "+v"(B_[3]) :: "memory"); \
    else asm volatile("s_waitcnt lgkmcnt(" #N4 ")" : "+v"(ARR[I][0]), "+v"(ARR[I][1]), "+v"(ARR[I][MI - 2]), "+v"(ARR[I][MI - 1]), "+v"(B_[0]), "+v"(B_[1]), "+v"(B_[2]), "+v"(B_[3]) :: "memory"); }
// 4 MI MFMAs: the MI tiles ARR[I] of a plane of A against the four tiles B_ of a plane of B
#define X2_GROUP(ARR, I, B_)                                                                              \
  {                                                                                                       \
    _Pragma("unroll") for (int i_ = 0; i_ < MI; ++i_)                                                     \
      _Pragma("unroll") for (int j_ = 0; j_ < 4; ++j_)                                                    \
        acc[i_][j_] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, ARR[I][i_]),       \
                                                             __builtin_bit_cast(f16x8, B_[j_]), acc[i_][j_], 0, 0, 0); \
  }

// TM x 256 workgroup tile of wavefront tiles WM x 128.  NB: planes of B (2, or 1 for the scaled
// gradient); A always has two.
template <int TM, int WM, int NB, int EPI>
__global__ __launch_bounds__(TM / WM * 128, 1) void gemm_f16x2_kernel(const GemmX2Args g) {
  static_assert((TM == 128 && WM == 64) || (TM == 256 && (WM == 64 || WM == 128)), "wavefront tiles of 64 or 128 rows");
  static_assert(NB == 1 || NB == 2, "planes of B");
  constexpr int NA = 2;
  constexpr int MI = WM / 32;                  // 32-row MFMA tiles per wavefront
  constexpr int NW = TM / WM * 2;              // wavefronts, as TM / WM x 2
  constexpr int AL = TM / (16 * NW);           // 1 KiB pieces of an A plane slab that one wavefront loads
  constexpr int BL = 16 / NW;                  // and of a B plane slab
  constexpr int A_SLAB = TM * X2_BK * 2;       // bytes of one plane of the A slab
  // TM = 128: 48 KB (2 + 2 planes), 32 KB (2 + 1); TM = 256: 64 KB (2 + 2), 48 KB (2 + 1)
  constexpr int STAGE = NA * A_SLAB + NB * X2_B_SLAB;
  constexpr int NST = STAGE > 49152 ? 2 : 3;
  static_assert(NST * STAGE <= 147456, "LDS");
  constexpr int PW = AL * NA + BL * NB;        // loads per wavefront per slab
  __shared__ __align__(128) unsigned char smem[NST * STAGE];   // the k-step addresses below differ by an XOR
  __shared__ float red[NW];
  const int tiles = g.tiles_m * g.tiles_n;
  const int total = tiles * g.batch;
  const int logical = xcd_remap(blockIdx.x, total);
  if (logical >= total) return;
  const int b = logical / tiles;
  const int tile = logical - b * tiles;
  const int ti = tile / g.tiles_n, tj = tile - ti * g.tiles_n;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = ti * TM, col0 = tj * X2_TN;
  const uint16_t *pa = g.a + (int64_t)b * g.a_batch_stride + (int64_t)row0 * g.lda;
  const uint16_t *pb = g.b + (int64_t)b * g.b_batch_stride + (int64_t)col0 * g.ldb;
  const int rows_a = g.M - row0, rows_b = g.N - col0;

  // Chunk position p = 64 q + lane of a plane slab: LDS row p / 4, position p % 4 within it.
  // Rows past the end of the matrix read its last row instead: they only reach elements of
  // the tile that are never stored.
  const int uw = __builtin_amdgcn_readfirstlane(wave);
  uint32_t offa[AL], offb[BL];
  int chunk_a[AL], chunk_b[BL];
#pragma unroll
  for (int t = 0; t < AL; ++t) {
    const int p = (wave * AL + t) * 64 + lane, row = p >> 2, ch = (p & 3) ^ ((row >> 2) & 3);
    chunk_a[t] = ch * 8;
    offa[t] = (uint32_t)(min(row, rows_a - 1) * g.lda + ch * 8) * 2u;
  }
#pragma unroll
  for (int t = 0; t < BL; ++t) {
    const int p = (wave * BL + t) * 64 + lane, row = p >> 2, ch = (p & 3) ^ ((row >> 2) & 3);
    chunk_b[t] = ch * 8;
    offb[t] = (uint32_t)(min(row, rows_b - 1) * g.ldb + ch * 8) * 2u;
  }
  auto issue = [&](int stage, int k0) {
    unsigned char *st = smem + stage * STAGE;
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      const char *ga = uniform_ptr(pa + s * g.a_plane_stride + k0);
#pragma unroll
      for (int t = 0; t < AL; ++t)
        __builtin_amdgcn_global_load_lds((glb_void *)(ga + offa[t]), (lds_void *)(st + s * A_SLAB + (uw * AL + t) * 1024), 16, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const char *gb = uniform_ptr(pb + u * g.b_plane_stride + k0);
#pragma unroll
      for (int t = 0; t < BL; ++t)
        __builtin_amdgcn_global_load_lds((glb_void *)(gb + offb[t]), (lds_void *)(st + NA * A_SLAB + u * X2_B_SLAB + (uw * BL + t) * 1024), 16, 0, 0);
    }
  };

  // LDS byte addresses of this lane's operand rows in stage 0, k step 0 (k step 1: ^ 32)
  const int fi = lane & 31, fq = lane >> 5;
  const uint32_t lbase = (uint32_t)(uintptr_t)(lds_void *)smem;
  const uint32_t la0 = lbase + (wm * WM + fi) * 64 + ((fq ^ ((fi >> 2) & 3)) * 16);
  const uint32_t lb0 = lbase + NA * A_SLAB + (wn * 128 + fi) * 64 + ((fq ^ ((fi >> 2) & 3)) * 16);

  floatx16 acc[MI][4];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // operand registers: a[0] / a[1] the planes h / l of A and b0 / b1 those of B at the first k
  // step; ay / by0 the h planes at the second k step, whose l planes go into the registers that
  // b1 and a[0] have left by then
  u32x4 a[2][MI], b0[4], b1[4], ay[1][MI], by0[4];

  // One 1 KiB piece of the next slab: the loads are spread between the MFMA groups, so that a
  // wavefront never queues more than the texture path takes at once (a wavefront stalled on
  // issuing loads issues no MFMAs either).  With eight wavefronts each loads two pieces of a
  // plane, not four: pieces 2 and 3 do not exist then.
#define X2_DMA_A(S, T) { if constexpr ((T) < AL) __builtin_amdgcn_global_load_lds((glb_void *)(ga[S] + offa[(T) < AL ? (T) : 0]), (lds_void *)(st_in + (S) * A_SLAB + (uw * AL + (T)) * 1024), 16, 0, 0); }
#define X2_DMA_B(U, T) { if constexpr ((T) < BL) __builtin_amdgcn_global_load_lds((glb_void *)(gb[U] + offb[(T) < BL ? (T) : 0]), (lds_void *)(st_in + NA * A_SLAB + (U) * X2_B_SLAB + (uw * BL + (T)) * 1024), 16, 0, 0); }
  // The products of one slab (two k steps of 16) in the stage at byte offset `so`, and, if
  // `feed`, the loads of the slab at k0 into the stage at `st_in`.
  auto slab_product = [&](uint32_t so, bool feed, unsigned char *st_in, int k0) {
    const uint32_t la = la0 + so, lb = lb0 + so, la1 = la ^ 32, lb1 = lb ^ 32;
    const char *ga[NA], *gb[NB];
#pragma unroll
    for (int s = 0; s < NA; ++s) ga[s] = uniform_ptr(pa + s * g.a_plane_stride + k0);
#pragma unroll
    for (int u = 0; u < NB; ++u) gb[u] = uniform_ptr(pb + u * g.b_plane_stride + k0);
    if constexpr (NB == 1) {
      // planes (h, l) of A against the single plane of B; the wait counts are the reads issued
      // after the ones waited for (MI per A plane, 4 per B plane)
      X2_RD_A(a, 0, 0, la); X2_RD_B(b0, 0, lb); X2_RD_A(a, 1, 1, la);
      X2_SB();
      X2_WAIT_AB(2, 4, a, 0, b0); X2_SB();              // outstanding after ah, b: al
      X2_GROUP(a, 0, b0); X2_RD_A(ay, 0, 0, la1); X2_RD_B(by0, 0, lb1);
      if (feed) { X2_DMA_A(0, 0); X2_DMA_A(0, 1); X2_DMA_A(0, 2); X2_DMA_A(0, 3); } X2_SB();
      X2_WAIT_A(6, 8, a, 1); X2_SB();                   // ah' b'
      X2_GROUP(a, 1, b0); X2_RD_A(a, 0, 1, la1);        // al' into a[0]
      if (feed) { X2_DMA_A(1, 0); X2_DMA_A(1, 1); X2_DMA_A(1, 2); X2_DMA_A(1, 3); } X2_SB();
      X2_WAIT_AB(2, 4, ay, 0, by0); X2_SB();            // al'
      X2_GROUP(ay, 0, by0); if (feed) { X2_DMA_B(0, 0); X2_DMA_B(0, 1); } X2_SB();
      X2_WAIT_A(0, 0, a, 0); X2_SB();
      X2_GROUP(a, 0, by0); if (feed) { X2_DMA_B(0, 2); X2_DMA_B(0, 3); } X2_SB();
    } else {
      // planes (h, l) of both operands: the pairs (h,h) (h,l) (l,h)
      X2_RD_A(a, 0, 0, la); X2_RD_B(b0, 0, lb); X2_RD_B(b1, 1, lb); X2_RD_A(a, 1, 1, la);
      X2_SB();
      X2_WAIT_AB(6, 8, a, 0, b0); X2_SB();              // outstanding after ah, bh: bl al
      X2_GROUP(a, 0, b0); X2_RD_A(ay, 0, 0, la1); X2_RD_B(by0, 0, lb1);
      if (feed) { X2_DMA_A(0, 0); X2_DMA_A(0, 1); X2_DMA_A(0, 2); X2_DMA_A(0, 3); } X2_SB();
      X2_WAIT_B(8, 12, b1); X2_SB();                    // al ah' bh'
      X2_GROUP(a, 0, b1); X2_RD_B(b1, 1, lb1);          // bl' into b1
      if (feed) { X2_DMA_A(1, 0); X2_DMA_A(1, 1); X2_DMA_A(1, 2); X2_DMA_A(1, 3); } X2_SB();
      X2_WAIT_A(10, 12, a, 1); X2_SB();                 // ah' bh' bl'
      X2_GROUP(a, 1, b0); X2_RD_A(a, 0, 1, la1);        // al' into a[0]
      if (feed) { X2_DMA_B(0, 0); X2_DMA_B(0, 1); } X2_SB();
      X2_WAIT_AB(6, 8, ay, 0, by0); X2_SB();            // bl' al'
      X2_GROUP(ay, 0, by0); if (feed) { X2_DMA_B(0, 2); X2_DMA_B(0, 3); } X2_SB();
      X2_WAIT_B(2, 4, b1); X2_SB();                     // al'
      X2_GROUP(ay, 0, b1); if (feed) { X2_DMA_B(1, 0); X2_DMA_B(1, 1); } X2_SB();
      X2_WAIT_A(0, 0, a, 0); X2_SB();
      X2_GROUP(a, 0, by0); if (feed) { X2_DMA_B(1, 2); X2_DMA_B(1, 3); } X2_SB();
    }
  };

  const int nk = g.K / X2_BK;                    // full slabs; K % 32 values of k remain
#pragma unroll
  for (int s = 0; s < NST - 1; ++s)
    if (s < nk) issue(s, s * X2_BK);
  if (g.K % X2_BK) {
    // The ragged end of k goes first, through registers with zero fill, into the last stage,
    // while the first full slabs are on their way.
    const int k0 = nk * X2_BK;
    unsigned char *st = smem + (NST - 1) * STAGE;
#pragma unroll
    for (int s = 0; s < NA; ++s)
#pragma unroll
      for (int t = 0; t < AL; ++t) {
        const bool kin = k0 + chunk_a[t] < g.K;    // K % 8 == 0: a chunk is entirely in or out
        const uint4 v = kin ? *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(pa + s * g.a_plane_stride + k0) + offa[t])
                            : make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4 *>(st + s * A_SLAB + (wave * AL + t) * 1024 + lane * 16) = v;
      }
#pragma unroll
    for (int u = 0; u < NB; ++u)
#pragma unroll
      for (int t = 0; t < BL; ++t) {
        const bool kin = k0 + chunk_b[t] < g.K;
        const uint4 v = kin ? *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(pb + u * g.b_plane_stride + k0) + offb[t])
                            : make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4 *>(st + NA * A_SLAB + u * X2_B_SLAB + (wave * BL + t) * 1024 + lane * 16) = v;
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
    slab_product((uint32_t)(stage * STAGE), kin < nk, smem + stage_in * STAGE, min(kin, nk - 1) * X2_BK);
    stage = stage + 1 == NST ? 0 : stage + 1;
    stage_in = stage_in + 1 == NST ? 0 : stage_in + 1;
  }
  LDS_DMA_WAIT_VM(0);

  // epilogue: accumulator element v of MFMA tile (mi, ni) is
  // row = wm*WM + mi*32 + 8*(v/4) + 4*(lane/32) + v%4, col = wn*128 + ni*32 + lane%32
  // (one store instruction covers two rows of 32 consecutive columns: whole 128-byte lines
  // for the float32 result; storing runs of four columns per lane from transposed result
  // tiles takes a quarter of the instructions and measured slower, 5.0 -> 5.8 ms for T)
  float ss = 0.f;
  const float alpha = g.out_scale ? g.alpha * g.out_scale[b] : g.alpha;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
      const int j = col0 + wn * 128 + ni * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = row0 + wm * WM + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (i < g.M && j < g.N) {
          const float x = alpha * acc[mi][ni][v];
          const int64_t at = (int64_t)b * g.c_batch_stride + (int64_t)i * g.ldc + j;
          if (EPI == X2_STORE_SPLIT) {
            uint16_t h, l;
            split2h(x, h, l);
            g.c2[at] = h; g.c2[g.c2_plane_stride + at] = l;
          } else {
            g.c[at] = x;
            ss += x * x;
          }
        }
      }
    }
  if (EPI == X2_STORE_NORM) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (tid == 0) {
      float tot = (red[0] + red[1]) + (red[2] + red[3]);
      if constexpr (NW == 8) tot += (red[4] + red[5]) + (red[6] + red[7]);
      g.norm_partial[(int64_t)b * tiles + tile] = tot;
    }
  }
}
#undef X2_DMA_A
#undef X2_DMA_B

}  // namespace shampoo
