// Factor update for bf16 gradients on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16).
//
// The product of two bf16 values is exact in float32, so G G^T of a bf16 gradient
// loses nothing on the bf16 MFMA path (16x the float32 MFMA rate) but the roundings of the
// float32 accumulator, one per MFMA of 16 values of k: measured 1.3e-7 ... 1.9e-7 of the
// factor's norm at k = 1024, against a bar of 1e-5.  That is enough once a factor holds a
// few times more gradient columns than it has rows (condition number of order 10).  Before
// that -- the factor of the very first steps is a near-singular Gram matrix, and the first
// root refresh is taken from it -- its smallest eigenvalues are at 1e-7 of the largest and
// the sum has to be as good as float32 storage allows: the ACC64 variant starts every slab
// (32 values of k) from zero accumulators and adds the result into float64 registers
// (measured 4e-8; 128 more registers per lane, two workgroups per CU, a third slower).  The
// host picks the variant per step.  beta2 L + (1 - beta2) S is evaluated in float64 before
// the single rounding to float32.  R = G^T G runs through the same kernel on a 16-bit transpose of the
// block (transpose_bf16_kernel), so both operands are always read along k; where the
// fp16 preconditioning products follow, that transpose holds fp16(s G) with a power of
// two s per block (8 significant bits go into 11, so nothing is lost unless it
// underflows), the fp16 instruction is used and 1 / s^2 is applied with alpha.
//
// Tile 128 x 128 per workgroup of 4 wavefronts (64 x 64 each, 2 x 2 MFMA tiles).
// The operand slabs (128 rows x 32 k of each operand) never pass through registers:
// global_load_lds_dwordx4 moves 16 bytes per lane straight into LDS, three slabs deep,
// so that two slabs are in flight while one is multiplied.  Such a load writes the 64
// lanes' chunks to consecutive LDS addresses, which leaves no room for row padding;
// bank conflicts are avoided by a swizzle instead: the 16-byte chunk c of row r sits at
// chunk position c ^ ((r >> 2) & 3) of its 64-byte LDS row (the lane picks its global
// address accordingly).  A 16-byte read is served 16 lanes at a time from 64 banks of 4 bytes:
// the 16 rows of such a group start at banks 16 (r % 4), and rows with equal r % 4 take
// different chunk positions, so the group covers every bank once.  An MFMA operand is 8
// consecutive k of one row per lane: lane = row % 32 + 32 * (k / 8).
//
// The compiler's own wait-count placement would wait for every outstanding load before
// the first LDS read of a slab (it cannot tell the stages apart), so the LDS reads of the
// main loop and the waits that belong to them are written as inline assembly, and the
// workgroup barrier of the loop is the bare s_barrier: the loads of later slabs stay in
// flight across it.
//
// Only the tiles on and below the diagonal of tiles are computed and written; the mirror image
// is left to mirror_upper_tiles_kernel: nothing in a step reads the tiles above the diagonal,
// only the refresh and the state query do.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "gemm_mfma.h"
#include "lds_dma.h"

namespace shampoo {

constexpr int SBK = 32;                        // k per slab: two MFMAs per 32 x 32 tile
constexpr int SYRK_SLAB = BM * SBK * 2;        // bytes of one operand slab
constexpr int SYRK_STAGE = 2 * SYRK_SLAB;      // A slab, then B slab
constexpr int SYRK_STAGES = 3;                 // a fourth stage fits the LDS footprint and measured no faster

struct SyrkBf16Args {
  Operand a;                 // bf16 matrix X (rows x K, k contiguous); C = beta C + alpha X X^T
  const BlockDesc *desc;
  const void *const *ptr_table;
  float *c; int64_t c_batch_stride; int32_t ldc;
  int32_t M, K;              // C is M x M
  double alpha, beta;
  const float *x_scale2;     // [batch] X holds fp16 values s x: 1 / s^2, applied with alpha (nullptr: X is bf16)
  int32_t tiles;             // lower-triangular tile count per batch entry
  int32_t batch;
};

typedef _Float16 syrk_f16x8 __attribute__((ext_vector_type(8)));

template <bool F16>
__device__ __forceinline__ floatx16 syrk_mfma(floatx16 acc, const u32x4 &a0, const u32x4 &b0) {
  if constexpr (F16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(syrk_f16x8, a0), __builtin_bit_cast(syrk_f16x8, b0), acc, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0), __builtin_bit_cast(bf16x8, b0), acc, 0, 0, 0);
  }
}

// Requires: operand base 16-byte aligned, ld % 8 == 0, K % 8 == 0 (checked by the host).
// F16: the operand holds fp16 values (the scaled transpose of a bf16 block: products of two
// such values are exact in float32 as well) and the fp16 matrix-core instruction is used.
// ACC64: float64 accumulators, see the head of this file.
template <bool F16, bool ACC64>
__global__ __launch_bounds__(GEMM_THREADS, ACC64 ? 2 : 3) void syrk_bf16_kernel(const SyrkBf16Args g) {
  __shared__ __align__(128) unsigned char smem[SYRK_STAGES * SYRK_STAGE];   // the k-step addresses below differ by an XOR
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

  // Chunk position p = 64 q + lane of a slab (q = 2 wave + t): LDS row p / 4, position p % 4
  // within it.  Rows past the end of the matrix read its last row instead: they only reach
  // elements of the tile that are never stored.
  constexpr int PER_WAVE = BM * (SBK / 8) / 64 / 4;
  constexpr int PW = 2 * PER_WAVE;               // loads per wavefront per slab
  const int uw = __builtin_amdgcn_readfirstlane(wave);
  uint32_t offa[PER_WAVE], offb[PER_WAVE];
  int chunk_k[PER_WAVE];
#pragma unroll
  for (int t = 0; t < PER_WAVE; ++t) {
    const int p = (wave * PER_WAVE + t) * 64 + lane;
    const int row = p >> 2, ch = (p & 3) ^ ((row >> 2) & 3);
    chunk_k[t] = ch * 8;
    offa[t] = (uint32_t)(min(row, rows_a - 1) * ld + ch * 8) * 2u;
    offb[t] = (uint32_t)(min(row, rows_b - 1) * ld + ch * 8) * 2u;
  }
  // A tile on the diagonal multiplies a row panel by itself: only the B slab is loaded, and
  // the A operand is read from it as well.
  const bool diag = ti == tj;
  auto issue = [&](int stage, int k0) {
    const char *ga = uniform_ptr(xa + k0);
    const char *gb = uniform_ptr(xb + k0);
    unsigned char *sa = smem + stage * SYRK_STAGE, *sb = sa + SYRK_SLAB;
#pragma unroll
    for (int t = 0; t < PER_WAVE; ++t) {
      const int q = uw * PER_WAVE + t;
      if (!diag) __builtin_amdgcn_global_load_lds((glb_void *)(ga + offa[t]), (lds_void *)(sa + q * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((glb_void *)(gb + offb[t]), (lds_void *)(sb + q * 1024), 16, 0, 0);
    }
  };

  // LDS byte addresses of this lane's operand rows: k step s of a slab is chunk 2 s + lane / 32
  const int fi = lane & 31, fq = lane >> 5;
  const uint32_t lbase = (uint32_t)(uintptr_t)(lds_void *)smem;
  const uint32_t la0 = lbase + (diag ? SYRK_SLAB : 0) + ((wm * 64 + fi) * SBK + ((fq ^ ((fi >> 2) & 3)) * 8)) * 2, la1 = la0 ^ 32;
  const uint32_t lb0 = lbase + ((wn * 64 + fi) * SBK + ((fq ^ ((fi >> 2) & 3)) * 8)) * 2, lb1 = lb0 ^ 32;

  floatx16 acc[2][2];
  double acc64[ACC64 ? 2 : 1][ACC64 ? 2 : 1][16];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        acc[i][j][v] = 0.f;
        if constexpr (ACC64) acc64[i][j][v] = 0.0;
      }

  const int nk = g.K / SBK;                      // full slabs; K % SBK values of k remain
  if (nk > 0) issue(0, 0);
  if (nk > 1) issue(1, SBK);
  u32x4 oa[2][2], ob[2][2];                      // [i or j][k step]
  // The eight operand reads of the slab in stage S, then the eight MFMAs of the wavefront's four
  // 32 x 32 tiles (the two of one tile four instructions apart).
#define SYRK_SLAB_PRODUCT(S)                                                              \
  {                                                                                       \
    LDS_DS_READ_B128(oa[0][0], la0, (S) * SYRK_STAGE);                                        \
    LDS_DS_READ_B128(ob[0][0], lb0, (S) * SYRK_STAGE + SYRK_SLAB);                            \
    LDS_DS_READ_B128(oa[0][1], la1, (S) * SYRK_STAGE);                                        \
    LDS_DS_READ_B128(ob[0][1], lb1, (S) * SYRK_STAGE + SYRK_SLAB);                            \
    LDS_DS_READ_B128(oa[1][0], la0, (S) * SYRK_STAGE + 32 * SBK * 2);                         \
    LDS_DS_READ_B128(ob[1][0], lb0, (S) * SYRK_STAGE + SYRK_SLAB + 32 * SBK * 2);             \
    LDS_DS_READ_B128(oa[1][1], la1, (S) * SYRK_STAGE + 32 * SBK * 2);                         \
    LDS_DS_READ_B128(ob[1][1], lb1, (S) * SYRK_STAGE + SYRK_SLAB + 32 * SBK * 2);             \
    asm volatile("s_waitcnt lgkmcnt(0)"                                                   \
                 : "+v"(oa[0][0]), "+v"(oa[0][1]), "+v"(oa[1][0]), "+v"(oa[1][1]),        \
                   "+v"(ob[0][0]), "+v"(ob[0][1]), "+v"(ob[1][0]), "+v"(ob[1][1]) :: "memory"); \
    LDS_SCHED_BARRIER();                                                                            \
    acc[0][0] = syrk_mfma<F16>(acc[0][0], oa[0][0], ob[0][0]);                            \
    acc[0][1] = syrk_mfma<F16>(acc[0][1], oa[0][0], ob[1][0]);                            \
    acc[1][0] = syrk_mfma<F16>(acc[1][0], oa[1][0], ob[0][0]);                            \
    acc[1][1] = syrk_mfma<F16>(acc[1][1], oa[1][0], ob[1][0]);                            \
    acc[0][0] = syrk_mfma<F16>(acc[0][0], oa[0][1], ob[0][1]);                            \
    acc[0][1] = syrk_mfma<F16>(acc[0][1], oa[0][1], ob[1][1]);                            \
    acc[1][0] = syrk_mfma<F16>(acc[1][0], oa[1][1], ob[0][1]);                            \
    acc[1][1] = syrk_mfma<F16>(acc[1][1], oa[1][1], ob[1][1]);                            \
    LDS_SCHED_BARRIER();                                                                  \
    if constexpr (ACC64) {                                                                \
      _Pragma("unroll") for (int i_ = 0; i_ < 2; ++i_)                                    \
        _Pragma("unroll") for (int j_ = 0; j_ < 2; ++j_)                                  \
          _Pragma("unroll") for (int v_ = 0; v_ < 16; ++v_) {                             \
            acc64[i_][j_][v_] += (double)acc[i_][j_][v_];                                 \
            acc[i_][j_][v_] = 0.f;                                                        \
          }                                                                               \
    }                                                                                     \
  }

  if (g.K % SBK) {
    // The ragged end of k goes first, through registers with zero fill, into the last
    // stage, while the first full slabs are on their way.
    const int k0 = nk * SBK;
#pragma unroll
    for (int t = 0; t < PER_WAVE; ++t) {
      const int q = wave * PER_WAVE + t;
      const bool kin = k0 + chunk_k[t] < g.K;      // K % 8 == 0: a chunk is entirely in or out
      const uint4 va = kin ? *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(xa + k0) + offa[t]) : make_uint4(0, 0, 0, 0);
      const uint4 vb = kin ? *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(xb + k0) + offb[t]) : make_uint4(0, 0, 0, 0);
      *reinterpret_cast<uint4 *>(smem + (SYRK_STAGES - 1) * SYRK_STAGE + q * 1024 + lane * 16) = va;
      *reinterpret_cast<uint4 *>(smem + (SYRK_STAGES - 1) * SYRK_STAGE + SYRK_SLAB + q * 1024 + lane * 16) = vb;
    }
    __syncthreads();
    SYRK_SLAB_PRODUCT(SYRK_STAGES - 1);
  }
  // Slab kt is multiplied while slabs kt + 1 and kt + 2 are on their way.
#define SYRK_WAIT(N) { if (diag) { LDS_DMA_WAIT_VM((N) * PER_WAVE); } else { LDS_DMA_WAIT_VM((N) * PW); } }
#define SYRK_STEP(S, NEXT, KT)                                                            \
  {                                                                                       \
    if ((KT) + 1 < nk) SYRK_WAIT(1) else SYRK_WAIT(0)                                     \
    __builtin_amdgcn_s_barrier();                                                         \
    if ((KT) + 2 < nk) issue(NEXT, ((KT) + 2) * SBK);                                     \
    if ((KT) < nk) SYRK_SLAB_PRODUCT(S);                                                  \
  }
  for (int kt = 0; kt < nk; kt += 3) {
    SYRK_STEP(0, 2, kt);
    SYRK_STEP(1, 0, kt + 1);
    SYRK_STEP(2, 1, kt + 2);
  }
  LDS_DMA_WAIT_VM(0);

  // Epilogue.  Every computed tile (on or below the diagonal of tiles) is stored from the
  // accumulators, rows of 32 consecutive floats per half wavefront.  A tile on the diagonal is
  // stored whole: its elements (i, j) and (j, i) are the same products summed in the same order
  // by the matrix cores, from the same old values, so they carry the same bits and the factor
  // stays exactly symmetric.  The tiles above the diagonal are mirror_upper_tiles_kernel's.
  float *c = g.c + (int64_t)b * g.c_batch_stride;
  const int ldc = g.ldc;
  const double alpha = g.x_scale2 ? g.alpha * (double)g.x_scale2[b] : g.alpha;
  // The old values of half a quadrant (32 x 64) are requested before any of them is used,
  // from clamped (always valid) addresses so that the loads are unconditional: one memory
  // round trip per half instead of one per element.
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
    float old[2][16];
    if (g.beta != 0.0) {
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int j = min(col0 + wn * 64 + ni * 32 + (lane & 31), g.M - 1);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = min(row0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3), g.M - 1);
          old[ni][v] = __builtin_nontemporal_load(c + (int64_t)i * ldc + j);
        }
      }
    } else {
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) old[ni][v] = 0.f;
    }
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int j = col0 + wn * 64 + ni * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = row0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        double sum;
        if constexpr (ACC64) sum = acc64[mi][ni][v]; else sum = (double)acc[mi][ni][v];
        const float x = (float)(alpha * sum + g.beta * (double)old[ni][v]);
        if (i < g.M && j < g.M) __builtin_nontemporal_store(x, c + (int64_t)i * ldc + j);
      }
    }
  }
}
#undef SYRK_STEP
#undef SYRK_WAIT
#undef SYRK_SLAB_PRODUCT

// C[i][j] = C[j][i] for every element whose tile (of BM x BM) lies above the diagonal of tiles:
// completes a factor that syrk_bf16_kernel has updated.  grid (ceil(n / 32),
// ceil(n / 32), batch), 256 threads; a 32 x 32 piece never straddles two tiles.
__global__ __launch_bounds__(256) void mirror_upper_tiles_kernel(float *c, int64_t batch_stride, int n) {
  __shared__ float t[32][33];
  const int i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;     // destination piece (i0, j0)
  if (i0 / BM >= j0 / BM) return;
  float *m = c + (int64_t)blockIdx.z * batch_stride;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int r = ty; r < 32; r += 8) {
    const int si = j0 + r, sj = i0 + tx;                       // source piece (j0, i0)
    if (si < n && sj < n) t[r][tx] = m[(int64_t)si * n + sj];
  }
  __syncthreads();
#pragma unroll
  for (int r = ty; r < 32; r += 8) {
    const int di = i0 + r, dj = j0 + tx;
    if (di < n && dj < n) m[(int64_t)di * n + dj] = t[tx][r];
  }
}

struct TransposeArgs {
  const BlockDesc *desc;
  const void *const *g_table;
  uint16_t *out;             // [slot][n][m]
  const float *scale;        // [slot] nullptr: out is bf16 like the block; else out = fp16(scale * block)
  int32_t m, n;
};

// out[slot][j][i] = G_block[i][j] (bf16 bits, or fp16 bits of the scaled value).  grid (ceil(n/64), ceil(m/64), blocks), 256 threads.
// Both sides move 16 bytes per lane (8 bf16 along the contiguous direction); the transposition
// itself happens in LDS.  Requires m % 8 == 0, n % 8 == 0, 16-byte aligned rows on both sides
// (the conditions of the bf16 matrix-core path, checked by the host).
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const TransposeArgs g) {
  __shared__ uint16_t tile[64][66];
  const BlockDesc d = g.desc[blockIdx.z];
  const uint16_t *src = reinterpret_cast<const uint16_t *>(g.g_table[d.param]) + d.offset;
  uint16_t *dst = g.out + (int64_t)blockIdx.z * g.m * g.n;
  const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int idx = threadIdx.x + 256 * h, r = idx >> 3, c = (idx & 7) * 8;
    const int i = i0 + r, j = j0 + c;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (i < g.m && j < g.n) v = *reinterpret_cast<const uint4 *>(src + (int64_t)i * d.ld + j);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
    if (g.scale) {      // uniform: bf16 -> scaled fp16 (exact unless it underflows: 8 significant bits go into 11)
      const float sc = g.scale[blockIdx.z];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const _Float16 lo = (_Float16)(__uint_as_float(w[e] << 16) * sc), hi = (_Float16)(__uint_as_float(w[e] & 0xffff0000u) * sc);
        w[e] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {      // rows of 66 elements are only 4-byte aligned
      *reinterpret_cast<uint32_t *>(&tile[r][c + 2 * e]) = w[e];
    }
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int idx = threadIdx.x + 256 * h, jr = idx >> 3, c = (idx & 7) * 8;   // output row jr, columns c .. c + 7
    const int j = j0 + jr, i = i0 + c;
    if (j >= g.n || i >= g.m) continue;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (uint32_t)tile[c + 2 * e][jr] | ((uint32_t)tile[c + 2 * e + 1][jr] << 16);
    typedef uint32_t tr_u32x4 __attribute__((ext_vector_type(4)));
    const tr_u32x4 packed = {w[0], w[1], w[2], w[3]};
    __builtin_nontemporal_store(packed, reinterpret_cast<tr_u32x4 *>(dst + (int64_t)j * g.m + i));
  }
}

}  // namespace shampoo
