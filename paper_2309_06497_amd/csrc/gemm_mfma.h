// Batched fp32 GEMM / SYRK on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32).
//
// One workgroup (256 threads = 4 wavefronts of 64) computes a 128 x 128 tile of
// C = alpha * A * B (+ beta * C).  Each wavefront owns a 64 x 64 quadrant as
// 2 x 2 MFMA tiles of 32 x 32.  Operand tiles are staged through LDS in
// k-major order ([k][row]), so that the 64 lanes of an MFMA operand read two
// rows of 32 consecutive floats, and are double-buffered against the global
// loads of the next k-slab.  Operands may be float32 or bfloat16 in memory
// (bf16 is widened exactly on the way into LDS); accumulation is float32.
//
// The operands of the Shampoo step (Sec. 2.3, 3.1.1 of the paper) map onto it as
//   L <- beta2 L + (1-beta2) G G^T   A(i,k) = G[i][k]   B(k,j) = G[j][k]   (both k-contiguous)
//   R <- beta2 R + (1-beta2) G^T G   A(i,k) = G[k][i]   B(k,j) = G[k][j]   (both row-contiguous)
//   T = Lbar G                       A(i,k) = Lbar[k][i] (symmetric)  B(k,j) = G[k][j]
//   P = T Rbar                       A(i,k) = T[i][k]   B(k,j) = Rbar[k][j]
//   X = Q f(Lambda) Q^T              A(i,k) = f_k Qt[k][i]  B(k,j) = Qt[k][j]
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace shampoo {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128;
constexpr int BN = 128;
constexpr int BK = 16;          // k-slab depth (multiple of 8)
constexpr int LDS_PAD = 4;
constexpr int LOAD_PASSES = BK / 8;          // 128 x BK floats = 256 threads x LOAD_PASSES float4
constexpr int GEMM_THREADS = 256;
constexpr int NUM_XCD = 8;

// How element (row, k) of an operand is laid out in memory.
//   K_CONTIG:   ptr[row * ld + k]     (a row-major matrix used as A, or B given transposed)
//   ROW_CONTIG: ptr[k * ld + row]     (a row-major matrix used as B, or A given transposed)
enum { K_CONTIG = 0, ROW_CONTIG = 1 };

enum { EPI_STORE = 0, EPI_STORE_NORM = 1, EPI_SYRK = 2 };

// One block of a 2-D parameter (Sec. 4.2.1 blocking): where it sits inside the
// caller's row-major tensor.
struct BlockDesc {
  int32_t param;   // index into the pointer table
  int32_t ld;      // columns of the parameter
  int64_t offset;  // row0 * ld + col0 (elements)
  int64_t state_offset;  // offset of the parameter inside the A / M state arrays, plus `offset`
};

// Where an operand of batch entry b lives.
struct Operand {
  const void *base;      // used when !from_table
  int64_t batch_stride;  // elements
  int32_t ld;
  int32_t from_table;    // 1: pointer = ptr_table[desc[b].param] + desc[b].offset, ld = desc[b].ld
};

struct GemmArgs {
  Operand a, b;
  float *c;
  int64_t c_batch_stride;
  int32_t ldc;
  int32_t M, N, K;
  float alpha, beta;
  double alpha_d, beta_d;       // used instead of alpha, beta by the ACC64 kernels
  const BlockDesc *desc;
  const void *const *ptr_table;
  const float *kscale;          // per-k multiplier of A (length K per batch entry), or nullptr
  int64_t kscale_stride;
  const int32_t *skip;          // per batch entry: nonzero = leave C untouched, or nullptr
  float *norm_partial;          // EPI_STORE_NORM: [batch][tiles] sums of squares of the stored tile
  int32_t tiles_m, tiles_n, tiles;  // tiles = tiles per batch entry (triangular count for SYRK)
  int32_t batch;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float(((uint32_t)h) << 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ void load4(const float *p, float v[4]) {
    const float4 t = *reinterpret_cast<const float4 *>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ float load1(const float *p) { return *p; }
};
template <> struct Elem<uint16_t> {
  static __device__ __forceinline__ void load4(const uint16_t *p, float v[4]) {
    const uint2 t = *reinterpret_cast<const uint2 *>(p);
    v[0] = __uint_as_float(t.x << 16);
    v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16);
    v[3] = __uint_as_float(t.y & 0xffff0000u);
  }
  static __device__ __forceinline__ float load1(const uint16_t *p) { return bf16_to_f32(*p); }
};

// Fetches one 128 x BK operand slab into registers (4 * LOAD_PASSES floats per thread)
// and later writes it into LDS in [k][row] order.
template <int ORIENT, typename T>
struct TileLoader {
  const T *ptr;     // operand origin for this batch entry, already offset to the tile's first row
  int ld;
  int rows_left;    // valid rows from the tile's first row
  int K;
  bool fast;        // whole tile in range and 4-element vectors aligned
  float r[LOAD_PASSES][4];

  __device__ __forceinline__ void init(const T *p, int ld_, int rows_left_, int K_) {
    ptr = p; ld = ld_; rows_left = rows_left_; K = K_;
    const bool aligned = ((ld_ & 3) == 0) && ((reinterpret_cast<uintptr_t>(p) & (4 * sizeof(T) - 1)) == 0);
    fast = aligned && rows_left_ >= 128 && (K_ % BK) == 0;
  }

  __device__ __forceinline__ void fetch(int k0, int tid) {
    if (ORIENT == K_CONTIG) {
      constexpr int TPR = BK / 4, RPP = GEMM_THREADS / TPR;   // threads per row, rows per pass
      const int row = tid / TPR, kq = (tid % TPR) * 4;
#pragma unroll
      for (int h = 0; h < LOAD_PASSES; ++h) {
        const int rr = row + RPP * h;
        if (fast) {
          Elem<T>::load4(ptr + (int64_t)rr * ld + k0 + kq, r[h]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            r[h][j] = (rr < rows_left && k0 + kq + j < K) ? Elem<T>::load1(ptr + (int64_t)rr * ld + k0 + kq + j) : 0.f;
        }
      }
    } else {
      const int kk = tid >> 5, r4 = (tid & 31) * 4;
#pragma unroll
      for (int h = 0; h < LOAD_PASSES; ++h) {
        const int k = k0 + kk + 8 * h;
        if (fast) {
          Elem<T>::load4(ptr + (int64_t)k * ld + r4, r[h]);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            r[h][j] = (k < K && r4 + j < rows_left) ? Elem<T>::load1(ptr + (int64_t)k * ld + r4 + j) : 0.f;
        }
      }
    }
  }

  // kscale: optional per-k multiplier (already offset to this batch entry), k0 = slab origin
  __device__ __forceinline__ void scale(const float *kscale, int k0, int tid) {
    if (ORIENT == K_CONTIG) {
      const int kq = (tid % (BK / 4)) * 4;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float s = (k0 + kq + j < K) ? kscale[k0 + kq + j] : 0.f;
#pragma unroll
        for (int h = 0; h < LOAD_PASSES; ++h) r[h][j] *= s;
      }
    } else {
      const int kk = tid >> 5;
#pragma unroll
      for (int h = 0; h < LOAD_PASSES; ++h) {
        const int k = k0 + kk + 8 * h;
        const float s = (k < K) ? kscale[k] : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) r[h][j] *= s;
      }
    }
  }

  __device__ __forceinline__ void store(float (*lds)[BM + LDS_PAD], int tid) const {
    if (ORIENT == K_CONTIG) {
      constexpr int TPR = BK / 4, RPP = GEMM_THREADS / TPR;
      const int row = tid / TPR, kq = (tid % TPR) * 4;
#pragma unroll
      for (int h = 0; h < LOAD_PASSES; ++h)
#pragma unroll
        for (int j = 0; j < 4; ++j) lds[kq + j][row + RPP * h] = r[h][j];
    } else {
      const int kk = tid >> 5, r4 = (tid & 31) * 4;
#pragma unroll
      for (int h = 0; h < LOAD_PASSES; ++h)
        *reinterpret_cast<float4 *>(&lds[kk + 8 * h][r4]) = make_float4(r[h][0], r[h][1], r[h][2], r[h][3]);
    }
  }
};

// Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each with its
// own L2.  Re-map so that every XCD works on one contiguous range of tiles:
// tiles that share operand panels then hit the same L2.
__device__ __forceinline__ int xcd_remap(int wg, int total) {
  const int per = (total + NUM_XCD - 1) / NUM_XCD;
  return (wg % NUM_XCD) * per + wg / NUM_XCD;
}

template <typename T>
__device__ __forceinline__ const T *operand_ptr(const Operand &o, const BlockDesc *desc,
                                                const void *const *table, int b, int &ld) {
  if (o.from_table) {
    const BlockDesc d = desc[b];
    ld = d.ld;
    return reinterpret_cast<const T *>(table[d.param]) + d.offset;
  }
  ld = o.ld;
  return reinterpret_cast<const T *>(o.base) + (int64_t)b * o.batch_stride;
}

// ACC64 = N > 0: after every N k-slabs of 16 the float32 MFMA accumulators are added
// into float64 registers and cleared, and the epilogue (alpha * acc + beta * C) is
// evaluated in float64 before the single rounding to float32.  Used for the
// factor updates: the first root refresh sees L = G G^T of a single gradient,
// whose condition number is the square of G's, and a plain float32 running sum
// over k would perturb its small eigenvalues by more than the parity budget.
template <int AO, int BO, typename TA, typename TB, int EPI, bool KSCALE, int ACC64 = 0>
__global__ __launch_bounds__(GEMM_THREADS, 2) void gemm_mfma_kernel(const GemmArgs g) {
  __shared__ __align__(16) float As[2][BK][BM + LDS_PAD];
  __shared__ __align__(16) float Bs[2][BK][BN + LDS_PAD];
  __shared__ float red[4];

  const int total = g.tiles * g.batch;
  const int logical = xcd_remap(blockIdx.x, total);
  if (logical >= total) return;
  const int b = logical / g.tiles;
  const int tile = logical - b * g.tiles;
  int ti, tj;
  if (EPI == EPI_SYRK) {
    // lower-triangular tile index: tile = ti (ti + 1) / 2 + tj, tj <= ti
    ti = (int)((sqrtf(8.f * (float)tile + 1.f) - 1.f) * 0.5f);
    while ((ti + 1) * (ti + 2) / 2 <= tile) ++ti;
    while (ti * (ti + 1) / 2 > tile) --ti;
    tj = tile - ti * (ti + 1) / 2;
  } else {
    ti = tile / g.tiles_n;
    tj = tile - ti * g.tiles_n;
  }
  if (g.skip != nullptr && g.skip[b] != 0) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = ti * BM, col0 = tj * BN;

  int lda, ldb;
  const TA *pa = operand_ptr<TA>(g.a, g.desc, g.ptr_table, b, lda);
  const TB *pb = operand_ptr<TB>(g.b, g.desc, g.ptr_table, b, ldb);
  TileLoader<AO, TA> la;
  TileLoader<BO, TB> lb;
  la.init(pa + (AO == K_CONTIG ? (int64_t)row0 * lda : (int64_t)row0), lda, g.M - row0, g.K);
  lb.init(pb + (BO == K_CONTIG ? (int64_t)col0 * ldb : (int64_t)col0), ldb, g.N - col0, g.K);
  const float *ks = KSCALE ? g.kscale + (int64_t)b * g.kscale_stride : nullptr;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  double acc64[ACC64 ? 2 : 1][ACC64 ? 2 : 1][ACC64 ? 16 : 1];
  if (ACC64) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc64[ACC64 ? i : 0][ACC64 ? j : 0][ACC64 ? v : 0] = 0.0;
  }

  const int nk = (g.K + BK - 1) / BK;
  la.fetch(0, tid);
  lb.fetch(0, tid);
  if (KSCALE) la.scale(ks, 0, tid);
  la.store(As[0], tid);
  lb.store(Bs[0], tid);
  __syncthreads();

  const int arow = wm * 64 + (lane & 31);
  const int bcol = wn * 64 + (lane & 31);
  const int khalf = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      la.fetch((kt + 1) * BK, tid);
      lb.fetch((kt + 1) * BK, tid);
    }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const float a0 = As[cur][kk + khalf][arow];
      const float a1 = As[cur][kk + khalf][arow + 32];
      const float b0 = Bs[cur][kk + khalf][bcol];
      const float b1 = Bs[cur][kk + khalf][bcol + 32];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
    if (ACC64 && ((kt + 1) % (ACC64 ? ACC64 : 1) == 0 || kt + 1 == nk)) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            acc64[ACC64 ? i : 0][ACC64 ? j : 0][ACC64 ? v : 0] += (double)acc[i][j][v];
            acc[i][j][v] = 0.f;
          }
    }
    if (kt + 1 < nk) {
      if (KSCALE) la.scale(ks, (kt + 1) * BK, tid);
      la.store(As[cur ^ 1], tid);
      lb.store(Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }

  // ---- epilogue.  Accumulator element v of MFMA tile (mi, ni) is
  //      row = wm*64 + mi*32 + 8*(v/4) + 4*(lane/32) + v%4, col = wn*64 + ni*32 + lane%32.
  float *c = g.c + (int64_t)b * g.c_batch_stride;
  const int ldc = g.ldc;
  float ss = 0.f;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
      const int j = col0 + wn * 64 + ni * 32 + (lane & 31);
      // EPI_SYRK with a nonzero beta: the 16 old values of an MFMA tile are requested before
      // its first store.  The mirrored stores may alias later loads, so interleaved they
      // would cost one memory round trip per element instead of one per tile.
      float old[EPI == EPI_SYRK ? 16 : 1];
      if (EPI == EPI_SYRK) {
        const bool need = ACC64 ? (g.beta_d != 0.0) : (g.beta != 0.f);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = row0 + wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          old[EPI == EPI_SYRK ? v : 0] = (need && i < g.M && j <= i) ? c[(int64_t)i * ldc + j] : 0.f;
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int ibase = row0 + wm * 64 + mi * 32 + 8 * q + 4 * (lane >> 5);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = ibase + e;
          float v = g.alpha * acc[mi][ni][4 * q + e];
          if (i < g.M && j < g.N) {
            if (EPI == EPI_SYRK) {
              // only the lower triangle is computed; its mirror image is written with the
              // same bits so the factor stays exactly symmetric
              if (j <= i) {
                const float o = old[EPI == EPI_SYRK ? 4 * q + e : 0];
                if (ACC64) v = (float)(g.alpha_d * acc64[ACC64 ? mi : 0][ACC64 ? ni : 0][ACC64 ? 4 * q + e : 0] + g.beta_d * (double)o);
                else v += g.beta * o;
                c[(int64_t)i * ldc + j] = v;
                if (j < i) c[(int64_t)j * ldc + i] = v;
              }
            } else {
              c[(int64_t)i * ldc + j] = v;
              if (EPI == EPI_STORE_NORM) ss += v * v;
            }
          }
        }
      }
    }
  if (EPI == EPI_STORE_NORM) {
    // fixed-order reduction: lanes by xor-shuffle, then the 4 wavefronts in order
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (tid == 0) g.norm_partial[(int64_t)b * g.tiles + tile] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

}  // namespace shampoo
