// Host side of libshampoo: configuration checks, block planner, workspace
// layout, kernel launches and the extern "C" boundary declared in shampoo.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <new>
#include <utility>
#include <vector>

#include "../../include/shampoo.h"
#include "block_step_small.h"
#include "congruence_f64.h"
#include "diag_shampoo.h"
#include "eigh_jacobi.h"
#include "elementwise.h"
#include "gemm_f16x2.h"
#include "gemm_mfma.h"
#include "newton_root.h"
#include "syrk_bf16.h"
#include "tensor_blocks.h"

using namespace shampoo;

// Scratch of shampoo_root_inverse_static: the block solver's working arrays (float64 copy of
// the matrices, accumulated rotations, pivot blocks, flags) for as many matrices at a time as
// fit.  One copy per GPU the library runs on, held until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress: kernels are given the address obtained there.
static __device__ __align__(256) unsigned char scratch[SHAMPOO_STATIC_SCRATCH_BYTES];

namespace {

constexpr int64_t MAX_BLOCK_SIZE = 8192;
constexpr size_t ALIGN = 256;
constexpr size_t EIG_CHUNK_BYTES = (size_t)3 << 30;   // W + Qt of one chunk of the block solver

inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

#define HIP_TRY(expr)                          \
  do {                                         \
    hipError_t e_ = (expr);                    \
    if (e_ != hipSuccess) return SHAMPOO_ERR_HIP; \
  } while (0)

// ---------------------------------------------------------------------------
// Planner (Sec. 4.2.1 blocking)
// ---------------------------------------------------------------------------
struct Block {
  int32_t param;
  int64_t row0, col0;
  int32_t m, n;
  int32_t bucket, slot;
  // tensor blocks (Sec. 2.3): start and size along the third and fourth dimension, and where
  // the block sits in the block-contiguous copy of the parameter that the kernels work on
  int64_t s3 = 0, s4 = 0;
  int32_t d3 = 1, d4 = 1;
  int64_t voff = 0;
  bool tensor = false;
};
// How a parameter is worked on after merging of small dimensions (Sec. 4.2.1).
enum { P_VECTOR = 0, P_MATRIX = 1, P_TENSOR = 2 };
struct PShape {
  int kind = P_VECTOR;
  int64_t rows = 1, cols = 1;   // P_MATRIX: the (merged) shape; P_VECTOR: rows = length
  int64_t d[4] = {1, 1, 1, 1};  // P_TENSOR: the merged dimensions
  int modes = 0;                // P_TENSOR: 3 or 4, or 1 when everything merged into one dimension
  int64_t elems() const { return kind == P_TENSOR ? d[0] * d[1] * d[2] * d[3] : rows * cols; }
};
struct Bucket {
  int32_t m, n, count;
  // byte offsets into the workspace
  size_t off_L, off_R, off_Linv, off_Rinv, off_P, off_desc, off_sgp, off_sshp, off_scale, off_norms;
  // bf16 gradients, bf16_mfma buckets: both roots as two scaled fp16 planes, what the scales
  // are made from (matrix_stats_kernel of both roots, max |G| per piece of a block) and the
  // scales themselves
  size_t off_Linv2h = 0, off_Rinv2h = 0, off_stat_l = 0, off_stat_r = 0, off_gmaxp = 0, off_s_g = 0, off_inv_g2 = 0, off_t_scale = 0, off_inv_ts = 0;
  size_t off_QtL = 0, off_QtR = 0;   // warm start: eigenvectors of the previous refresh, [count][np][np] float32
  size_t off_Gt = 0;     // 16-bit transpose of the bucket's gradient blocks (bf16, or scaled fp16 where the fp16 products follow), made by the factor update and
                         // read again by the first preconditioning product of the same step
  bool planes = false;
  EwGeom geom;
  int32_t tiles_m, tiles_n;
  bool bf16_mfma;   // shapes, offsets and leading dimensions allow the bf16 matrix-core factor update
  // diagonal Shampoo (Sec. 4.2.3): the factor of that side is a vector (its diagonal); such a
  // bucket holds whole parameters, one per slot
  bool diagL = false, diagR = false;
  int32_t col_segs = 1, rows_per_seg = 0;   // row segments of the column-sum reduction
  // tensor blocks d1 x d2 x d3 (x d4): the elementwise kernels see them as m x n = d1 x (d2 d3 d4)
  // matrices inside a block-contiguous copy of the parameter; L belongs to the first
  // dimension, R to the last, mid[0] (and mid[1] for order 4) to the ones between
  bool t3 = false;
  int32_t td[4] = {1, 1, 1, 1}, modes = 0;
  size_t off_mid[2] = {0, 0}, off_midinv[2] = {0, 0}, off_desc3 = 0;
  int32_t split3 = 1;   // row ranges of the (N / d_last) x d_last unfolding whose Gram matrices are formed separately
  bool whole() const { return diagL || diagR; }
  int32_t dlast() const { return modes > 1 ? td[modes - 1] : 1; }
  int32_t rdim() const { return t3 ? dlast() : n; }
  size_t l_elems() const { return diagL ? (size_t)m : (size_t)m * m; }
  size_t r_elems() const { return diagR ? (size_t)n : (size_t)rdim() * rdim(); }
};
struct Plan {
  std::vector<Block> blocks;
  std::vector<Bucket> buckets;
  std::vector<std::vector<int32_t>> param_blocks;  // per parameter: indices into blocks (row-major)
  std::vector<int64_t> param_state_offset;         // element offset of each parameter in A / M
  std::vector<DiagChunk> diag_chunks;   // 1-D parameters
  std::vector<DiagChunk> prep_chunks;   // 2-D parameters, flat (used by the l2 / filtering pre-pass)
  std::vector<PShape> pshape;           // per parameter
  int64_t total_elems = 0;
};

// Merging of small dimensions (Sec. 4.2.1) and the resulting kind of parameter.  Returns
// SHAMPOO_OK, or the error for a shape that is out of range.
int param_shape(const shampoo_config *c, int i, PShape &ps) {
  const int nd = c->ndim[i];
  if (nd < 1 || nd > SHAMPOO_MAX_NDIM) return SHAMPOO_ERR_SHAPE;
  const int64_t *sh = c->shape + (size_t)SHAMPOO_MAX_NDIM * i;
  for (int k = 0; k < nd; ++k) {
    if (sh[k] < 1) return SHAMPOO_ERR_SHAPE;
    if (sh[k] > (int64_t)1 << 30) return SHAMPOO_ERR_UNSUPPORTED;
  }
  ps = PShape();
  if (nd == 1) { ps.kind = P_VECTOR; ps.rows = sh[0]; return SHAMPOO_OK; }
  if (nd == 2) { ps.kind = P_MATRIX; ps.rows = sh[0]; ps.cols = sh[1]; return SHAMPOO_OK; }
  int64_t merged[SHAMPOO_MAX_NDIM];
  int cnt = 0;
  int64_t cur = sh[0];
  for (int k = 1; k < nd; ++k) {
    // a dimension of size 1 changes no product and always merges
    if (cur * sh[k] <= c->block_size || sh[k] == 1 || cur == 1) cur *= sh[k];
    else { merged[cnt++] = cur; cur = sh[k]; }
  }
  merged[cnt++] = cur;
  if (cnt == 2) { ps.kind = P_MATRIX; ps.rows = merged[0]; ps.cols = merged[1]; return SHAMPOO_OK; }
  ps.kind = P_TENSOR;
  ps.modes = cnt;
  for (int k = 0; k < cnt; ++k) ps.d[k] = merged[k];
  if ((double)ps.d[0] * (double)ps.d[1] * (double)ps.d[2] * (double)ps.d[3] > (double)((int64_t)1 << 40)) return SHAMPOO_ERR_UNSUPPORTED;
  // one block is indexed with 32-bit products of its sizes
  double block_elems = 1.0;
  for (int k = 0; k < cnt; ++k) block_elems *= (double)std::min<int64_t>(ps.d[k], c->block_size);
  if (block_elems > (double)(1 << 30)) return SHAMPOO_ERR_UNSUPPORTED;
  return SHAMPOO_OK;
}

// p = 1 / r when that is 1, 2, 4 or 8 (the powers the coupled Newton iteration forms by
// repeated squaring), else 0
int newton_p_of(float r) {
  for (int p : {1, 2, 4, 8})
    if (std::fabs(1.0 / (double)r - (double)p) <= 1e-4 * p) return p;
  return 0;
}

int check_config(const shampoo_config *c) {
  if (!c || !c->ndim || !c->shape) return SHAMPOO_ERR_NULL;
  if (c->n_params < 1) return SHAMPOO_ERR_SHAPE;
  if (c->block_size < 1) return SHAMPOO_ERR_SHAPE;
  if (c->block_size > MAX_BLOCK_SIZE) return SHAMPOO_ERR_UNSUPPORTED;
  for (int i = 0; i < c->n_params; ++i) {
    PShape ps;
    const int rc = param_shape(c, i, ps);
    if (rc) return rc;
  }
  if (!(c->beta2 > 0.f && c->beta2 <= 1.f)) return SHAMPOO_ERR_HYPER;
  if (!(c->epsilon > 0.f) || !std::isfinite(c->epsilon)) return SHAMPOO_ERR_HYPER;
  if (!(c->root_exponent > 0.f) || !std::isfinite(c->root_exponent)) return SHAMPOO_ERR_HYPER;
  if (c->precondition_frequency < 1 || c->start_preconditioning_step < 0) return SHAMPOO_ERR_HYPER;
  if (!(c->graft_epsilon >= 0.f) || !std::isfinite(c->graft_epsilon)) return SHAMPOO_ERR_HYPER;
  if (!(c->momentum >= 0.f && c->momentum < 1.f)) return SHAMPOO_ERR_HYPER;
  if (c->grad_dtype != SHAMPOO_GRAD_F32 && c->grad_dtype != SHAMPOO_GRAD_BF16) return SHAMPOO_ERR_HYPER;
  if (!(c->beta1 >= 0.f && c->beta1 < 1.f)) return SHAMPOO_ERR_HYPER;
  if (!(c->weight_decay >= 0.f) || !std::isfinite(c->weight_decay)) return SHAMPOO_ERR_HYPER;
  if (c->grafting_type < SHAMPOO_GRAFT_ADAGRAD || c->grafting_type > SHAMPOO_GRAFT_ADAM) return SHAMPOO_ERR_HYPER;
  if ((c->grafting_type == SHAMPOO_GRAFT_RMSPROP || c->grafting_type == SHAMPOO_GRAFT_ADAM) &&
      !(c->grafting_beta2 > 0.f && c->grafting_beta2 <= 1.f))
    return SHAMPOO_ERR_HYPER;
  if (c->large_dim_method < SHAMPOO_LARGE_DIM_BLOCKING || c->large_dim_method > SHAMPOO_LARGE_DIM_DIAGONAL)
    return SHAMPOO_ERR_HYPER;
  if (c->large_dim_method == SHAMPOO_LARGE_DIM_DIAGONAL)
    for (int i = 0; i < c->n_params; ++i) {
      PShape ps;
      param_shape(c, i, ps);
      if (ps.kind == P_MATRIX && (ps.rows > INT32_MAX / 2 || ps.cols > INT32_MAX / 2)) return SHAMPOO_ERR_UNSUPPORTED;
    }
  if (c->root_method != SHAMPOO_ROOT_EIGH && c->root_method != SHAMPOO_ROOT_NEWTON) return SHAMPOO_ERR_HYPER;
  if (c->precond_matrix_cores != SHAMPOO_MATRIX_CORES_AUTO && c->precond_matrix_cores != SHAMPOO_MATRIX_CORES_FP32)
    return SHAMPOO_ERR_HYPER;
  if (c->root_method == SHAMPOO_ROOT_NEWTON) {
    if (c->newton_tolerance < 0.f || !std::isfinite(c->newton_tolerance)) return SHAMPOO_ERR_HYPER;
    if (c->newton_max_iterations < 0 || c->newton_max_iterations > 1000) return SHAMPOO_ERR_HYPER;
    if (newton_p_of(c->root_exponent) == 0) return SHAMPOO_ERR_UNSUPPORTED;
    for (int i = 0; i < c->n_params; ++i) {
      PShape ps;
      param_shape(c, i, ps);
      if (ps.kind == P_TENSOR && newton_p_of(2.f * c->root_exponent / (float)ps.modes) == 0) return SHAMPOO_ERR_UNSUPPORTED;
    }
  }
  return SHAMPOO_OK;
}

EwGeom make_geom(int m, int n) {
  EwGeom g;
  const int vecs = (n + 3) / 4;
  int lx = 0;
  while ((1 << lx) < vecs && lx < 6) ++lx;
  g.lanes_x_log2 = lx;
  const int ny = EW_THREADS >> lx;
  const int cols_per_pass = 4 << lx;
  const int passes = (n + cols_per_pass - 1) / cols_per_pass;
  // about 8192 elements per workgroup, a whole number of thread rows
  int rows = std::max(1, 8192 / (cols_per_pass * passes));
  rows = (rows + ny - 1) / ny * ny;
  g.rows_per_wg = rows;
  g.chunks = (m + rows - 1) / rows;
  return g;
}

void make_plan(const shampoo_config *c, Plan &p) {
  const int64_t b = c->block_size;
  // (m, n, diagonal sides | tensor, d2, d3, d4) -> bucket
  std::map<std::tuple<int, int, int, int, int, int>, int> bucket_of;
  p.param_blocks.assign(c->n_params, {});
  p.param_state_offset.assign(c->n_params, 0);
  p.pshape.assign(c->n_params, PShape());
  int64_t off = 0;
  auto bucket_for = [&](int m, int n, int flags, int d2, int d3, int d4, int modes) {
    auto key = std::make_tuple(m, n, flags, d2, d3, d4);
    auto it = bucket_of.find(key);
    if (it == bucket_of.end()) {
      Bucket bk{};
      bk.m = m; bk.n = n; bk.count = 0;
      bk.diagL = (flags & 1) != 0; bk.diagR = (flags & 2) != 0;
      bk.t3 = (flags & 4) != 0; bk.td[0] = m; bk.td[1] = d2; bk.td[2] = d3; bk.td[3] = d4; bk.modes = modes;
      bucket_of[key] = (int)p.buckets.size();
      p.buckets.push_back(bk);
      it = bucket_of.find(key);
    }
    return it->second;
  };
  for (int i = 0; i < c->n_params; ++i) {
    p.param_state_offset[i] = off;
    PShape &ps = p.pshape[i];
    param_shape(c, i, ps);
    const int64_t rows = ps.rows, cols = ps.cols;
    const bool large = ps.kind == P_MATRIX && (rows > b || cols > b);
    // 1-D parameters, and under the "adagrad" large-dimension method (Sec. 4.2.2) every
    // matrix with a dimension above the block size, take the diagonal path on their entries
    if (ps.kind == P_VECTOR || (large && c->large_dim_method == SHAMPOO_LARGE_DIM_ADAGRAD)) {
      const int64_t len = rows * cols;
      for (int64_t s = 0; s < len; s += DIAG_CHUNK) {
        DiagChunk dc;
        dc.param = i;
        dc.len = (int32_t)std::min<int64_t>(DIAG_CHUNK, len - s);
        dc.start = s;
        dc.state_offset = off + s;
        p.diag_chunks.push_back(dc);
      }
      off += (len + 3) / 4 * 4;
      continue;
    }
    const int64_t elems = ps.elems();
    for (int64_t st = 0; st < elems; st += DIAG_CHUNK) {
      DiagChunk dc;
      dc.param = i;
      dc.len = (int32_t)std::min<int64_t>(DIAG_CHUNK, elems - st);
      dc.start = st;
      dc.state_offset = off + st;
      p.prep_chunks.push_back(dc);
    }
    if (ps.kind == P_TENSOR) {
      // every dimension cut into pieces of at most b; blocks in row-major order of their
      // indices.  All pieces before the last one of a dimension are full, which gives the
      // offset of a block inside the block-contiguous copy in closed form.
      const int64_t D1 = ps.d[0], D2 = ps.d[1], D3 = ps.d[2], D4 = ps.d[3];
      const int64_t k1n = (D1 + b - 1) / b, k2n = (D2 + b - 1) / b, k3n = (D3 + b - 1) / b, k4n = (D4 + b - 1) / b;
      for (int64_t k1 = 0; k1 < k1n; ++k1)
        for (int64_t k2 = 0; k2 < k2n; ++k2)
          for (int64_t k3 = 0; k3 < k3n; ++k3)
            for (int64_t k4 = 0; k4 < k4n; ++k4) {
              Block blk;
              blk.param = i; blk.tensor = true;
              blk.row0 = k1 * b; blk.col0 = k2 * b; blk.s3 = k3 * b; blk.s4 = k4 * b;
              blk.m = (int32_t)std::min<int64_t>(b, D1 - blk.row0);
              blk.n = (int32_t)std::min<int64_t>(b, D2 - blk.col0);
              blk.d3 = (int32_t)std::min<int64_t>(b, D3 - blk.s3);
              blk.d4 = (int32_t)std::min<int64_t>(b, D4 - blk.s4);
              blk.voff = blk.row0 * D2 * D3 * D4 + (int64_t)blk.m * (blk.col0 * D3 * D4) +
                         (int64_t)blk.m * blk.n * (blk.s3 * D4) + (int64_t)blk.m * blk.n * blk.d3 * blk.s4;
              blk.bucket = bucket_for(blk.m, blk.n * blk.d3 * blk.d4, 4, blk.n, blk.d3, blk.d4, ps.modes);
              blk.slot = p.buckets[blk.bucket].count++;
              p.param_blocks[i].push_back((int32_t)p.blocks.size());
              p.blocks.push_back(blk);
            }
      off += (elems + 3) / 4 * 4;
      continue;
    }
    // diagonal Shampoo (Sec. 4.2.3): the parameter stays whole, one "block"
    const bool whole = large && c->large_dim_method == SHAMPOO_LARGE_DIM_DIAGONAL;
    const int64_t bb = whole ? std::max(rows, cols) : b;
    const int flags = whole ? ((rows > b ? 1 : 0) | (cols > b ? 2 : 0)) : 0;
    const int64_t km = (rows + bb - 1) / bb, kn = (cols + bb - 1) / bb;
    for (int64_t bi = 0; bi < km; ++bi)
      for (int64_t bj = 0; bj < kn; ++bj) {
        Block blk;
        blk.param = i;
        blk.row0 = bi * bb;
        blk.col0 = bj * bb;
        blk.m = (int32_t)std::min<int64_t>(bb, rows - blk.row0);
        blk.n = (int32_t)std::min<int64_t>(bb, cols - blk.col0);
        blk.bucket = bucket_for(blk.m, blk.n, flags, 1, 1, 1, 0);
        blk.slot = p.buckets[blk.bucket].count++;
        p.param_blocks[i].push_back((int32_t)p.blocks.size());
        p.blocks.push_back(blk);
      }
    off += (rows * cols + 3) / 4 * 4;
  }
  p.total_elems = off;
  for (auto &bk : p.buckets)
    bk.bf16_mfma = (bk.m % 8 == 0) && (bk.n % 8 == 0) && bk.count <= 65535 && !bk.whole() && !bk.t3;
  for (const Block &blk : p.blocks) {
    if (blk.tensor) continue;
    const int64_t ld = p.pshape[blk.param].cols;
    if (ld % 8 != 0 || (blk.row0 * ld + blk.col0) % 8 != 0) p.buckets[blk.bucket].bf16_mfma = false;
  }
  for (auto &bk : p.buckets) {
    if (bk.t3 && bk.modes >= 3) {
      // the factor of the last dimension sums over N / d_last rows into one small tile per
      // block: split the rows (whole slices of the first index) so that the launch fills the GPU
      const int64_t inner = (int64_t)bk.n / bk.dlast();   // rows of the unfolding per slice of the first index
      for (int sdiv = 1; sdiv <= std::min(bk.m, 64); ++sdiv)
        if (bk.m % sdiv == 0 && (int64_t)(bk.m / sdiv) * inner >= 64 && (int64_t)sdiv * bk.dlast() <= (int64_t)bk.m * inner &&
            (int64_t)bk.count * sdiv <= 1 << 20)
          bk.split3 = sdiv;
    }
    bk.geom = make_geom(bk.m, bk.n);
    bk.tiles_m = (bk.m + BM - 1) / BM;
    bk.tiles_n = (bk.n + BN - 1) / BN;
    bk.col_segs = std::max(1, std::min(64, bk.m / 256));
    bk.rows_per_seg = (bk.m + bk.col_segs - 1) / bk.col_segs;
  }
}

// Whole-parameter and tensor buckets are launched with the block index as grid.y / grid.z.
int check_plan(const Plan &p) {
  for (const auto &b : p.buckets)
    if ((b.whole() || b.t3) && b.count > 65535) return SHAMPOO_ERR_UNSUPPORTED;
  return SHAMPOO_OK;
}

// ---------------------------------------------------------------------------
// Root-inverse workspace (shared by the optimizer and the stand-alone call)
// ---------------------------------------------------------------------------
constexpr int CONGRUENCE_PANEL = 256;   // columns of T = A Qt^T formed at a time (warm start)

struct EigLayout {
  int32_t np = 0, chunk = 0;
  bool warm = false;       // block solver: room for the float64 panel of the congruence W = Qt A Qt^T
  size_t off_w = 0, off_qt = 0, off_j = 0, off_ident = 0, off_j16 = 0, off_rot = 0, off_dmax = 0, off_failed = 0, off_f = 0, off_t = 0;
  size_t bytes = 0;
};

// Offsets for chunks of `chunk` matrices of the block solver (np already set).
void eig_offsets(EigLayout &e) {
  const size_t mat = (size_t)e.np * e.np * sizeof(float);
  size_t off = 0;
  e.off_w = off; off += align_up(2 * mat * e.chunk);
  e.off_qt = off; off += align_up(mat * e.chunk);
  const int hp = e.np / JAC_PIV;
  // rotation blocks and flags of two rounds (the Q^T update of a meeting of two super-columns
  // reads both): [2][chunk][hp]
  e.off_j = off; off += align_up(2 * (size_t)e.chunk * hp * JAC_PIV * JAC_PIV * sizeof(float));
  e.off_ident = off; off += align_up(2 * (size_t)e.chunk * hp * sizeof(int32_t));
  e.off_j16 = off; off += align_up(2 * (size_t)e.chunk * hp * 2 * JAC_PIV * JAC_PIV * sizeof(uint16_t));   // the same blocks, transposed, as two fp16 planes
  e.off_rot = off; off += align_up((size_t)e.chunk * JAC_OUTER_SWEEPS * sizeof(int32_t));
  e.off_dmax = off; off += align_up(2 * (size_t)e.chunk * sizeof(float));   // largest |diagonal entry|, largest absolute row sum
  e.off_failed = off; off += align_up(3 * (size_t)e.chunk * sizeof(int32_t));   // failed, done, skip (failed | done)
  e.off_f = off; off += align_up(2 * (size_t)e.chunk * e.np * sizeof(float));   // weights of the reconstruction; float32 eigenvalues of matrices that skip the float64 phase
  if (e.warm) { e.off_t = off; off += align_up((size_t)e.chunk * e.np * std::min(e.np, CONGRUENCE_PANEL) * sizeof(double)); }
  e.bytes = off;
}

// budget: bytes that the W and Qt arrays of one chunk may take (the other arrays are small);
// hard_cap != 0: the whole layout must fit into that many bytes (bytes = 0 in the result if
// not even one matrix does).
EigLayout eig_layout(int n, int batch, size_t budget = EIG_CHUNK_BYTES, size_t hard_cap = 0, bool warm = false) {
  EigLayout e;
  (void)warm;
  e.warm = n > JAC_SMALL_MAX;   // the float64 panel serves the warm start and the mixed-precision cold solve alike
  if (n <= JAC_SMALL_MAX) {     // LDS solver: no scratch in device memory
    e.chunk = batch;
    e.off_failed = 0;
    e.bytes = align_up((size_t)std::max(batch, 1) * sizeof(int32_t));
    return e;
  }
  e.np = (n + JAC_PIV - 1) / JAC_PIV * JAC_PIV;
  const size_t mat = (size_t)e.np * e.np * sizeof(float);
  // W is float64, Qt float32: 3 float-sized matrices per solve
  e.chunk = (int)std::max<size_t>(1, std::min<size_t>(std::min<size_t>((size_t)batch, 32768), budget / (3 * mat)));
  eig_offsets(e);
  if (hard_cap) {
    while (e.bytes > hard_cap && e.chunk > 1) { --e.chunk; eig_offsets(e); }
    if (e.bytes > hard_cap) e.bytes = 0;
  }
  return e;
}

template <int AO, int BO, typename TA, typename TB, int EPI, bool KS, int ACC64 = 0>
int launch_gemm(GemmArgs &g, hipStream_t s) {
  const int64_t total = (int64_t)g.tiles * g.batch;
  if (total <= 0) return SHAMPOO_OK;
  if (total > (int64_t)1 << 30) return SHAMPOO_ERR_UNSUPPORTED;
  const int per = (int)((total + NUM_XCD - 1) / NUM_XCD);
  hipLaunchKernelGGL((gemm_mfma_kernel<AO, BO, TA, TB, EPI, KS, ACC64>), dim3(per * NUM_XCD), dim3(GEMM_THREADS), 0, s, g);
  HIP_TRY(hipGetLastError());
  return SHAMPOO_OK;
}

int launch_fill(float *p, float v, int64_t n, hipStream_t s) {
  if (n <= 0) return SHAMPOO_OK;
  hipLaunchKernelGGL(fill_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, v, n);
  HIP_TRY(hipGetLastError());
  return SHAMPOO_OK;
}

constexpr int JAC_STREAMS = 4;   // sub-chunks of the block solver that run concurrently

// Helper streams (default priority) and fork / join events of the block solver.
struct AuxStreams {
  hipStream_t stream[JAC_STREAMS - 1] = {};
  hipEvent_t fork = nullptr, join[JAC_STREAMS - 1] = {};
  int state = 0;   // 0 = not tried, 1 = ready, -1 = unavailable (everything then runs on the caller's stream)
  bool ready() {
    if (state == 0) {
      state = 1;
      if (hipEventCreateWithFlags(&fork, hipEventDisableTiming) != hipSuccess) { fork = nullptr; state = -1; }
      for (int i = 0; i < JAC_STREAMS - 1 && state == 1; ++i) {
        if (hipStreamCreateWithFlags(&stream[i], hipStreamNonBlocking) != hipSuccess) { stream[i] = nullptr; state = -1; }
        else if (hipEventCreateWithFlags(&join[i], hipEventDisableTiming) != hipSuccess) { join[i] = nullptr; state = -1; }
      }
      if (state == -1) release();
    }
    return state == 1;
  }
  // Waits for the helper streams' work, then frees streams and events.
  void release() {
    for (int i = 0; i < JAC_STREAMS - 1; ++i) {
      if (stream[i]) { (void)hipStreamSynchronize(stream[i]); (void)hipStreamDestroy(stream[i]); stream[i] = nullptr; }
      if (join[i]) { (void)hipEventDestroy(join[i]); join[i] = nullptr; }
    }
    if (fork) { (void)hipEventDestroy(fork); fork = nullptr; }
  }
};

// What the stand-alone entry points keep per GPU until the process ends.
constexpr int MAX_DEVICES = 64;
struct PerDevice {
  std::mutex mutex;
  AuxStreams aux;                      // helper streams of shampoo_root_inverse
  unsigned char *scratch = nullptr;    // device address of `scratch` on this GPU
};
PerDevice per_device[MAX_DEVICES];

// Block-Jacobi root inverse of `cnt` matrices, using workspace slots [slot0, slot0 + cnt).
// Warm start (WarmStart::qt != nullptr): the rows of Qt are kept between solves in the caller's
// array; with `start` set the solve begins at W = Qt A Qt^T instead of W = A, Qt = I.
struct WarmStart {
  float *qt = nullptr;          // [batch][np][np]: eigenvectors, read (start) and written
  bool start = false;
  int32_t *sweeps = nullptr;    // optional [batch]: sweeps in which anything rotated
  bool young = false;           // the factors have seen few gradient columns (young_factor): badly conditioned, they
                                // take three more sweeps than well-conditioned ones, and a cold solve then runs two
                                // more of them in float32, where a sweep costs half of what it does in float64
                                // (256 factors of a single gradient, n = 1024: 345 -> 322 ms; well-conditioned
                                // factors would pay for the two sweeps and gain nothing: 268 -> 293 ms)
};

// One sub-chunk of a block-Jacobi solve: `cnt` matrices in workspace slots [slot0, slot0 + cnt),
// all of its work on one stream.  The solve is enqueued phase by phase (begin, then sweep after
// sweep, then finish) so that the caller can interleave the sub-chunks of a chunk: the host
// needs a few microseconds per launch and a solve is thousands of launches, so a sub-chunk
// that were enqueued whole before the next one would run alone for most of its time.
struct BlockSolve {
  const float *a; int n, cnt; float eps, r, scale; float *x, *lambda; int32_t *failed_user;
  unsigned long long *fail_count; unsigned char *ws; const EigLayout *e; int slot0; hipStream_t s;
  const int32_t *only; WarmStart warm_in;
  // derived
  int np = 0, nblk = 0, hp = 0, sw = 0;
  bool warm = false;
  double *w = nullptr; float *w32 = nullptr, *qt = nullptr, *fv = nullptr, *d32 = nullptr;
  int32_t *rot = nullptr, *failed = nullptr, *done = nullptr, *skipc = nullptr;
  float *jslot[2] = {nullptr, nullptr}; int32_t *islot[2] = {nullptr, nullptr}; uint16_t *hslot[2] = {nullptr, nullptr};
  BlockJacArgs ja{};

  int begin() {
    np = e->np; nblk = np / JAC_NB; hp = nblk / 2;
    w = reinterpret_cast<double *>(ws + e->off_w) + (int64_t)slot0 * np * np;
    qt = warm_in.qt ? warm_in.qt : reinterpret_cast<float *>(ws + e->off_qt) + (int64_t)slot0 * np * np;
    warm = warm_in.qt && warm_in.start && e->warm;
    for (int k = 0; k < 2; ++k) {
      jslot[k] = reinterpret_cast<float *>(ws + e->off_j) + ((int64_t)k * e->chunk + slot0) * hp * JAC_PIV * JAC_PIV;
      islot[k] = reinterpret_cast<int32_t *>(ws + e->off_ident) + ((int64_t)k * e->chunk + slot0) * hp;
      hslot[k] = reinterpret_cast<uint16_t *>(ws + e->off_j16) + ((int64_t)k * e->chunk + slot0) * hp * 2 * JAC_PIV * JAC_PIV;
    }
    rot = reinterpret_cast<int32_t *>(ws + e->off_rot) + (int64_t)slot0 * JAC_OUTER_SWEEPS;
    float *dmax = reinterpret_cast<float *>(ws + e->off_dmax) + slot0;
    failed = reinterpret_cast<int32_t *>(ws + e->off_failed) + slot0;
    done = failed + e->chunk; skipc = failed + 2 * e->chunk;
    fv = reinterpret_cast<float *>(ws + e->off_f) + (int64_t)slot0 * np;
    d32 = reinterpret_cast<float *>(ws + e->off_f) + ((int64_t)e->chunk + slot0) * np;
    float *wbound = reinterpret_cast<float *>(ws + e->off_dmax) + e->chunk + slot0;
    int rc = launch_fill(dmax, 0.f, cnt, s);
    if (rc) return rc;
    rc = launch_fill(wbound, 0.f, cnt, s);
    if (rc) return rc;
    rc = launch_fill(reinterpret_cast<float *>(failed), 0.f, cnt, s);
    if (rc) return rc;
    rc = launch_fill(reinterpret_cast<float *>(done), 0.f, cnt, s);
    if (rc) return rc;
    BlockInitArgs ia;
    ia.a = a; ia.a_stride = (int64_t)n * n; ia.n = n;
    ia.qt = qt; ia.np = np; ia.dmax = dmax; ia.wbound = wbound; ia.failed = failed; ia.rot = rot; ia.only = only;
    // A solve runs its first sweeps on a float32 copy of W (twice the matrix-core and vector
    // rates, half the bytes): W = A, Qt = I for a cold solve, W = Qt A Qt^T rounded to float32
    // for a warm one.  Then W = Qt A Qt^T is formed in float64 from the rotations accumulated so
    // far, and float64 sweeps finish the job.  What the float32 sweeps cannot resolve
    // (eigenvalues below 1e-7 of the largest) is left to them.
    w32 = reinterpret_cast<float *>(w);      // shares the memory of W: it is dead when W is formed
    ia.warm = warm ? 1 : 0;
    ia.w = w32;
    hipLaunchKernelGGL(blockjac_init_kernel, dim3(nblk, cnt), dim3(256), 0, s, ia);
    HIP_TRY(hipGetLastError());
    if (warm) congruence(failed, true);
    ja.w = w; ja.w32 = w32; ja.qt = qt; ja.jbuf = jslot[0]; ja.ident = islot[0]; ja.rot = rot; ja.dmax = dmax; ja.wbound = wbound; ja.failed = failed; ja.done = done;
    ja.ident2 = islot[1]; ja.jt16 = hslot[0]; ja.jt16_2 = hslot[1];
    ja.np = np;
    ja.group = (nblk % 4 == 0) ? 2 : 1;
    ja.inner_sweeps = JAC_INNER_SWEEPS;
    sw = 0;
    return SHAMPOO_OK;
  }
  int f32_sweeps() const {
    if (warm) return JAC_F32_SWEEPS_WARM;
    return warm_in.young ? JAC_F32_SWEEPS_YOUNG : JAC_F32_SWEEPS;
  }
  // The next sweep: float32 while sw < f32_sweeps(), then (once) the congruence, then float64.
  int sweep() {
    const int appw_seg = appw_segments(hp);
    const int q_blocks = hp * ((np / JAC_PIV + APPQ_TILES - 1) / APPQ_TILES);
    const bool f32 = sw < f32_sweeps();
    if (f32) {
      ja.phase_start = 0; ja.tol_rel = JAC_F32_TOL_REL; ja.tol_abs_rel = JAC_F32_TOL_ABS;
    } else {
      if (sw == f32_sweeps()) {
        // matrices that float32 has served well enough leave here
        BlockVerdictArgs va{d32, w32, np, n, failed, done, skipc};
        hipLaunchKernelGGL(blockjac_f32_verdict_kernel, dim3(cnt), dim3(256), 0, s, va);
        congruence(skipc, false);
      }
      ja.phase_start = f32_sweeps(); ja.tol_rel = JAC_BLOCK_TOL_REL; ja.tol_abs_rel = JAC_SMALL_TOL_ABS;
    }
    for (int rd = 0; rd < nblk - 1; ++rd) {
      // group == 2: rounds 1 + 2 R and 2 + 2 R are the two rounds of one meeting of super-columns;
      // the second keeps its rotation blocks apart, and Q^T takes both after it
      const int sub = (ja.group == 2 && rd > 0) ? (rd - 1) & 1 : 0;
      ja.round = rd; ja.sweep = sw;
      ja.jbuf = jslot[sub]; ja.ident = islot[sub]; ja.jt16 = hslot[sub];
      // group == 2: the pairs inside a block column are rotated by the pivots of round 0 only (once
      // per sweep, like every other pair); the pivots of the other rounds keep to the pairs across
      // their two block columns, which halves their rounds
      ja.cross_only = (ja.group == 2 && rd > 0) ? 1 : 0;
      if (f32) {
        if (ja.cross_only) hipLaunchKernelGGL((blockjac_pivot_kernel<float, true>), dim3(hp, cnt), dim3(JAC_PIV_THREADS), 0, s, ja);
        else hipLaunchKernelGGL((blockjac_pivot_kernel<float, false>), dim3(hp, cnt), dim3(JAC_PIV_THREADS), 0, s, ja);
        hipLaunchKernelGGL(blockjac_apply_w32_kernel, dim3(appw_segments(hp, W16_SEG), cnt), dim3(JAC_THREADS), 0, s, ja);
      } else {
        if (ja.cross_only) hipLaunchKernelGGL((blockjac_pivot_kernel<double, true>), dim3(hp, cnt), dim3(JAC_PIV_THREADS), 0, s, ja);
        else hipLaunchKernelGGL((blockjac_pivot_kernel<double, false>), dim3(hp, cnt), dim3(JAC_PIV_THREADS), 0, s, ja);
        hipLaunchKernelGGL(blockjac_apply_w_kernel, dim3(appw_seg, cnt), dim3(JAC_THREADS), 0, s, ja);
      }
      if (ja.group == 1 || rd == 0) {
        hipLaunchKernelGGL(blockjac_apply_q_kernel, dim3(q_blocks, cnt), dim3(JAC_THREADS), 0, s, ja);
      } else if (sub == 1) {
        ja.round = rd - 1; ja.jbuf = jslot[0]; ja.ident = islot[0]; ja.jt16 = hslot[0];
        hipLaunchKernelGGL(blockjac_apply_q2_kernel, dim3(q_blocks / 2, cnt), dim3(APPQ2_THREADS), 0, s, ja);
      }
    }
    HIP_TRY(hipGetLastError());
    ++sw;
    return SHAMPOO_OK;
  }
  void congruence(const int32_t *skip, bool out32) {
    // W = Qt A Qt^T, a panel of columns at a time: T = A Qt^T[:, panel], W[:, panel] = Qt T
    // (out32: rounded to float32, into the float32 copy of W)
    const int pw_max = std::min(np, CONGRUENCE_PANEL);
    double *tp = reinterpret_cast<double *>(ws + e->off_t) + (int64_t)slot0 * np * pw_max;
    for (int col0 = 0; col0 < np; col0 += pw_max) {
      const int pw = std::min(pw_max, np - col0);
      CongruenceArgs c1{};
      c1.a = a; c1.a_batch = (int64_t)n * n; c1.lda = n;
      c1.b = qt + (int64_t)col0 * np; c1.b_batch = (int64_t)np * np; c1.ldb = np;
      c1.c = tp; c1.c_batch = (int64_t)np * pw_max; c1.ldc = pw_max;
      c1.M = n; c1.N = pw; c1.K = n; c1.col0 = 0; c1.skip = skip;
      hipLaunchKernelGGL((congruence_gemm_kernel<false, false>), dim3((pw + CG_TILE - 1) / CG_TILE, (n + CG_TILE - 1) / CG_TILE, cnt),
                         dim3(CG_THREADS), 0, s, c1);
      CongruenceArgs c2{};
      c2.a = qt; c2.a_batch = (int64_t)np * np; c2.lda = np;
      c2.b = tp; c2.b_batch = (int64_t)np * pw_max; c2.ldb = pw_max;
      c2.c = w; c2.c_batch = (int64_t)np * np; c2.ldc = np;
      c2.M = np; c2.N = pw; c2.K = n; c2.col0 = col0; c2.skip = skip;
      const dim3 grid2((pw + CG_TILE - 1) / CG_TILE, (np + CG_TILE - 1) / CG_TILE, cnt);
      if (out32) hipLaunchKernelGGL((congruence_gemm_kernel<true, true, true>), grid2, dim3(CG_THREADS), 0, s, c2);
      else hipLaunchKernelGGL((congruence_gemm_kernel<true, true, false>), grid2, dim3(CG_THREADS), 0, s, c2);
    }
  }
  int finish() {
    BlockFinalArgs fa;
    fa.w = w; fa.qt = qt; fa.np = np; fa.n = n; fa.epsilon = eps; fa.r = r; fa.scale = scale; fa.fvals = fv;
    fa.lambda = lambda;
    fa.failed = failed; fa.failed_out = failed_user; fa.fail_count = fail_count;
    fa.rot = rot; fa.sweeps_out = warm_in.sweeps; fa.done = done; fa.d32 = d32;
    BlockRowNormArgs rn{qt, fv, failed, np, n};
    hipLaunchKernelGGL(blockjac_rownorm_kernel, dim3((n + 3) / 4, cnt), dim3(256), 0, s, rn);
    hipLaunchKernelGGL(blockjac_final_kernel, dim3(cnt), dim3(256), 0, s, fa);
    HIP_TRY(hipGetLastError());
    GemmArgs g{};
    g.a.base = qt; g.a.batch_stride = (int64_t)np * np; g.a.ld = np; g.a.from_table = 0;
    g.b = g.a;
    g.c = x; g.c_batch_stride = (int64_t)n * n; g.ldc = n;
    g.M = n; g.N = n; g.K = np; g.alpha = 1.f; g.beta = 0.f;
    g.kscale = fv; g.kscale_stride = np; g.skip = failed;
    g.tiles_m = g.tiles_n = (n + BM - 1) / BM;
    g.tiles = g.tiles_m * (g.tiles_m + 1) / 2;
    g.batch = cnt;
    return launch_gemm<ROW_CONTIG, ROW_CONTIG, float, float, EPI_SYRK, true>(g, s);
  }
};

// X_i = rootinv(scale * A_i) for a batch of dense n x n matrices.  ws: eig_layout(n, >= chunk) region.
// aux: helper streams for the sub-chunks of the block solver (the caller owns them and
// serialises their use), or nullptr.
// only: optional device array [batch]; matrices whose entry is 0 are skipped (x left as it is).
int root_inverse_batched(const float *a, int n, int batch, float eps, float r, float scale, float *x, float *lambda,
                         int32_t *failed_user, unsigned long long *fail_count, unsigned char *ws,
                         const EigLayout &e, hipStream_t s, AuxStreams *aux, const int32_t *only = nullptr,
                         const WarmStart &warm = WarmStart()) {
  if (batch <= 0) return SHAMPOO_OK;
  if (n <= JAC_SMALL_MAX) {
    SmallRootArgs g;
    g.a = a; g.a_stride = (int64_t)n * n;
    g.x = x; g.x_stride = (int64_t)n * n;
    g.lambda = lambda; g.failed = failed_user; g.fail_count = fail_count;
    g.n = n; g.epsilon = eps; g.r = r; g.scale = scale; g.only = only;
    const size_t lds = rootinv_small_lds_bytes(n);
    if (n <= 64) {
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(rootinv_small_kernel<256>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
      hipLaunchKernelGGL(rootinv_small_kernel<256>, dim3(batch), dim3(256), lds, s, g);
    } else {
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(rootinv_small_kernel<1024>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
      hipLaunchKernelGGL(rootinv_small_kernel<1024>, dim3(batch), dim3(1024), lds, s, g);
    }
    HIP_TRY(hipGetLastError());
    return SHAMPOO_OK;
  }
  // Large matrices: block Jacobi.  A chunk of matrices is cut into a few sub-chunks
  // that run on separate streams: the pivot kernel is bound by LDS, the W update by
  // the float64 matrix cores and the Q update by HBM, so sub-chunks that are in
  // different phases overlap on the same CUs.
  // aux == nullptr: everything on the caller's stream.
  if (aux && !aux->ready()) aux = nullptr;
  const int n_sub = aux ? JAC_STREAMS : 1;
  for (int b0 = 0; b0 < batch; b0 += e.chunk) {
    const int cb = std::min(e.chunk, batch - b0);
    const int subs = std::min(n_sub, cb);
    if (subs > 1) {
      HIP_TRY(hipEventRecord(aux->fork, s));
      for (int k = 1; k < subs; ++k) HIP_TRY(hipStreamWaitEvent(aux->stream[k - 1], aux->fork, 0));
    }
    BlockSolve solve[JAC_STREAMS];
    int first = 0;
    for (int k = 0; k < subs; ++k) {
      const int cnt = cb / subs + (k < cb % subs ? 1 : 0);
      WarmStart wk = warm;
      if (wk.qt) wk.qt += (int64_t)(b0 + first) * e.np * e.np;
      if (wk.sweeps) wk.sweeps += b0 + first;
      solve[k] = BlockSolve{a + (int64_t)(b0 + first) * n * n, n, cnt, eps, r, scale,
                            x + (int64_t)(b0 + first) * n * n,
                            lambda ? lambda + (int64_t)(b0 + first) * n : nullptr,
                            failed_user ? failed_user + b0 + first : nullptr, fail_count, ws, &e, first,
                            k == 0 ? s : aux->stream[k - 1], only ? only + b0 + first : nullptr, wk};
      first += cnt;
    }
    // sweep by sweep across the sub-chunks, so that all of them are under way from the start
    for (int k = 0; k < subs; ++k)
      if (const int rc = solve[k].begin()) return rc;
    for (int sw = 0; sw < JAC_OUTER_SWEEPS; ++sw)
      for (int k = 0; k < subs; ++k)
        if (const int rc = solve[k].sweep()) return rc;
    for (int k = 0; k < subs; ++k)
      if (const int rc = solve[k].finish()) return rc;
    if (subs > 1)
      for (int k = 1; k < subs; ++k) {
        HIP_TRY(hipEventRecord(aux->join[k - 1], aux->stream[k - 1]));
        HIP_TRY(hipStreamWaitEvent(s, aux->join[k - 1], 0));
      }
  }
  return SHAMPOO_OK;
}

// ---------------------------------------------------------------------------
// Coupled inverse Newton iteration (Sec. 3.2.1, item 2): workspace and driver
// ---------------------------------------------------------------------------
struct NewtonLayout {
  int32_t chunk = 0;
  size_t mat = 0;          // bytes of one n x n float32 matrix (aligned)
  size_t off_mats = 0, off_rowpart = 0, off_err = 0, off_prev = 0, off_done = 0, off_failed = 0, off_iters = 0;
  size_t bytes = 0;
};
constexpr int NEWTON_MATS = 7;   // M, M', X, X', T and two buffers for the powers of T

NewtonLayout newton_layout(int n, int batch) {
  NewtonLayout e;
  e.mat = align_up((size_t)n * n * sizeof(float));
  // the kernels take the matrix index as grid.y
  e.chunk = (int)std::max<size_t>(1, std::min<size_t>(std::min<size_t>((size_t)std::max(batch, 1), 32768), EIG_CHUNK_BYTES / (NEWTON_MATS * e.mat)));
  size_t off = 0;
  e.off_mats = off; off += (size_t)NEWTON_MATS * e.chunk * e.mat;
  e.off_rowpart = off; off += align_up((size_t)e.chunk * n * sizeof(double));
  e.off_err = off; off += align_up((size_t)e.chunk * sizeof(float));
  e.off_prev = off; off += align_up((size_t)e.chunk * sizeof(float));
  e.off_done = off; off += align_up((size_t)e.chunk * sizeof(int32_t));
  e.off_failed = off; off += align_up((size_t)e.chunk * sizeof(int32_t));
  e.off_iters = off; off += align_up((size_t)e.chunk * sizeof(int32_t));
  e.bytes = off;
  return e;
}

// p must be 1, 2, 4 or 8: T^p is formed by repeated squaring
inline bool newton_p_supported(int p) { return p == 1 || p == 2 || p == 4 || p == 8; }

// C = A B on the lower tiles, mirrored (A, B symmetric and commuting), for the matrices not yet done
int newton_product(const float *A, const float *B, float *C, int n, int cnt, const int32_t *done, hipStream_t s) {
  GemmArgs g{};
  g.a.base = A; g.a.batch_stride = (int64_t)n * n; g.a.ld = n; g.a.from_table = 0;
  g.b.base = B; g.b.batch_stride = (int64_t)n * n; g.b.ld = n; g.b.from_table = 0;
  g.c = C; g.c_batch_stride = (int64_t)n * n; g.ldc = n;
  g.M = n; g.N = n; g.K = n; g.alpha = 1.f; g.beta = 0.f;
  g.skip = done;
  g.tiles_m = g.tiles_n = (n + BM - 1) / BM;
  g.tiles = g.tiles_m * (g.tiles_m + 1) / 2;
  g.batch = cnt;
  return launch_gemm<ROW_CONTIG, ROW_CONTIG, float, float, EPI_SYRK, false>(g, s);
}

// X_i = (scale * A_i + eps I)^(-1/p) for a batch of dense n x n matrices.
int newton_root_batched(const float *a, int n, int batch, float eps, int p, float scale, float tol, int max_iter,
                        float *x, int32_t *iters_user, int32_t *failed_user, unsigned long long *fail_count,
                        unsigned char *ws, const NewtonLayout &e, hipStream_t s) {
  if (batch <= 0) return SHAMPOO_OK;
  const size_t mat_elems = e.mat / sizeof(float);
  for (int b0 = 0; b0 < batch; b0 += e.chunk) {
    const int cb = std::min(e.chunk, batch - b0);
    float *buf[NEWTON_MATS];
    for (int i = 0; i < NEWTON_MATS; ++i) buf[i] = reinterpret_cast<float *>(ws + e.off_mats) + (size_t)i * e.chunk * mat_elems;
    // matrices of a chunk are stored back to back with stride n * n inside each buffer
    float *M = buf[0], *M2 = buf[1], *X = buf[2], *X2 = buf[3], *T = buf[4], *Pa = buf[5], *Pb = buf[6];
    NewtonArgs g{};
    g.a = a + (int64_t)b0 * n * n; g.a_stride = (int64_t)n * n;
    g.rowpart = reinterpret_cast<double *>(ws + e.off_rowpart);
    g.err = reinterpret_cast<float *>(ws + e.off_err); g.prev = reinterpret_cast<float *>(ws + e.off_prev);
    g.done = reinterpret_cast<int32_t *>(ws + e.off_done); g.failed = reinterpret_cast<int32_t *>(ws + e.off_failed);
    g.iters = reinterpret_cast<int32_t *>(ws + e.off_iters);
    g.n = n; g.p = p; g.max_iter = max_iter; g.epsilon = eps; g.scale = scale; g.tol = tol;
    int rc = launch_fill(reinterpret_cast<float *>(g.failed), 0.f, cb, s);
    if (rc) return rc;
    g.M = M; g.X = X; g.T = T;
    hipLaunchKernelGGL(newton_rownorm_kernel, dim3(n, cb), dim3(256), 0, s, g);
    hipLaunchKernelGGL(newton_init_kernel, dim3(n, cb), dim3(256), 0, s, g);
    HIP_TRY(hipGetLastError());
    for (int k = 0; k <= max_iter; ++k) {
      g.k = k; g.M = M; g.X = X; g.T = T;
      hipLaunchKernelGGL(newton_prep_kernel, dim3(n, cb), dim3(256), 0, s, g);
      hipLaunchKernelGGL(newton_check_kernel, dim3((cb + 255) / 256), dim3(256), 0, s, g, cb);
      HIP_TRY(hipGetLastError());
      // matrices whose iteration ended at this k hand their X over now: afterwards the X / M
      // buffers swap roles, and a finished matrix is no longer written by the products
      NewtonFinishArgs fa;
      fa.X = X; fa.x = x + (int64_t)b0 * n * n; fa.x_stride = (int64_t)n * n;
      fa.done = g.done; fa.failed = g.failed; fa.failed_out = failed_user ? failed_user + b0 : nullptr;
      fa.fail_count = fail_count;
      fa.iters = g.iters; fa.iters_out = iters_user ? iters_user + b0 : nullptr; fa.n = n; fa.k = k;
      hipLaunchKernelGGL(newton_finish_kernel, dim3(n, cb), dim3(256), 0, s, fa);
      HIP_TRY(hipGetLastError());
      if (k == max_iter) break;
      // T^p by repeated squaring, X' = X T, M' = T^p M
      const float *Tp = T;
      float *sq[2] = {Pa, Pb};
      int w = 0;
      for (int q = 1; q < p; q *= 2) {
        if ((rc = newton_product(Tp, Tp, sq[w], n, cb, g.done, s))) return rc;
        Tp = sq[w]; w ^= 1;
      }
      if ((rc = newton_product(X, T, X2, n, cb, g.done, s))) return rc;
      if ((rc = newton_product(Tp, M, M2, n, cb, g.done, s))) return rc;
      std::swap(M, M2); std::swap(X, X2);
    }
  }
  return SHAMPOO_OK;
}

}  // namespace

// ---------------------------------------------------------------------------
// The optimizer object
// ---------------------------------------------------------------------------
struct shampoo_opt {
  shampoo_config cfg;
  std::vector<int32_t> ndim;
  std::vector<int64_t> shape;   // [SHAMPOO_MAX_NDIM * n_params], as given
  Plan plan;
  unsigned char *ws = nullptr;
  size_t ws_bytes = 0;
  // workspace offsets
  size_t off_G1 = 0, off_Gf = 0, off_g1tab = 0, off_gftab = 0, off_prep = 0, off_small = 0;
  int64_t n_small = 0;     // blocks of at most 128 x 128 (single-workgroup step kernel)
  bool use_l2 = false, use_b1 = false;
  size_t off_A = 0, off_M = 0, off_T = 0, off_wtab = 0, off_gtab = 0, off_diag = 0, off_count = 0, off_eig = 0;
  std::vector<EigLayout> eig_L, eig_R, eig_mid[2];   // per bucket (eig_mid: the middle dimensions of tensor blocks)
  // tensor parameters: block-contiguous copies of the gradient and the parameter (byte offsets
  // into the workspace, 0 for other parameters), and a second scratch array the size of T
  std::vector<size_t> off_Gb, off_Wb;
  size_t off_T2 = 0;
  bool has_tensor = false;
  size_t off_nfail = 0;   // coupled Newton: per-matrix failure flags of one batch (int32)
  std::vector<void *> last_w, last_g;    // the caller's pointers of the last step
  std::vector<void *> tab_w, tab_g;      // the pointer tables as sent to the device (source of the asynchronous copies)
  AuxStreams aux;                        // helper streams of the block solver, created at the first large refresh
  bool ptrs_aligned16 = false;           // every gradient pointer is 16-byte aligned
  std::vector<char> upper_stale;         // per bucket: the factors' tiles above the diagonal of tiles are out of date
  int64_t last_step = -1;
  int64_t n_refresh = 0;
  bool timing = false;
  struct Interval { hipEvent_t a, b; };
  std::vector<Interval> intervals[SHAMPOO_STAGE_COUNT];
};

namespace {

size_t layout(const shampoo_config *c, Plan &p, shampoo_opt *o) {
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off += align_up(bytes); return r; };
  const size_t offA = take((size_t)p.total_elems * 4);
  const size_t offM = c->momentum > 0.f ? take((size_t)p.total_elems * 4) : 0;
  const bool use_l2 = c->weight_decay > 0.f && !c->use_decoupled_weight_decay;
  const bool use_b1 = c->beta1 > 0.f;
  const size_t offG1 = use_l2 ? take((size_t)p.total_elems * 4) : 0;
  const size_t offGf = use_b1 ? take((size_t)p.total_elems * 4) : 0;
  const size_t offG1tab = take((size_t)c->n_params * sizeof(void *));
  const size_t offGftab = take((size_t)c->n_params * sizeof(void *));
  const size_t offPrep = (use_l2 || use_b1) ? take(std::max<size_t>(1, p.prep_chunks.size()) * sizeof(DiagChunk)) : 0;
  size_t t_elems = 0, t2_elems = 0, eig_bytes = 0, max_count = 1;
  std::vector<EigLayout> eL, eR, eM[2];
  for (auto &b : p.buckets) {
    const size_t B = b.count, m = b.m, n = b.n;
    b.off_L = take(B * b.l_elems() * 4);
    b.off_R = take(B * b.r_elems() * 4);
    b.off_Linv = take(B * b.l_elems() * 4);
    b.off_Rinv = take(B * b.r_elems() * 4);
    if (b.t3) {
      for (int k = 0; k + 2 < b.modes; ++k) {
        b.off_mid[k] = take(B * (size_t)b.td[k + 1] * b.td[k + 1] * 4);
        b.off_midinv[k] = take(B * (size_t)b.td[k + 1] * b.td[k + 1] * 4);
      }
      b.off_desc3 = take(B * (size_t)b.split3 * sizeof(BlockDesc));
      t2_elems = std::max(t2_elems, B * m * n);
    }
    b.off_P = take(B * m * n * 4);
    // bf16 gradients: the preconditioning products run on the fp16 matrix cores from
    // operands kept split in two scaled fp16 planes
    b.planes = c->grad_dtype == SHAMPOO_GRAD_BF16 && b.bf16_mfma && !use_l2 && !use_b1 &&
               c->precond_matrix_cores != SHAMPOO_MATRIX_CORES_FP32;
    if (b.planes) {
      b.off_Linv2h = take(B * m * m * 4);
      b.off_Rinv2h = take(B * n * n * 4);
      b.off_stat_l = take(B * 8);
      b.off_stat_r = take(B * 8);
      b.off_gmaxp = take(B * b.geom.chunks * 4);
      b.off_s_g = take(B * 4);
      b.off_inv_g2 = take(B * 4);
      b.off_t_scale = take(B * 4);
      b.off_inv_ts = take(B * 4);
    }
    b.off_desc = take(B * sizeof(BlockDesc));
    b.off_sgp = take(B * b.geom.chunks * 4);
    // partial sums of ||P_shampoo||^2: one per tile of the last product (tensor blocks: the
    // (d2 d1) x d3 product of the third dimension) or per chunk of an elementwise pass
    size_t ssh_parts = std::max<size_t>((size_t)b.tiles_m * b.tiles_n, (size_t)b.geom.chunks);
    if (b.t3) ssh_parts = std::max(ssh_parts, (size_t)((m * n / b.dlast() + BM - 1) / BM) * ((b.dlast() + BN - 1) / BN));
    b.off_sshp = take(B * ssh_parts * 4);
    b.off_scale = take(B * 4);
    b.off_norms = take(B * 8);
    t_elems = std::max(t_elems, B * m * n);   // float32, or two fp16 planes
    if (c->grad_dtype == SHAMPOO_GRAD_BF16 && b.bf16_mfma && !use_l2) b.off_Gt = take(B * m * n * 2);
    // a diagonalised side needs no eigensolver workspace (stand-in layout of a 1 x 1 problem)
    const int em = b.diagL ? 1 : b.m, en = b.diagR ? 1 : b.rdim();
    const bool warm = c->warm_start_roots != 0 && c->root_method == SHAMPOO_ROOT_EIGH;
    eL.push_back(eig_layout(em, b.count, EIG_CHUNK_BYTES, 0, warm));
    eR.push_back(eig_layout(en, b.count, EIG_CHUNK_BYTES, 0, warm));
    if (warm && eL.back().np > 0) b.off_QtL = take(B * (size_t)eL.back().np * eL.back().np * 4);
    if (warm && eR.back().np > 0) b.off_QtR = take(B * (size_t)eR.back().np * eR.back().np * 4);
    for (int k = 0; k < 2; ++k) eM[k].push_back(eig_layout(b.td[k + 1], b.count));
    // under coupled Newton the eigensolver is the fallback of the guard (Sec. 3.2.3): room for both
    if (c->root_method == SHAMPOO_ROOT_NEWTON)
      eig_bytes = std::max(eig_bytes, std::max(std::max(newton_layout(em, b.count).bytes, newton_layout(en, b.count).bytes),
                                               std::max(newton_layout(b.td[1], b.count).bytes, newton_layout(b.td[2], b.count).bytes)));
    eig_bytes = std::max(eig_bytes, std::max(std::max(eL.back().bytes, eR.back().bytes),
                                             std::max(eM[0].back().bytes, eM[1].back().bytes)));
    max_count = std::max(max_count, (size_t)b.count);
  }
  const size_t offT = take(t_elems * 4);
  const size_t offT2 = t2_elems ? take(t2_elems * 4) : 0;
  std::vector<size_t> offGb(c->n_params, 0), offWb(c->n_params, 0);
  bool has_tensor = false;
  for (int i = 0; i < c->n_params; ++i) {
    if (p.pshape[i].kind != P_TENSOR) continue;
    has_tensor = true;
    const size_t el = (size_t)p.pshape[i].elems();
    offGb[i] = take(el * (c->grad_dtype == SHAMPOO_GRAD_BF16 ? 2 : 4));
    offWb[i] = take(el * 4);
  }
  const size_t offW = take((size_t)c->n_params * sizeof(void *));
  const size_t offG = take((size_t)c->n_params * sizeof(void *));
  const size_t offD = take(std::max<size_t>(1, p.diag_chunks.size()) * sizeof(DiagChunk));
  int64_t n_small = 0;
  for (auto &b : p.buckets) if (b.m <= SB && b.n <= SB && !b.whole() && !b.t3) n_small += b.count;
  const size_t offSmall = take(std::max<size_t>(1, (size_t)n_small) * sizeof(SmallBlock));
  const size_t offC = take(64);
  const size_t offNf = take(max_count * 4);
  const size_t offE = take(eig_bytes);
  if (o) {
    o->off_A = offA; o->off_M = offM; o->off_T = offT;
    o->off_G1 = offG1; o->off_Gf = offGf; o->off_g1tab = offG1tab; o->off_gftab = offGftab; o->off_prep = offPrep;
    o->use_l2 = use_l2; o->use_b1 = use_b1; o->off_wtab = offW; o->off_gtab = offG;
    o->off_diag = offD; o->off_count = offC; o->off_eig = offE;
    o->off_small = offSmall; o->n_small = n_small;
    o->eig_L = eL; o->eig_R = eR; o->eig_mid[0] = eM[0]; o->eig_mid[1] = eM[1];
    o->upper_stale.assign(o->plan.buckets.size(), 0);
    o->off_nfail = offNf;
    o->off_T2 = offT2; o->off_Gb = offGb; o->off_Wb = offWb; o->has_tensor = has_tensor;
  }
  return off;
}

struct StageTimer {
  shampoo_opt *o; int stage; hipStream_t s; bool on; hipEvent_t a{};
  StageTimer(shampoo_opt *o_, int st, hipStream_t s_) : o(o_), stage(st), s(s_), on(o_->timing) {
    if (on) { if (hipEventCreate(&a) != hipSuccess) { on = false; return; } (void)hipEventRecord(a, s); }
  }
  ~StageTimer() {
    if (!on) return;
    hipEvent_t b;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
    (void)hipEventRecord(b, s);
    o->intervals[stage].push_back({a, b});
  }
};

// Re-splits the roots of every bucket that keeps them as planes (after create and after
// every refresh).
int split_roots(shampoo_opt *o, hipStream_t s) {
  for (auto &b : o->plan.buckets) {
    if (!b.planes) continue;
    const int64_t nl = (int64_t)b.count * b.m * b.m, nr = (int64_t)b.count * b.n * b.n;
    const float *Li = reinterpret_cast<const float *>(o->ws + b.off_Linv), *Ri = reinterpret_cast<const float *>(o->ws + b.off_Rinv);
    float *stat_l = reinterpret_cast<float *>(o->ws + b.off_stat_l), *stat_r = reinterpret_cast<float *>(o->ws + b.off_stat_r);
    hipLaunchKernelGGL(matrix_stats_kernel, dim3(b.count), dim3(256), 0, s, Li, stat_l, b.m);
    hipLaunchKernelGGL(matrix_stats_kernel, dim3(b.count), dim3(256), 0, s, Ri, stat_r, b.n);
    hipLaunchKernelGGL(split2h_kernel, dim3((unsigned)((nl + 255) / 256)), dim3(256), 0, s,
                       Li, stat_l, reinterpret_cast<uint16_t *>(o->ws + b.off_Linv2h), (int64_t)b.m * b.m, nl);
    hipLaunchKernelGGL(split2h_kernel, dim3((unsigned)((nr + 255) / 256)), dim3(256), 0, s,
                       Ri, stat_r, reinterpret_cast<uint16_t *>(o->ws + b.off_Rinv2h), (int64_t)b.n * b.n, nr);
    HIP_TRY(hipGetLastError());
  }
  return SHAMPOO_OK;
}

// Coupled Newton with the guard of Sec. 3.2.3.  The paper retries a failed root computation in
// higher precision and keeps the previous root only if that fails too; here the float32
// iteration is the first attempt, and a matrix whose iterates do not stay finite (a condition
// number beyond float32) is handed to the eigendecomposition, which works on a float64 copy.
// Whether any matrix failed is read back, so a refresh under root_method = NEWTON waits for
// the stream once per factor batch; failures of the fallback are what gets counted.
int newton_root_guarded(shampoo_opt *o, const float *F, int dim, int count, float r_exp, float c2, float *Fi,
                        const EigLayout &lay, hipStream_t s) {
  const shampoo_config &c = o->cfg;
  unsigned char *ws = o->ws;
  unsigned long long *counters = reinterpret_cast<unsigned long long *>(ws + o->off_count);
  unsigned long long *newton_failed = counters + 1;
  int32_t *flags = reinterpret_cast<int32_t *>(ws + o->off_nfail);
  const float tol = c.newton_tolerance > 0.f ? c.newton_tolerance : 1e-6f;
  const int cap = c.newton_max_iterations > 0 ? c.newton_max_iterations : 100;
  int rc = launch_fill(reinterpret_cast<float *>(newton_failed), 0.f, 2, s);
  if (rc) return rc;
  rc = newton_root_batched(F, dim, count, c.epsilon, newton_p_of(r_exp), c2, tol, cap, Fi, nullptr, flags, newton_failed,
                           ws + o->off_eig, newton_layout(dim, count), s);
  if (rc) return rc;
  unsigned long long n_failed = 0;
  HIP_TRY(hipMemcpyAsync(&n_failed, newton_failed, sizeof(n_failed), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  if (n_failed == 0) return SHAMPOO_OK;
  return root_inverse_batched(F, dim, count, c.epsilon, r_exp, c2, Fi, nullptr, nullptr, counters, ws + o->off_eig, lay, s,
                              &o->aux, flags);
}

// GT: element type of the caller's gradients.  GS: of the gradients that feed the factors and
// the grafting state (GT, or float when l2 weight decay materialises G + wd W).  GD: of the
// gradients that feed the directions (float when filtered or shifted, else GT).
// The bf16 factor update writes only the tiles on and below the diagonal of tiles; whoever
// needs the whole symmetric factor (the refresh, the state query) completes it first.
int complete_factors(shampoo_opt *o, size_t bucket, hipStream_t s) {
  if (!o->upper_stale[bucket]) return SHAMPOO_OK;
  const Bucket &b = o->plan.buckets[bucket];
  const int dims[2] = {(int)b.m, (int)b.n};
  const size_t offs[2] = {b.off_L, b.off_R};
  for (int side = 0; side < 2; ++side) {
    const int n = dims[side], pieces = (n + 31) / 32;
    if (n <= BM) continue;   // a single tile: nothing above the diagonal
    hipLaunchKernelGGL(mirror_upper_tiles_kernel, dim3(pieces, pieces, b.count), dim3(256), 0, s,
                       reinterpret_cast<float *>(o->ws + offs[side]), (int64_t)n * n, n);
  }
  HIP_TRY(hipGetLastError());
  o->upper_stale[bucket] = 0;
  return SHAMPOO_OK;
}

// A factor of dimension `dim` that has so far summed (step + 1) gradients of `cols` columns
// each is a near-singular Gram matrix until it holds a few times more columns than it has
// rows (a Gaussian dim x N matrix has the condition number ((sqrt N + sqrt dim) / (sqrt N -
// sqrt dim))^2 squared into its Gram matrix: 1e7 and more at N = dim, 34 at N = 2 dim, 9 at
// N = 4 dim).  While it is, a root taken from it weights its smallest eigenvalues most, and
// the bf16 factor update sums in float64 (syrk_bf16.h).
constexpr int64_t WARM_RESTART_PERIOD = 16;

inline bool young_factor(int64_t step, int cols, int dim) { return (step + 1) * (int64_t)cols < 4 * (int64_t)dim; }

template <typename GT, typename GS, typename GD>
int step_impl(shampoo_opt *o, float lr, int64_t step, hipStream_t s) {
  const shampoo_config &c = o->cfg;
  Plan &p = o->plan;
  unsigned char *ws = o->ws;
  float *A = reinterpret_cast<float *>(ws + o->off_A);
  float *M = c.momentum > 0.f ? reinterpret_cast<float *>(ws + o->off_M) : nullptr;
  float *T = reinterpret_cast<float *>(ws + o->off_T);
  float *G1 = o->use_l2 ? reinterpret_cast<float *>(ws + o->off_G1) : nullptr;
  float *Gf = o->use_b1 ? reinterpret_cast<float *>(ws + o->off_Gf) : nullptr;
  void *const *wtab = reinterpret_cast<void *const *>(ws + o->off_wtab);
  const void *const *gtab = reinterpret_cast<const void *const *>(ws + o->off_gtab);
  // gradients feeding factors + grafting state / feeding the directions
  const void *const *gs_tab = o->use_l2 ? reinterpret_cast<const void *const *>(ws + o->off_g1tab) : gtab;
  const void *const *gd_tab = o->use_b1 ? reinterpret_cast<const void *const *>(ws + o->off_gftab) : gs_tab;
  unsigned long long *fail_count = reinterpret_cast<unsigned long long *>(ws + o->off_count);
  const bool use_shampoo = step >= c.start_preconditioning_step;
  const bool refresh = use_shampoo && (step % c.precondition_frequency == 0);
  // EMA weights from the float32 beta2 the caller gave, evaluated in float64
  const double alpha = c.beta2 < 1.f ? 1.0 - (double)c.beta2 : 1.0;
  const double beta = c.beta2 < 1.f ? (double)c.beta2 : 1.0;
  // k-slabs between float64 flushes of the factor accumulators (flushing every 4 slabs
  // measured 3x larger errors in the stale-root directions, for a 5 % gain)
  constexpr int FLUSH = 1;
  const float wd_l2 = o->use_l2 ? c.weight_decay : 0.f;
  const float wd_dec = (c.weight_decay > 0.f && c.use_decoupled_weight_decay) ? c.weight_decay : 0.f;
  const int sgd = c.grafting_type == SHAMPOO_GRAFT_SGD ? 1 : 0;
  // bias correction (Sec. 3.1.1): directions use Gf / (1 - beta1^(t+1)), roots are taken of
  // L / (1 - beta2^(t+1)); the stored state stays uncorrected
  const bool bc = c.use_bias_correction != 0;
  const float c1 = (bc && c.beta1 > 0.f) ? (float)(1.0 / (1.0 - std::pow((double)c.beta1, (double)(step + 1)))) : 1.f;
  const float c2 = (bc && c.beta2 < 1.f) ? (float)(1.0 / (1.0 - std::pow((double)c.beta2, (double)(step + 1)))) : 1.f;
  // grafting second moment: sum (AdaGrad) or EMA (RMSprop, Adam; Adam bias-corrected on request)
  const bool ema = c.grafting_type == SHAMPOO_GRAFT_RMSPROP || c.grafting_type == SHAMPOO_GRAFT_ADAM;
  const float a_decay = ema ? c.grafting_beta2 : 1.f;
  const float a_gain = (ema && c.grafting_beta2 < 1.f) ? (float)(1.0 - (double)c.grafting_beta2) : 1.f;
  const float a_bc = (c.grafting_type == SHAMPOO_GRAFT_ADAM && bc && c.grafting_beta2 < 1.f)
                         ? (float)(1.0 / (1.0 - std::pow((double)c.grafting_beta2, (double)(step + 1)))) : 1.f;
  int rc;

  // Tensor parameters (Sec. 2.3): the step works on block-contiguous copies of their gradient
  // and of the parameter itself; the pointer tables on the device name those copies.
  auto tensor_copy_args = [&](int i) {
    const PShape &ps = p.pshape[i];
    TensorCopyArgs ta{};
    ta.D1 = ps.d[0]; ta.D2 = ps.d[1]; ta.D3 = ps.d[2]; ta.D4 = ps.d[3]; ta.b = c.block_size;
    ta.k2n = (int32_t)((ps.d[1] + c.block_size - 1) / c.block_size);
    ta.k3n = (int32_t)((ps.d[2] + c.block_size - 1) / c.block_size);
    ta.k4n = (int32_t)((ps.d[3] + c.block_size - 1) / c.block_size);
    return ta;
  };
  auto tensor_copy_grid = [&](int i) {
    const int64_t per = std::min<int64_t>(c.block_size, p.pshape[i].d[0]) * std::min<int64_t>(c.block_size, p.pshape[i].d[1]) *
                        std::min<int64_t>(c.block_size, p.pshape[i].d[2]) * std::min<int64_t>(c.block_size, p.pshape[i].d[3]);
    return dim3((unsigned)p.param_blocks[i].size(), (unsigned)std::max<int64_t>(1, std::min<int64_t>(64, (per + 2047) / 2048)));
  };
  if (o->has_tensor) {
    StageTimer t(o, SHAMPOO_STAGE_GRAFT, s);
    for (int i = 0; i < c.n_params; ++i) {
      if (p.pshape[i].kind != P_TENSOR) continue;
      TensorCopyArgs ta = tensor_copy_args(i);
      ta.tensor_in = o->last_g[i]; ta.copy_out = ws + o->off_Gb[i];
      hipLaunchKernelGGL((tensor_block_copy_kernel<GT, false>), tensor_copy_grid(i), dim3(256), 0, s, ta);
      ta.tensor_in = o->last_w[i]; ta.copy_out = ws + o->off_Wb[i];
      hipLaunchKernelGGL((tensor_block_copy_kernel<float, false>), tensor_copy_grid(i), dim3(256), 0, s, ta);
    }
    HIP_TRY(hipGetLastError());
  }

  if ((o->use_l2 || o->use_b1) && !p.prep_chunks.empty()) {
    StageTimer t(o, SHAMPOO_STAGE_GRAFT, s);
    PrepArgs pa;
    pa.chunks = reinterpret_cast<const DiagChunk *>(ws + o->off_prep);
    pa.w_table = wtab; pa.g_table = gtab; pa.g1 = G1; pa.gf = Gf; pa.wd_l2 = wd_l2; pa.beta1 = c.beta1;
    hipLaunchKernelGGL(prep_kernel<GT>, dim3((unsigned)p.prep_chunks.size()), dim3(EW_THREADS), 0, s, pa);
    HIP_TRY(hipGetLastError());
  }
  // Blocks of at most 128 x 128 take the whole step in one workgroup (gradient block
  // resident in LDS) whenever no refresh separates the factor update from the
  // preconditioning and the default heuristics are in force.
  const bool small_ok = use_shampoo && !refresh && !o->use_l2 && !o->use_b1 && !sgd;
  auto fused = [&](const Bucket &b) { return small_ok && b.m <= SB && b.n <= SB && !b.whole() && !b.t3; };
  if (small_ok && o->n_small > 0) {
    StageTimer t(o, SHAMPOO_STAGE_FUSED, s);
    SmallStepArgs f;
    f.blocks = reinterpret_cast<const SmallBlock *>(ws + o->off_small); f.ws = ws;
    f.w_table = wtab; f.g_table = gtab; f.a_state = A; f.m_state = M;
    f.alpha_d = alpha; f.beta_d = beta;
    f.graft_eps = c.graft_epsilon; f.mu = c.momentum; f.lr = lr; f.wd_decoupled = wd_dec;
    f.nesterov = c.use_nesterov ? 1 : 0;
    f.a_decay = a_decay; f.a_gain = a_gain; f.a_bc = a_bc;
    hipLaunchKernelGGL(block_step_small_kernel<GT>, dim3((unsigned)o->n_small), dim3(SB_THREADS), 0, s, f);
    HIP_TRY(hipGetLastError());
  }
  // scales of the fp16 operands of a bucket's preconditioning products (and of R's update)
  auto launch_x2_scales = [&](const Bucket &b) {
    X2ScaleArgs xs;
    xs.gmax_partial = reinterpret_cast<const float *>(ws + b.off_gmaxp); xs.parts = b.geom.chunks;
    xs.stat_l = reinterpret_cast<const float *>(ws + b.off_stat_l); xs.stat_r = reinterpret_cast<const float *>(ws + b.off_stat_r);
    xs.c1 = c1;
    xs.s_g = reinterpret_cast<float *>(ws + b.off_s_g); xs.inv_g2 = reinterpret_cast<float *>(ws + b.off_inv_g2);
    xs.t_scale = reinterpret_cast<float *>(ws + b.off_t_scale); xs.inv_ts = reinterpret_cast<float *>(ws + b.off_inv_ts);
    hipLaunchKernelGGL(x2_scales_kernel, dim3(b.count), dim3(64), 0, s, xs);
  };
  for (auto &b : p.buckets) {
    if (fused(b)) continue;
    const BlockDesc *desc = reinterpret_cast<const BlockDesc *>(ws + b.off_desc);
    // grafting state and norm first: the same pass finds max |G| of every block, which scales
    // the fp16 planes of this step's first product
    {
      StageTimer t(o, SHAMPOO_STAGE_GRAFT, s);
      EwArgs e{};
      e.desc = desc; e.w_table = wtab; e.g_table = gs_tab; e.gd_table = gd_tab; e.a_state = A; e.m_state = M;
      e.sg_partial = reinterpret_cast<float *>(ws + b.off_sgp);
      e.m = b.m; e.n = b.n; e.geom = b.geom; e.graft_eps = c.graft_epsilon; e.mu = c.momentum; e.lr = lr;
      e.sgd_graft = sgd; e.same_src = (gs_tab == gd_tab) ? 1 : 0; e.gd_scale = c1;
      e.a_decay = a_decay; e.a_gain = a_gain; e.a_bc = a_bc;
      if (b.planes) e.gmax_partial = reinterpret_cast<float *>(ws + b.off_gmaxp);
      hipLaunchKernelGGL((graft_kernel<GS, GD>), dim3((unsigned)b.geom.chunks * b.count), dim3(EW_THREADS), 0, s, e);
      HIP_TRY(hipGetLastError());
    }
    if (sizeof(GS) == 2 && b.bf16_mfma && o->ptrs_aligned16) {
      StageTimer t(o, SHAMPOO_STAGE_FACTOR, s);
      // fp16 operands of this step's preconditioning products (and of R's update): their scales first
      const bool x2 = sizeof(GD) == 2 && b.planes;
      if (x2) launch_x2_scales(b);
      uint16_t *Gt = reinterpret_cast<uint16_t *>(ws + b.off_Gt);
      TransposeArgs ta;
      ta.desc = desc; ta.g_table = gs_tab; ta.out = Gt; ta.m = b.m; ta.n = b.n;
      ta.scale = x2 ? reinterpret_cast<const float *>(ws + b.off_s_g) : nullptr;
      hipLaunchKernelGGL(transpose_bf16_kernel, dim3((b.n + 63) / 64, (b.m + 63) / 64, b.count), dim3(256), 0, s, ta);
      SyrkBf16Args sa{};
      sa.desc = desc; sa.ptr_table = gs_tab; sa.alpha = alpha; sa.beta = beta; sa.batch = b.count;
      o->upper_stale[&b - p.buckets.data()] = 1;   // the kernel writes the tiles on and below the diagonal only
      // L <- beta L + alpha G G^T
      sa.a.from_table = 1;
      sa.c = reinterpret_cast<float *>(ws + b.off_L); sa.c_batch_stride = (int64_t)b.m * b.m; sa.ldc = b.m;
      sa.M = b.m; sa.K = b.n; sa.tiles = b.tiles_m * (b.tiles_m + 1) / 2;
      {
        const int64_t total = (int64_t)sa.tiles * sa.batch;
        const int per = (int)((total + NUM_XCD - 1) / NUM_XCD);
        if (young_factor(step, b.n, b.m))
          hipLaunchKernelGGL((syrk_bf16_kernel<false, true>), dim3(per * NUM_XCD), dim3(GEMM_THREADS), 0, s, sa);
        else
          hipLaunchKernelGGL((syrk_bf16_kernel<false, false>), dim3(per * NUM_XCD), dim3(GEMM_THREADS), 0, s, sa);
      }
      // R <- beta R + alpha (G^T)(G^T)^T
      sa.a.from_table = 0; sa.a.base = Gt; sa.a.batch_stride = (int64_t)b.m * b.n; sa.a.ld = b.m;
      sa.c = reinterpret_cast<float *>(ws + b.off_R); sa.c_batch_stride = (int64_t)b.n * b.n; sa.ldc = b.n;
      sa.M = b.n; sa.K = b.m; sa.tiles = b.tiles_n * (b.tiles_n + 1) / 2;
      {
        const int64_t total = (int64_t)sa.tiles * sa.batch;
        const int per = (int)((total + NUM_XCD - 1) / NUM_XCD);
        const bool young = young_factor(step, b.m, b.n);
        if (x2) {
          sa.x_scale2 = reinterpret_cast<const float *>(ws + b.off_inv_g2);
          if (young) hipLaunchKernelGGL((syrk_bf16_kernel<true, true>), dim3(per * NUM_XCD), dim3(GEMM_THREADS), 0, s, sa);
          else hipLaunchKernelGGL((syrk_bf16_kernel<true, false>), dim3(per * NUM_XCD), dim3(GEMM_THREADS), 0, s, sa);
        } else {
          if (young) hipLaunchKernelGGL((syrk_bf16_kernel<false, true>), dim3(per * NUM_XCD), dim3(GEMM_THREADS), 0, s, sa);
          else hipLaunchKernelGGL((syrk_bf16_kernel<false, false>), dim3(per * NUM_XCD), dim3(GEMM_THREADS), 0, s, sa);
        }
      }
      HIP_TRY(hipGetLastError());
    } else {
      StageTimer t(o, SHAMPOO_STAGE_FACTOR, s);
      o->upper_stale[&b - p.buckets.data()] = 0;   // these kernels read the lower triangle and write both
      GemmArgs g{};
      g.a.from_table = 1; g.b.from_table = 1;
      g.desc = desc; g.ptr_table = gs_tab;
      g.alpha = (float)alpha; g.beta = (float)beta; g.alpha_d = alpha; g.beta_d = beta; g.batch = b.count;
      DiagFactorArgs df{};
      df.desc = desc; df.g_table = gs_tab; df.a = beta; df.b = alpha; df.m = b.m; df.n = b.n;
      if (b.diagL) {
        // l_i <- beta l_i + alpha sum_j G_ij^2 (Sec. 4.2.3)
        df.vec = reinterpret_cast<float *>(ws + b.off_L);
        hipLaunchKernelGGL(diag_row_kernel<GS>, dim3((b.m + 3) / 4, b.count), dim3(256), 0, s, df);
        HIP_TRY(hipGetLastError());
      } else {
        // L <- beta L + alpha G G^T
        g.c = reinterpret_cast<float *>(ws + b.off_L); g.c_batch_stride = (int64_t)b.m * b.m; g.ldc = b.m;
        g.M = b.m; g.N = b.m; g.K = b.n;
        g.tiles_m = g.tiles_n = b.tiles_m; g.tiles = b.tiles_m * (b.tiles_m + 1) / 2;
        rc = launch_gemm<K_CONTIG, K_CONTIG, GS, GS, EPI_SYRK, false, FLUSH>(g, s);
        if (rc) return rc;
      }
      if (b.t3) {
        // Above: L_1 <- beta L_1 + alpha G_(1) G_(1)^T, the block being d1 x (d2 d3 d4).  The other
        // dimensions exist only for a tensor of order three or four.
        if (b.modes >= 3) {
          // Last dimension: the block as (N / d_last) x d_last, read "rows along k".  Its rows
          // are cut into split3 ranges, each a batch entry that leaves its Gram matrix in
          // scratch; gram_reduce_kernel adds them up in float64 and applies the moving average.
          float *T2 = reinterpret_cast<float *>(ws + o->off_T2);
          const int dl = b.dlast(), inner = b.n / dl;
          g.desc = reinterpret_cast<const BlockDesc *>(ws + b.off_desc3);
          g.c = T2; g.c_batch_stride = (int64_t)dl * dl; g.ldc = dl;
          g.M = dl; g.N = dl; g.K = (b.m / b.split3) * inner;
          g.alpha = 1.f; g.beta = 0.f; g.alpha_d = 1.0; g.beta_d = 0.0; g.batch = b.count * b.split3;
          g.tiles_m = g.tiles_n = (dl + BM - 1) / BM; g.tiles = g.tiles_m * (g.tiles_m + 1) / 2;
          rc = launch_gemm<ROW_CONTIG, ROW_CONTIG, GS, GS, EPI_SYRK, false, FLUSH>(g, s);
          if (rc) return rc;
          GramReduceArgs gr;
          gr.partial = T2; gr.factor = reinterpret_cast<float *>(ws + b.off_R); gr.d = dl; gr.splits = b.split3;
          gr.alpha = alpha; gr.beta = beta;
          hipLaunchKernelGGL(gram_reduce_kernel, dim3((dl * dl + 255) / 256, b.count), dim3(256), 0, s, gr);
          HIP_TRY(hipGetLastError());
          // Middle dimensions k: the block as pre x d_k x post with its first two indices swapped,
          // d_k x (pre post)
          int pre = b.m;
          for (int k = 1; k + 1 < b.modes; ++k) {
            const int dk = b.td[k], post = b.n / (pre / b.m * dk);
            PermuteArgs pm{};
            pm.desc = desc; pm.table = gs_tab; pm.dst = T2; pm.d1 = pre; pm.d2 = dk; pm.d3 = post;
            const unsigned pchunks = (unsigned)std::max<int64_t>(1, std::min<int64_t>(64, ((int64_t)b.m * b.n + 2047) / 2048));
            hipLaunchKernelGGL(permute_12_kernel<GS>, dim3(pchunks, b.count), dim3(256), 0, s, pm);
            HIP_TRY(hipGetLastError());
            GemmArgs h{};
            h.a.base = T2; h.a.batch_stride = (int64_t)b.m * b.n; h.a.ld = pre * post;
            h.b = h.a;
            h.alpha = (float)alpha; h.beta = (float)beta; h.alpha_d = alpha; h.beta_d = beta; h.batch = b.count;
            h.c = reinterpret_cast<float *>(ws + b.off_mid[k - 1]); h.c_batch_stride = (int64_t)dk * dk; h.ldc = dk;
            h.M = dk; h.N = dk; h.K = pre * post;
            h.tiles_m = h.tiles_n = (dk + BM - 1) / BM; h.tiles = h.tiles_m * (h.tiles_m + 1) / 2;
            rc = launch_gemm<K_CONTIG, K_CONTIG, float, float, EPI_SYRK, false, FLUSH>(h, s);
            if (rc) return rc;
            pre *= dk;
          }
        }
      } else if (b.diagR) {
        // r_j <- beta r_j + alpha sum_i G_ij^2, rows cut into segments whose partial sums go through T
        df.vec = reinterpret_cast<float *>(ws + b.off_R);
        df.partial = T; df.segs = b.col_segs; df.rows_per_seg = b.rows_per_seg;
        hipLaunchKernelGGL(diag_col_partial_kernel<GS>, dim3((b.n + 255) / 256, b.col_segs, b.count), dim3(256), 0, s, df);
        hipLaunchKernelGGL(diag_col_reduce_kernel, dim3((b.n + 255) / 256, b.count), dim3(256), 0, s, df);
        HIP_TRY(hipGetLastError());
      } else {
        // R <- beta R + alpha G^T G
        g.c = reinterpret_cast<float *>(ws + b.off_R); g.c_batch_stride = (int64_t)b.n * b.n; g.ldc = b.n;
        g.M = b.n; g.N = b.n; g.K = b.m;
        g.tiles_m = g.tiles_n = b.tiles_n; g.tiles = b.tiles_n * (b.tiles_n + 1) / 2;
        rc = launch_gemm<ROW_CONTIG, ROW_CONTIG, GS, GS, EPI_SYRK, false, FLUSH>(g, s);
        if (rc) return rc;
      }
    }
  }
  if (refresh) {
    StageTimer t(o, SHAMPOO_STAGE_ROOT, s);
    // Warm start: from the eigenvectors of the previous refresh, except at the first refresh and
    // at every WARM_RESTART_PERIOD-th one (the accumulated float32 eigenvectors drift away from
    // orthogonality by about 1e-6 per solve; a cold solve resets that).
    const bool warm_now = o->n_refresh > 0 && o->n_refresh % WARM_RESTART_PERIOD != 0;
    auto warm_of = [&](const EigLayout &lay, size_t off_qt, int cols, int dim) {
      WarmStart w;
      if (lay.warm && off_qt) { w.qt = reinterpret_cast<float *>(ws + off_qt); w.start = warm_now; }
      w.young = young_factor(step, cols, dim);
      return w;
    };
    for (size_t i = 0; i < p.buckets.size(); ++i) {
      auto &b = p.buckets[i];
      if ((rc = complete_factors(o, i, s))) return rc;
      if (b.whole()) {
        // diagonal sides: elementwise root; full sides: the eigensolver
        for (int side = 0; side < 2; ++side) {
          const bool dg = side == 0 ? b.diagL : b.diagR;
          const int dim = side == 0 ? b.m : b.n;
          float *F = reinterpret_cast<float *>(ws + (side == 0 ? b.off_L : b.off_R));
          float *Fi = reinterpret_cast<float *>(ws + (side == 0 ? b.off_Linv : b.off_Rinv));
          if (dg) {
            DiagRootArgs da;
            da.vec = F; da.out = Fi; da.dim = dim; da.epsilon = c.epsilon; da.r = c.root_exponent; da.scale = c2;
            da.fail_count = fail_count;
            hipLaunchKernelGGL(diag_root_kernel, dim3(b.count), dim3(256), 0, s, da);
            HIP_TRY(hipGetLastError());
          } else {
            rc = root_inverse_batched(F, dim, b.count, c.epsilon, c.root_exponent, c2, Fi, nullptr, nullptr, fail_count,
                                      ws + o->off_eig, side == 0 ? o->eig_L[i] : o->eig_R[i], s, &o->aux, nullptr,
                                      warm_of(side == 0 ? o->eig_L[i] : o->eig_R[i], side == 0 ? b.off_QtL : b.off_QtR,
                                              side == 0 ? b.n : b.m, dim));
            if (rc) return rc;
          }
        }
        continue;
      }
      if (b.t3) {
        // one root per dimension, exponent 2 r / w (Sec. 2.3: "root 2w")
        const float rw = 2.f * c.root_exponent / (float)b.modes;
        int dims[4]; size_t fac[4], inv[4]; const EigLayout *lay[4];
        for (int k = 0; k < b.modes; ++k) {
          dims[k] = b.td[k];
          if (k == 0) { fac[k] = b.off_L; inv[k] = b.off_Linv; lay[k] = &o->eig_L[i]; }
          else if (k == b.modes - 1) { fac[k] = b.off_R; inv[k] = b.off_Rinv; lay[k] = &o->eig_R[i]; }
          else { fac[k] = b.off_mid[k - 1]; inv[k] = b.off_midinv[k - 1]; lay[k] = &o->eig_mid[k - 1][i]; }
        }
        for (int k = 0; k < b.modes; ++k) {
          if (c.root_method == SHAMPOO_ROOT_NEWTON) {
            rc = newton_root_guarded(o, reinterpret_cast<float *>(ws + fac[k]), dims[k], b.count, rw, c2,
                                     reinterpret_cast<float *>(ws + inv[k]), *lay[k], s);
          } else {
            rc = root_inverse_batched(reinterpret_cast<float *>(ws + fac[k]), dims[k], b.count, c.epsilon, rw, c2,
                                      reinterpret_cast<float *>(ws + inv[k]), nullptr, nullptr, fail_count,
                                      ws + o->off_eig, *lay[k], s, &o->aux);
          }
          if (rc) return rc;
        }
        continue;
      }
      if (c.root_method == SHAMPOO_ROOT_NEWTON) {
        rc = newton_root_guarded(o, reinterpret_cast<float *>(ws + b.off_L), b.m, b.count, c.root_exponent, c2,
                                 reinterpret_cast<float *>(ws + b.off_Linv), o->eig_L[i], s);
        if (rc) return rc;
        rc = newton_root_guarded(o, reinterpret_cast<float *>(ws + b.off_R), b.n, b.count, c.root_exponent, c2,
                                 reinterpret_cast<float *>(ws + b.off_Rinv), o->eig_R[i], s);
        if (rc) return rc;
        continue;
      }
      rc = root_inverse_batched(reinterpret_cast<float *>(ws + b.off_L), b.m, b.count, c.epsilon, c.root_exponent, c2,
                                reinterpret_cast<float *>(ws + b.off_Linv), nullptr, nullptr, fail_count,
                                ws + o->off_eig, o->eig_L[i], s, &o->aux, nullptr, warm_of(o->eig_L[i], b.off_QtL, b.n, b.m));
      if (rc) return rc;
      rc = root_inverse_batched(reinterpret_cast<float *>(ws + b.off_R), b.n, b.count, c.epsilon, c.root_exponent, c2,
                                reinterpret_cast<float *>(ws + b.off_Rinv), nullptr, nullptr, fail_count,
                                ws + o->off_eig, o->eig_R[i], s, &o->aux, nullptr, warm_of(o->eig_R[i], b.off_QtR, b.m, b.n));
      if (rc) return rc;
    }
    o->n_refresh++;
    if ((rc = split_roots(o, s))) return rc;
  }
  for (auto &b : p.buckets) {
    const BlockDesc *desc = reinterpret_cast<const BlockDesc *>(ws + b.off_desc);
    float *P = reinterpret_cast<float *>(ws + b.off_P);
    float *scale = reinterpret_cast<float *>(ws + b.off_scale);
    if (fused(b)) continue;
    int ssh_count = b.tiles_m * b.tiles_n;
    if (use_shampoo && b.t3) {
      // P = G x_1 Lbar_1 x_2 Lbar_2 ... x_w Lbar_w (Sec. 2.3).  Mode 1 on the block as
      // d1 x (d2 ... dw); a middle mode k on the block as pre x d_k x post: its first two
      // indices are swapped, the product is the plain one on d_k x (pre post), and they are
      // swapped back; the last mode on the block as (N / d_w) x d_w, with the norm epilogue.
      StageTimer t(o, SHAMPOO_STAGE_PRECOND, s);
      float *T2 = reinterpret_cast<float *>(ws + o->off_T2);
      float *ssh = reinterpret_cast<float *>(ws + b.off_sshp);
      const int64_t mn = (int64_t)b.m * b.n;
      GemmArgs g{};
      g.a.base = ws + b.off_Linv; g.a.batch_stride = (int64_t)b.m * b.m; g.a.ld = b.m;
      g.b.from_table = 1; g.desc = desc; g.ptr_table = gd_tab;
      g.c_batch_stride = mn; g.ldc = b.n;
      g.M = b.m; g.N = b.n; g.K = b.m; g.alpha = c1; g.beta = 0.f;
      g.tiles_m = b.tiles_m; g.tiles_n = b.tiles_n; g.tiles = b.tiles_m * b.tiles_n; g.batch = b.count;
      if (b.modes == 1) {
        g.c = P; g.norm_partial = ssh;
        rc = launch_gemm<ROW_CONTIG, ROW_CONTIG, float, GD, EPI_STORE_NORM, false>(g, s);
        if (rc) return rc;
      } else {
        float *cur = T, *other = T2;
        g.c = cur;
        rc = launch_gemm<ROW_CONTIG, ROW_CONTIG, float, GD, EPI_STORE, false>(g, s);
        if (rc) return rc;
        const unsigned pchunks = (unsigned)std::max<int64_t>(1, std::min<int64_t>(64, (mn + 2047) / 2048));
        int pre = b.m;
        for (int k = 1; k + 1 < b.modes; ++k) {
          const int dk = b.td[k], post = (int)(mn / ((int64_t)pre * dk));
          PermuteArgs pm{};
          pm.src = cur; pm.dst = other; pm.d1 = pre; pm.d2 = dk; pm.d3 = post;
          hipLaunchKernelGGL(permute_12_kernel<float>, dim3(pchunks, b.count), dim3(256), 0, s, pm);
          HIP_TRY(hipGetLastError());
          GemmArgs h{};
          h.a.base = ws + b.off_midinv[k - 1]; h.a.batch_stride = (int64_t)dk * dk; h.a.ld = dk;
          h.b.base = other; h.b.batch_stride = mn; h.b.ld = pre * post;
          h.c = cur; h.c_batch_stride = mn; h.ldc = pre * post;
          h.M = dk; h.N = pre * post; h.K = dk; h.alpha = 1.f; h.beta = 0.f;
          h.tiles_m = (h.M + BM - 1) / BM; h.tiles_n = (h.N + BN - 1) / BN; h.tiles = h.tiles_m * h.tiles_n; h.batch = b.count;
          rc = launch_gemm<ROW_CONTIG, ROW_CONTIG, float, float, EPI_STORE, false>(h, s);
          if (rc) return rc;
          pm.src = cur; pm.dst = other; pm.d1 = dk; pm.d2 = pre; pm.d3 = post;
          hipLaunchKernelGGL(permute_12_kernel<float>, dim3(pchunks, b.count), dim3(256), 0, s, pm);
          HIP_TRY(hipGetLastError());
          std::swap(cur, other);
          pre *= dk;
        }
        const int dl = b.dlast();
        GemmArgs q{};
        q.a.base = cur; q.a.batch_stride = mn; q.a.ld = dl;
        q.b.base = ws + b.off_Rinv; q.b.batch_stride = (int64_t)dl * dl; q.b.ld = dl;
        q.c = P; q.c_batch_stride = mn; q.ldc = dl;
        q.M = (int)(mn / dl); q.N = dl; q.K = dl; q.alpha = 1.f; q.beta = 0.f;
        q.tiles_m = (q.M + BM - 1) / BM; q.tiles_n = (q.N + BN - 1) / BN; q.tiles = q.tiles_m * q.tiles_n; q.batch = b.count;
        q.norm_partial = ssh;
        rc = launch_gemm<K_CONTIG, ROW_CONTIG, float, float, EPI_STORE_NORM, false>(q, s);
        if (rc) return rc;
        ssh_count = q.tiles;
      }
    } else if (use_shampoo && b.whole()) {
      // diagonal Shampoo: a diagonalised side scales rows / columns instead of multiplying
      StageTimer t(o, SHAMPOO_STAGE_PRECOND, s);
      DiagScaleArgs ds{};
      ds.desc = desc; ds.g_table = gd_tab; ds.m = b.m; ds.n = b.n; ds.geom = b.geom;
      const float *dl = reinterpret_cast<const float *>(ws + b.off_Linv), *dr = reinterpret_cast<const float *>(ws + b.off_Rinv);
      float *ssh = reinterpret_cast<float *>(ws + b.off_sshp);
      const unsigned ew_grid = (unsigned)b.geom.chunks * b.count;
      if (b.diagL && b.diagR) {
        ds.dl = dl; ds.dr = dr; ds.out = P; ds.norm_partial = ssh; ds.alpha = c1;
        hipLaunchKernelGGL(diag_scale_kernel<GD>, dim3(ew_grid), dim3(EW_THREADS), 0, s, ds);
        HIP_TRY(hipGetLastError());
        ssh_count = b.geom.chunks;
      } else if (b.diagL) {
        // T = D_L G, then P = T Rbar with per-tile sums of squares
        ds.dl = dl; ds.out = T; ds.alpha = c1;
        hipLaunchKernelGGL(diag_scale_kernel<GD>, dim3(ew_grid), dim3(EW_THREADS), 0, s, ds);
        HIP_TRY(hipGetLastError());
        GemmArgs h{};
        h.a.base = T; h.a.batch_stride = (int64_t)b.m * b.n; h.a.ld = b.n;
        h.b.base = ws + b.off_Rinv; h.b.batch_stride = (int64_t)b.n * b.n; h.b.ld = b.n;
        h.c = P; h.c_batch_stride = (int64_t)b.m * b.n; h.ldc = b.n;
        h.M = b.m; h.N = b.n; h.K = b.n; h.alpha = 1.f; h.beta = 0.f;
        h.tiles_m = b.tiles_m; h.tiles_n = b.tiles_n; h.tiles = b.tiles_m * b.tiles_n; h.batch = b.count;
        h.norm_partial = ssh;
        rc = launch_gemm<K_CONTIG, ROW_CONTIG, float, float, EPI_STORE_NORM, false>(h, s);
        if (rc) return rc;
      } else {
        // T = Lbar G, then P = T D_R
        GemmArgs g{};
        g.a.base = ws + b.off_Linv; g.a.batch_stride = (int64_t)b.m * b.m; g.a.ld = b.m;
        g.b.from_table = 1; g.desc = desc; g.ptr_table = gd_tab;
        g.c = T; g.c_batch_stride = (int64_t)b.m * b.n; g.ldc = b.n;
        g.M = b.m; g.N = b.n; g.K = b.m; g.alpha = c1; g.beta = 0.f;
        g.tiles_m = b.tiles_m; g.tiles_n = b.tiles_n; g.tiles = b.tiles_m * b.tiles_n; g.batch = b.count;
        rc = launch_gemm<ROW_CONTIG, ROW_CONTIG, float, GD, EPI_STORE, false>(g, s);
        if (rc) return rc;
        ds.src = T; ds.dr = dr; ds.out = P; ds.norm_partial = ssh; ds.alpha = 1.f;
        hipLaunchKernelGGL(diag_scale_kernel<float>, dim3(ew_grid), dim3(EW_THREADS), 0, s, ds);
        HIP_TRY(hipGetLastError());
        ssh_count = b.geom.chunks;
      }
    } else if (use_shampoo && sizeof(GD) == 2 && sizeof(GS) == 2 && b.planes && o->ptrs_aligned16) {
      // bf16 gradients: both products on the fp16 matrix cores, float32-accurate through
      // two-plane splits of the float32 operands (Lbar, T, Rbar), each scaled by a power of two
      // into the fp16 range; the gradient is one fp16 plane (exact: 8 significant bits).
      // B operands are read along k: G^T is the scaled fp16 transpose made for the factor update.
      const int tm128 = (b.m + 127) / 128, x2_tn = (b.n + X2_TN - 1) / X2_TN;
      // tiles of 256 rows (half the operand traffic per multiply) unless padding the rows to
      // 256 would add more than an eighth to the work
      // and unless there are too few of them to give every CU one
      const int tm256 = (b.m + 255) / 256;
      const bool tall = tm256 * 256 * 8 <= tm128 * 128 * 9 && (int64_t)tm256 * x2_tn * b.count >= 256;
      const int h_tm = tall ? tm256 : tm128;
      const int64_t per_h = ((int64_t)h_tm * x2_tn * b.count + NUM_XCD - 1) / NUM_XCD;
      ssh_count = h_tm * x2_tn;
      uint16_t *T2h = reinterpret_cast<uint16_t *>(T);
      const int64_t t_plane = (int64_t)b.count * b.m * b.n;
      {
      StageTimer t(o, SHAMPOO_STAGE_PRECOND, s);
      if (refresh) launch_x2_scales(b);   // the roots, and with them their scales, have just changed
      GemmX2Args g{};
      g.a = reinterpret_cast<const uint16_t *>(ws + b.off_Linv2h);
      g.a_plane_stride = (int64_t)b.count * b.m * b.m; g.a_batch_stride = (int64_t)b.m * b.m; g.lda = b.m;
      g.b = reinterpret_cast<const uint16_t *>(ws + b.off_Gt); g.b_plane_stride = 0;
      g.b_batch_stride = (int64_t)b.m * b.n; g.ldb = b.m;
      g.c2 = T2h; g.c2_plane_stride = t_plane; g.c_batch_stride = (int64_t)b.m * b.n; g.ldc = b.n;
      g.M = b.m; g.N = b.n; g.K = b.m; g.alpha = c1; g.out_scale = reinterpret_cast<const float *>(ws + b.off_t_scale);
      g.tiles_m = h_tm; g.tiles_n = x2_tn; g.batch = b.count;
      if (tall)
        hipLaunchKernelGGL((gemm_f16x2_kernel<256, 128, 1, X2_STORE_SPLIT>), dim3((unsigned)(per_h * NUM_XCD)), dim3(256), 0, s, g);
      else
        hipLaunchKernelGGL((gemm_f16x2_kernel<128, 64, 1, X2_STORE_SPLIT>), dim3((unsigned)(per_h * NUM_XCD)), dim3(256), 0, s, g);
      }
      StageTimer t2(o, SHAMPOO_STAGE_PRECOND2, s);
      GemmX2Args h{};
      h.a = T2h; h.a_plane_stride = t_plane; h.a_batch_stride = (int64_t)b.m * b.n; h.lda = b.n;
      h.b = reinterpret_cast<const uint16_t *>(ws + b.off_Rinv2h);
      h.b_plane_stride = (int64_t)b.count * b.n * b.n; h.b_batch_stride = (int64_t)b.n * b.n; h.ldb = b.n;
      h.c = P; h.c_batch_stride = (int64_t)b.m * b.n; h.ldc = b.n;
      h.M = b.m; h.N = b.n; h.K = b.n; h.alpha = 1.f; h.out_scale = reinterpret_cast<const float *>(ws + b.off_inv_ts);
      h.norm_partial = reinterpret_cast<float *>(ws + b.off_sshp);
      h.tiles_m = h_tm; h.tiles_n = x2_tn; h.batch = b.count;
      if (tall)
        hipLaunchKernelGGL((gemm_f16x2_kernel<256, 128, 2, X2_STORE_NORM>), dim3((unsigned)(per_h * NUM_XCD)), dim3(256), 0, s, h);
      else
        hipLaunchKernelGGL((gemm_f16x2_kernel<128, 64, 2, X2_STORE_NORM>), dim3((unsigned)(per_h * NUM_XCD)), dim3(256), 0, s, h);
      HIP_TRY(hipGetLastError());
    } else if (use_shampoo) {
      {
      StageTimer t(o, SHAMPOO_STAGE_PRECOND, s);
      GemmArgs g{};
      // T = Lbar G   (Lbar symmetric: A(i,k) read as Lbar[k][i], contiguous in i)
      g.a.base = ws + b.off_Linv; g.a.batch_stride = (int64_t)b.m * b.m; g.a.ld = b.m;
      g.b.from_table = 1; g.desc = desc; g.ptr_table = gd_tab;
      g.c = T; g.c_batch_stride = (int64_t)b.m * b.n; g.ldc = b.n;
      g.M = b.m; g.N = b.n; g.K = b.m; g.alpha = c1; g.beta = 0.f;
      g.tiles_m = b.tiles_m; g.tiles_n = b.tiles_n; g.tiles = b.tiles_m * b.tiles_n; g.batch = b.count;
      rc = launch_gemm<ROW_CONTIG, ROW_CONTIG, float, GD, EPI_STORE, false>(g, s);
      if (rc) return rc;
      }
      // P = T Rbar, with per-tile sums of squares
      StageTimer t2(o, SHAMPOO_STAGE_PRECOND2, s);
      GemmArgs h{};
      h.a.base = T; h.a.batch_stride = (int64_t)b.m * b.n; h.a.ld = b.n;
      h.b.base = ws + b.off_Rinv; h.b.batch_stride = (int64_t)b.n * b.n; h.b.ld = b.n;
      h.c = P; h.c_batch_stride = (int64_t)b.m * b.n; h.ldc = b.n;
      h.M = b.m; h.N = b.n; h.K = b.n; h.alpha = 1.f; h.beta = 0.f;
      h.tiles_m = b.tiles_m; h.tiles_n = b.tiles_n; h.tiles = b.tiles_m * b.tiles_n; h.batch = b.count;
      h.norm_partial = reinterpret_cast<float *>(ws + b.off_sshp);
      rc = launch_gemm<K_CONTIG, ROW_CONTIG, float, float, EPI_STORE_NORM, false>(h, s);
      if (rc) return rc;
    }
    {
      StageTimer t(o, SHAMPOO_STAGE_UPDATE, s);
      if (use_shampoo) {
        ScaleArgs sa;
        sa.sg_partial = reinterpret_cast<const float *>(ws + b.off_sgp); sa.sg_count = b.geom.chunks;
        sa.ssh_partial = reinterpret_cast<const float *>(ws + b.off_sshp); sa.ssh_count = ssh_count;
        sa.scale = scale; sa.norms = reinterpret_cast<float *>(ws + b.off_norms);
        hipLaunchKernelGGL(scale_kernel, dim3(b.count), dim3(64), 0, s, sa);
      }
      EwArgs e{};
      e.desc = desc; e.w_table = wtab; e.g_table = gs_tab; e.gd_table = gd_tab; e.a_state = A; e.m_state = M;
      e.p = P; e.scale = scale;
      e.m = b.m; e.n = b.n; e.geom = b.geom; e.graft_eps = c.graft_epsilon; e.mu = c.momentum; e.lr = lr;
      e.wd_decoupled = wd_dec; e.nesterov = c.use_nesterov ? 1 : 0; e.sgd_graft = sgd; e.gd_scale = c1;
      e.a_decay = a_decay; e.a_gain = a_gain; e.a_bc = a_bc;
      e.graft_only = use_shampoo ? 0 : 1;
      hipLaunchKernelGGL(update_kernel<GD>, dim3((unsigned)b.geom.chunks * b.count), dim3(EW_THREADS), 0, s, e);
      HIP_TRY(hipGetLastError());
    }
  }
  if (o->has_tensor) {
    // the updated block-contiguous copies go back into the caller's tensors
    StageTimer t(o, SHAMPOO_STAGE_UPDATE, s);
    for (int i = 0; i < c.n_params; ++i) {
      if (p.pshape[i].kind != P_TENSOR) continue;
      TensorCopyArgs ta = tensor_copy_args(i);
      ta.copy_in = ws + o->off_Wb[i]; ta.tensor_out = o->last_w[i];
      hipLaunchKernelGGL((tensor_block_copy_kernel<float, true>), tensor_copy_grid(i), dim3(256), 0, s, ta);
    }
    HIP_TRY(hipGetLastError());
  }
  if (!p.diag_chunks.empty()) {
    StageTimer t(o, SHAMPOO_STAGE_DIAG, s);
    DiagArgs d;
    d.chunks = reinterpret_cast<const DiagChunk *>(ws + o->off_diag);
    d.w_table = wtab; d.g_table = gtab; d.a_state = A; d.m_state = M; d.gf_state = Gf;
    d.graft_eps = c.graft_epsilon; d.mu = c.momentum; d.lr = lr;
    d.beta1 = c.beta1; d.wd_l2 = wd_l2; d.wd_decoupled = wd_dec; d.nesterov = c.use_nesterov ? 1 : 0;
    d.gd_scale = c1; d.a_decay = a_decay; d.a_gain = a_gain; d.a_bc = a_bc;
    hipLaunchKernelGGL(diag_kernel<GT>, dim3((unsigned)p.diag_chunks.size()), dim3(EW_THREADS), 0, s, d);
    HIP_TRY(hipGetLastError());
  }
  return SHAMPOO_OK;
}

}  // namespace

// ---------------------------------------------------------------------------
// extern "C" boundary
// ---------------------------------------------------------------------------
extern "C" {

int shampoo_plan(const shampoo_config *cfg, int64_t *table, int64_t cap, int64_t *n_blocks, int64_t *n_buckets) {
  const int rc = check_config(cfg);
  if (rc) return rc;
  if (cap < 0 || (cap > 0 && !table)) return SHAMPOO_ERR_NULL;
  Plan p;
  make_plan(cfg, p);
  if (const int rp = check_plan(p)) return rp;
  if (n_blocks) *n_blocks = (int64_t)p.blocks.size();
  if (n_buckets) *n_buckets = (int64_t)p.buckets.size();
  const int64_t cnt = std::min<int64_t>(cap, (int64_t)p.blocks.size());
  for (int64_t i = 0; i < cnt; ++i) {
    const Block &b = p.blocks[i];
    int64_t *row = table + 12 * i;
    row[0] = b.param; row[1] = b.row0; row[2] = b.col0; row[3] = b.m; row[4] = b.n;
    row[5] = b.bucket; row[6] = b.slot;
    row[7] = (p.buckets[b.bucket].diagL ? 1 : 0) | (p.buckets[b.bucket].diagR ? 2 : 0) | (b.tensor ? 4 | (p.buckets[b.bucket].modes << 4) : 0);
    row[8] = b.s3; row[9] = b.d3; row[10] = b.s4; row[11] = b.d4;
  }
  return SHAMPOO_OK;
}

size_t shampoo_workspace_bytes(const shampoo_config *cfg) {
  if (check_config(cfg)) return 0;
  Plan p;
  make_plan(cfg, p);
  if (check_plan(p)) return 0;
  return layout(cfg, p, nullptr);
}

int shampoo_create(const shampoo_config *cfg, void *workspace, size_t workspace_bytes, void *stream,
                   shampoo_opt **out) {
  if (!out) return SHAMPOO_ERR_NULL;
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc) return rc;
  shampoo_opt *o = new (std::nothrow) shampoo_opt();
  if (!o) return SHAMPOO_ERR_HIP;
  o->cfg = *cfg;
  o->ndim.assign(cfg->ndim, cfg->ndim + cfg->n_params);
  o->shape.assign(cfg->shape, cfg->shape + (size_t)SHAMPOO_MAX_NDIM * cfg->n_params);
  o->cfg.ndim = o->ndim.data();
  o->cfg.shape = o->shape.data();
  make_plan(&o->cfg, o->plan);
  if ((rc = check_plan(o->plan))) { delete o; return rc; }
  const size_t need = layout(&o->cfg, o->plan, o);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % ALIGN) != 0 || workspace_bytes < need) {
    delete o;
    return SHAMPOO_ERR_WORKSPACE;
  }
  o->ws = static_cast<unsigned char *>(workspace);
  o->ws_bytes = workspace_bytes;
  hipStream_t s = static_cast<hipStream_t>(stream);
  auto fail = [&](int code) { delete o; return code; };
  if (hipSetDevice(cfg->device) != hipSuccess) return fail(SHAMPOO_ERR_HIP);
  Plan &p = o->plan;
  // state: A = M = 0, L = R = 0, roots = I
  if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + o->off_A), 0.f, p.total_elems, s))) return fail(rc);
  if (cfg->momentum > 0.f)
    if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + o->off_M), 0.f, p.total_elems, s))) return fail(rc);
  if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + o->off_count), 0.f, 16, s))) return fail(rc);
  if (o->use_b1)
    if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + o->off_Gf), 0.f, p.total_elems, s))) return fail(rc);
  {
    // pointer tables of the library-owned gradient buffers (same layout as A / M)
    std::vector<void *> t1(cfg->n_params), t2(cfg->n_params);
    for (int i = 0; i < cfg->n_params; ++i) {
      t1[i] = o->use_l2 ? reinterpret_cast<float *>(o->ws + o->off_G1) + p.param_state_offset[i] : nullptr;
      t2[i] = o->use_b1 ? reinterpret_cast<float *>(o->ws + o->off_Gf) + p.param_state_offset[i] : nullptr;
    }
    if (hipMemcpyAsync(o->ws + o->off_g1tab, t1.data(), t1.size() * sizeof(void *), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipMemcpyAsync(o->ws + o->off_gftab, t2.data(), t2.size() * sizeof(void *), hipMemcpyHostToDevice, s) != hipSuccess)
      return fail(SHAMPOO_ERR_HIP);
    if ((o->use_l2 || o->use_b1) && !p.prep_chunks.empty())
      if (hipMemcpyAsync(o->ws + o->off_prep, p.prep_chunks.data(), p.prep_chunks.size() * sizeof(DiagChunk),
                         hipMemcpyHostToDevice, s) != hipSuccess)
        return fail(SHAMPOO_ERR_HIP);
    if (hipStreamSynchronize(s) != hipSuccess) return fail(SHAMPOO_ERR_HIP);   // t1, t2 go out of scope
  }
  std::vector<std::vector<BlockDesc>> descs(p.buckets.size()), descs3(p.buckets.size());
  for (size_t i = 0; i < p.buckets.size(); ++i) {
    descs[i].resize(p.buckets[i].count);
    if (p.buckets[i].t3) descs3[i].resize((size_t)p.buckets[i].count * p.buckets[i].split3);
  }
  for (const Block &b : p.blocks) {
    BlockDesc d;
    d.param = b.param;
    if (b.tensor) {
      // a block of the block-contiguous copy, as a d1 x (d2 d3) matrix; the second descriptor
      // shows the same memory as the (d1 d2) x d3 matrix of the third dimension
      d.ld = b.n * b.d3 * b.d4;
      d.offset = b.voff;
      d.state_offset = p.param_state_offset[b.param] + d.offset;
      // (one entry per row range of the split Gram product, see split3)
      const int sp = p.buckets[b.bucket].split3;
      for (int k = 0; k < sp; ++k) {
        BlockDesc d3 = d;
        d3.ld = p.buckets[b.bucket].dlast();
        d3.offset = b.voff + (int64_t)k * (b.m / sp) * d.ld;
        descs3[b.bucket][(size_t)b.slot * sp + k] = d3;
      }
    } else {
      d.ld = (int32_t)p.pshape[b.param].cols;
      d.offset = b.row0 * d.ld + b.col0;
      d.state_offset = p.param_state_offset[b.param] + d.offset;
    }
    descs[b.bucket][b.slot] = d;
  }
  for (size_t i = 0; i < p.buckets.size(); ++i) {
    Bucket &b = p.buckets[i];
    const int64_t B = b.count;
    if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + b.off_L), 0.f, B * (int64_t)b.l_elems(), s))) return fail(rc);
    if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + b.off_R), 0.f, B * (int64_t)b.r_elems(), s))) return fail(rc);
    if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + b.off_P), 0.f, B * b.m * b.n, s))) return fail(rc);
    if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + b.off_norms), 0.f, B * 2, s))) return fail(rc);
    if (b.t3) {
      for (int k = 0; k + 2 < b.modes; ++k) {
        const int64_t t2 = B * b.td[k + 1] * b.td[k + 1];
        if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + b.off_mid[k]), 0.f, t2, s))) return fail(rc);
        hipLaunchKernelGGL(eye_kernel, dim3((unsigned)((t2 + 255) / 256)), dim3(256), 0, s,
                           reinterpret_cast<float *>(o->ws + b.off_midinv[k]), b.td[k + 1], t2);
      }
      if (hipMemcpyAsync(o->ws + b.off_desc3, descs3[i].data(), descs3[i].size() * sizeof(BlockDesc),
                         hipMemcpyHostToDevice, s) != hipSuccess)
        return fail(SHAMPOO_ERR_HIP);
    }
    // roots start as the identity (a diagonalised side: the vector of ones)
    const int64_t tl = B * b.m * b.m, tr = B * (int64_t)b.rdim() * b.rdim();
    if (b.diagL) { if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + b.off_Linv), 1.f, B * b.m, s))) return fail(rc); }
    else hipLaunchKernelGGL(eye_kernel, dim3((unsigned)((tl + 255) / 256)), dim3(256), 0, s,
                            reinterpret_cast<float *>(o->ws + b.off_Linv), b.m, tl);
    if (b.diagR) { if ((rc = launch_fill(reinterpret_cast<float *>(o->ws + b.off_Rinv), 1.f, B * b.n, s))) return fail(rc); }
    else hipLaunchKernelGGL(eye_kernel, dim3((unsigned)((tr + 255) / 256)), dim3(256), 0, s,
                            reinterpret_cast<float *>(o->ws + b.off_Rinv), b.rdim(), tr);
    if (hipGetLastError() != hipSuccess) return fail(SHAMPOO_ERR_HIP);
    if (hipMemcpyAsync(o->ws + b.off_desc, descs[i].data(), descs[i].size() * sizeof(BlockDesc),
                       hipMemcpyHostToDevice, s) != hipSuccess)
      return fail(SHAMPOO_ERR_HIP);
  }
  if ((rc = split_roots(o, s))) return fail(rc);
  if (o->n_small > 0) {
    // largest blocks first, so that the tail of the launch is made of the cheapest workgroups
    std::vector<SmallBlock> small;
    for (size_t i = 0; i < p.buckets.size(); ++i) {
      const Bucket &b = p.buckets[i];
      if (b.m > SB || b.n > SB || b.whole() || b.t3) continue;
      for (int64_t k = 0; k < b.count; ++k) {
        SmallBlock sb;
        sb.d = descs[i][k]; sb.m = b.m; sb.n = b.n;
        sb.off_L = (int64_t)(b.off_L + (size_t)k * b.m * b.m * 4); sb.off_R = (int64_t)(b.off_R + (size_t)k * b.n * b.n * 4);
        sb.off_Linv = (int64_t)(b.off_Linv + (size_t)k * b.m * b.m * 4);
        sb.off_Rinv = (int64_t)(b.off_Rinv + (size_t)k * b.n * b.n * 4);
        sb.off_P = (int64_t)(b.off_P + (size_t)k * b.m * b.n * 4); sb.off_norms = (int64_t)(b.off_norms + (size_t)k * 8);
        small.push_back(sb);
      }
    }
    std::stable_sort(small.begin(), small.end(), [](const SmallBlock &x, const SmallBlock &y) {
      return (int64_t)x.m * x.n > (int64_t)y.m * y.n;
    });
    if (hipMemcpy(o->ws + o->off_small, small.data(), small.size() * sizeof(SmallBlock), hipMemcpyHostToDevice) != hipSuccess)
      return fail(SHAMPOO_ERR_HIP);
  }
  if (!p.diag_chunks.empty())
    if (hipMemcpyAsync(o->ws + o->off_diag, p.diag_chunks.data(), p.diag_chunks.size() * sizeof(DiagChunk),
                       hipMemcpyHostToDevice, s) != hipSuccess)
      return fail(SHAMPOO_ERR_HIP);
  if (hipStreamSynchronize(s) != hipSuccess) return fail(SHAMPOO_ERR_HIP);
  *out = o;
  return SHAMPOO_OK;
}

int shampoo_step(shampoo_opt *o, void *const *params, const void *const *grads, float lr, int64_t step,
                 void *stream) {
  if (!o || !params || !grads) return SHAMPOO_ERR_NULL;
  const int np = o->cfg.n_params;
  for (int i = 0; i < np; ++i)
    if (!params[i] || !grads[i]) return SHAMPOO_ERR_NULL;
  if (step < 0 || step <= o->last_step) return SHAMPOO_ERR_STEP;
  if (!std::isfinite(lr)) return SHAMPOO_ERR_HYPER;
  hipStream_t s = static_cast<hipStream_t>(stream);
  HIP_TRY(hipSetDevice(o->cfg.device));
  // pointer tables: re-sent only when they change
  bool same = (int)o->last_w.size() == np;
  for (int i = 0; same && i < np; ++i) same = o->last_w[i] == params[i] && o->last_g[i] == grads[i];
  if (!same) {
    o->last_w.assign(params, params + np);
    o->ptrs_aligned16 = true;
    for (int i = 0; i < np; ++i)
      if (reinterpret_cast<uintptr_t>(grads[i]) % 16 != 0) o->ptrs_aligned16 = false;
    o->last_g.resize(np);
    for (int i = 0; i < np; ++i) o->last_g[i] = const_cast<void *>(grads[i]);
    // The tables are copied from vectors that the handle owns.  An earlier copy may still be
    // reading them (the runtime is free to defer a copy from pageable memory), so the stream
    // is drained before they are overwritten: once per change of the caller's pointers.
    if (!o->tab_w.empty()) HIP_TRY(hipStreamSynchronize(s));
    o->tab_w = o->last_w; o->tab_g = o->last_g;
    // tensor parameters are worked on in block-contiguous copies inside the workspace
    for (int i = 0; i < np; ++i)
      if (o->plan.pshape[i].kind == P_TENSOR) { o->tab_w[i] = o->ws + o->off_Wb[i]; o->tab_g[i] = o->ws + o->off_Gb[i]; }
    HIP_TRY(hipMemcpyAsync(o->ws + o->off_wtab, o->tab_w.data(), np * sizeof(void *), hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(o->ws + o->off_gtab, o->tab_g.data(), np * sizeof(void *), hipMemcpyHostToDevice, s));
  }
  int rc;
  if (o->cfg.grad_dtype == SHAMPOO_GRAD_BF16) {
    if (o->use_l2) rc = step_impl<uint16_t, float, float>(o, lr, step, s);
    else if (o->use_b1) rc = step_impl<uint16_t, uint16_t, float>(o, lr, step, s);
    else rc = step_impl<uint16_t, uint16_t, uint16_t>(o, lr, step, s);
  } else {
    rc = step_impl<float, float, float>(o, lr, step, s);
  }
  // A step whose launches failed (SHAMPOO_ERR_HIP) leaves the state partly updated; the step
  // counter then stays where it was, so the error is not masked by SHAMPOO_ERR_STEP on a retry.
  if (rc == SHAMPOO_OK) o->last_step = step;
  return rc;
}

int shampoo_get(shampoo_opt *o, int32_t param, int32_t block, int32_t which, void *dst, size_t bytes,
                void *stream) {
  if (!o || !dst) return SHAMPOO_ERR_NULL;
  if (param < 0 || param >= o->cfg.n_params) return SHAMPOO_ERR_SHAPE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  HIP_TRY(hipSetDevice(o->cfg.device));
  Plan &p = o->plan;
  unsigned char *ws = o->ws;
  if (p.param_blocks[param].empty()) {   // 1-D, or a matrix on the diagonal-method path
    if (block != 0 || (which != SHAMPOO_GET_A && which != SHAMPOO_GET_M && which != SHAMPOO_GET_GF)) return SHAMPOO_ERR_SHAPE;
    if (which == SHAMPOO_GET_M && !(o->cfg.momentum > 0.f)) return SHAMPOO_ERR_SHAPE;
    if (which == SHAMPOO_GET_GF && !o->use_b1) return SHAMPOO_ERR_SHAPE;
    const size_t len = (size_t)p.pshape[param].elems();
    if (bytes != len * 4) return SHAMPOO_ERR_SHAPE;
    const size_t off_state = which == SHAMPOO_GET_A ? o->off_A : (which == SHAMPOO_GET_M ? o->off_M : o->off_Gf);
    const float *src = reinterpret_cast<const float *>(ws + off_state) + p.param_state_offset[param];
    HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, s));
    return SHAMPOO_OK;
  }
  if (block < 0 || block >= (int32_t)p.param_blocks[param].size()) return SHAMPOO_ERR_SHAPE;
  const Block &b = p.blocks[p.param_blocks[param][block]];
  const Bucket &bk = p.buckets[b.bucket];
  const size_t m = b.m, n = b.n;
  const unsigned char *src = nullptr;
  size_t need = 0;
  switch (which) {
    case SHAMPOO_GET_L:
    case SHAMPOO_GET_R: {
      const int rcf = complete_factors(o, (size_t)b.bucket, s);
      if (rcf) return rcf;
      need = (which == SHAMPOO_GET_L ? bk.l_elems() : bk.r_elems()) * 4;
      src = ws + (which == SHAMPOO_GET_L ? bk.off_L : bk.off_R) + (size_t)b.slot * need;
      break;
    }
    case SHAMPOO_GET_LINV: need = bk.l_elems() * 4; src = ws + bk.off_Linv + (size_t)b.slot * need; break;
    case SHAMPOO_GET_RINV: need = bk.r_elems() * 4; src = ws + bk.off_Rinv + (size_t)b.slot * need; break;
    case SHAMPOO_GET_L2:
    case SHAMPOO_GET_L2INV:
    case SHAMPOO_GET_L3:
    case SHAMPOO_GET_L3INV: {
      const int k = (which == SHAMPOO_GET_L2 || which == SHAMPOO_GET_L2INV) ? 0 : 1;
      if (!bk.t3 || k + 2 >= bk.modes) return SHAMPOO_ERR_SHAPE;
      need = (size_t)bk.td[k + 1] * bk.td[k + 1] * 4;
      src = ws + ((which == SHAMPOO_GET_L2 || which == SHAMPOO_GET_L3) ? bk.off_mid[k] : bk.off_midinv[k]) + (size_t)b.slot * need;
      break;
    }
    case SHAMPOO_GET_PSH: need = m * n * (size_t)b.d3 * b.d4 * 4; src = ws + bk.off_P + (size_t)b.slot * need; break;
    case SHAMPOO_GET_NORMS: src = ws + bk.off_norms + (size_t)b.slot * 8; need = 8; break;
    case SHAMPOO_GET_A:
    case SHAMPOO_GET_M:
    case SHAMPOO_GET_GF: {
      if (which == SHAMPOO_GET_M && !(o->cfg.momentum > 0.f)) return SHAMPOO_ERR_SHAPE;
      if (which == SHAMPOO_GET_GF && !o->use_b1) return SHAMPOO_ERR_SHAPE;
      const size_t off_state = which == SHAMPOO_GET_A ? o->off_A : (which == SHAMPOO_GET_M ? o->off_M : o->off_Gf);
      if (b.tensor) {   // state of a tensor parameter is kept block-contiguous
        const size_t need_t = m * n * (size_t)b.d3 * b.d4 * 4;
        if (bytes != need_t) return SHAMPOO_ERR_SHAPE;
        const float *base_t = reinterpret_cast<const float *>(ws + off_state) + p.param_state_offset[param] + b.voff;
        HIP_TRY(hipMemcpyAsync(dst, base_t, need_t, hipMemcpyDeviceToDevice, s));
        return SHAMPOO_OK;
      }
      if (bytes != m * n * 4) return SHAMPOO_ERR_SHAPE;
      const int64_t ld = p.pshape[param].cols;
      const float *base = reinterpret_cast<const float *>(ws + off_state) +
                          p.param_state_offset[param] + b.row0 * ld + b.col0;
      HIP_TRY(hipMemcpy2DAsync(dst, n * 4, base, (size_t)ld * 4, n * 4, m, hipMemcpyDeviceToDevice, s));
      return SHAMPOO_OK;
    }
    default: return SHAMPOO_ERR_SHAPE;
  }
  if (bytes != need) return SHAMPOO_ERR_SHAPE;
  HIP_TRY(hipMemcpyAsync(dst, src, need, hipMemcpyDeviceToDevice, s));
  return SHAMPOO_OK;
}

int shampoo_status(shampoo_opt *o, void *stream, int64_t *n_refreshes, int64_t *n_failed_roots) {
  if (!o) return SHAMPOO_ERR_NULL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  HIP_TRY(hipSetDevice(o->cfg.device));
  unsigned long long cnt = 0;
  HIP_TRY(hipMemcpyAsync(&cnt, o->ws + o->off_count, sizeof(cnt), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  if (n_refreshes) *n_refreshes = o->n_refresh;
  if (n_failed_roots) *n_failed_roots = (int64_t)cnt;
  return SHAMPOO_OK;
}

int shampoo_set_timing(shampoo_opt *o, int32_t enable) {
  if (!o) return SHAMPOO_ERR_NULL;
  o->timing = enable != 0;
  return SHAMPOO_OK;
}

int shampoo_get_timing(shampoo_opt *o, int32_t stage, double *ms_total, int64_t *intervals) {
  if (!o || !ms_total || !intervals) return SHAMPOO_ERR_NULL;
  if (stage < 0 || stage >= SHAMPOO_STAGE_COUNT) return SHAMPOO_ERR_SHAPE;
  double total = 0.0;
  int64_t cnt = 0;
  int rc = SHAMPOO_OK;
  for (auto &iv : o->intervals[stage]) {
    float ms = 0.f;
    if (hipEventSynchronize(iv.b) != hipSuccess || hipEventElapsedTime(&ms, iv.a, iv.b) != hipSuccess)
      rc = SHAMPOO_ERR_HIP;
    else { total += ms; ++cnt; }
    (void)hipEventDestroy(iv.a);
    (void)hipEventDestroy(iv.b);
  }
  o->intervals[stage].clear();
  *ms_total = total;
  *intervals = cnt;
  return rc;
}

int shampoo_destroy(shampoo_opt *o) {
  if (!o) return SHAMPOO_ERR_NULL;
  for (auto &v : o->intervals)
    for (auto &iv : v) { (void)hipEventDestroy(iv.a); (void)hipEventDestroy(iv.b); }
  if (o->aux.state == 1) { (void)hipSetDevice(o->cfg.device); o->aux.release(); }
  delete o;
  return SHAMPOO_OK;
}

size_t shampoo_root_inverse_workspace_bytes(int32_t n, int32_t batch) {
  if (n < 1 || batch < 1 || n > MAX_BLOCK_SIZE) return 0;
  return eig_layout(n, batch).bytes;
}

int shampoo_root_inverse(const float *a, int32_t n, int32_t batch, float epsilon, float r, float *x,
                         float *lambda, int32_t *failed, void *workspace, size_t workspace_bytes, void *stream) {
  if (!a || !x) return SHAMPOO_ERR_NULL;
  if (n < 1 || batch < 1) return SHAMPOO_ERR_SHAPE;
  if (n > MAX_BLOCK_SIZE) return SHAMPOO_ERR_UNSUPPORTED;
  if (!(epsilon > 0.f) || !std::isfinite(epsilon) || !(r > 0.f) || !std::isfinite(r)) return SHAMPOO_ERR_HYPER;
  const EigLayout e = eig_layout(n, batch);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % ALIGN) != 0 || workspace_bytes < e.bytes)
    return SHAMPOO_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (failed) {
    const int rc = launch_fill(reinterpret_cast<float *>(failed), 0.f, batch, s);
    if (rc) return rc;
  }
  // The helper streams of the stand-alone call are shared by every caller of a device: the
  // lock keeps one call's fork / join events together while its work is enqueued.
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES || n <= JAC_SMALL_MAX)
    return root_inverse_batched(a, n, batch, epsilon, r, 1.f, x, lambda, failed, nullptr,
                                static_cast<unsigned char *>(workspace), e, s, nullptr);
  std::lock_guard<std::mutex> lock(per_device[dev].mutex);
  return root_inverse_batched(a, n, batch, epsilon, r, 1.f, x, lambda, failed, nullptr,
                              static_cast<unsigned char *>(workspace), e, s, &per_device[dev].aux);
}

size_t shampoo_root_inverse_warm_workspace_bytes(int32_t n, int32_t batch) {
  if (n <= JAC_SMALL_MAX || batch < 1 || n > MAX_BLOCK_SIZE) return 0;
  return eig_layout(n, batch, EIG_CHUNK_BYTES, 0, true).bytes;
}

int shampoo_root_inverse_warm(const float *a, int32_t n, int32_t batch, float epsilon, float r, float *x,
                              float *lambda, int32_t *failed, float *qt, int32_t start, int32_t *sweeps,
                              void *workspace, size_t workspace_bytes, void *stream) {
  if (!a || !x || !qt) return SHAMPOO_ERR_NULL;
  if (n < 1 || batch < 1) return SHAMPOO_ERR_SHAPE;
  if (n > MAX_BLOCK_SIZE || n <= JAC_SMALL_MAX) return SHAMPOO_ERR_UNSUPPORTED;
  if (!(epsilon > 0.f) || !std::isfinite(epsilon) || !(r > 0.f) || !std::isfinite(r)) return SHAMPOO_ERR_HYPER;
  const EigLayout e = eig_layout(n, batch, EIG_CHUNK_BYTES, 0, true);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % ALIGN) != 0 || workspace_bytes < e.bytes)
    return SHAMPOO_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(qt) % 16 != 0) return SHAMPOO_ERR_WORKSPACE;   // the kernels move it 16 bytes at a time
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (failed) {
    const int rc = launch_fill(reinterpret_cast<float *>(failed), 0.f, batch, s);
    if (rc) return rc;
  }
  WarmStart w;
  w.qt = qt; w.start = start != 0; w.sweeps = sweeps;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES)
    return root_inverse_batched(a, n, batch, epsilon, r, 1.f, x, lambda, failed, nullptr,
                                static_cast<unsigned char *>(workspace), e, s, nullptr, nullptr, w);
  std::lock_guard<std::mutex> lock(per_device[dev].mutex);
  return root_inverse_batched(a, n, batch, epsilon, r, 1.f, x, lambda, failed, nullptr,
                              static_cast<unsigned char *>(workspace), e, s, &per_device[dev].aux, nullptr, w);
}

int shampoo_root_inverse_static(const float *a, int32_t n, int32_t batch, float epsilon, float r, float *x,
                                float *lambda, int32_t *failed, void *stream) {
  if (!a || !x) return SHAMPOO_ERR_NULL;
  if (n < 1 || batch < 1) return SHAMPOO_ERR_SHAPE;
  if (n > SHAMPOO_STATIC_MAX_N) return SHAMPOO_ERR_UNSUPPORTED;
  if (!(epsilon > 0.f) || !std::isfinite(epsilon) || !(r > 0.f) || !std::isfinite(r)) return SHAMPOO_ERR_HYPER;
  const EigLayout e = eig_layout(n, batch, SHAMPOO_STATIC_SCRATCH_BYTES, SHAMPOO_STATIC_SCRATCH_BYTES);
  if (e.bytes == 0 || e.bytes > SHAMPOO_STATIC_SCRATCH_BYTES) return SHAMPOO_ERR_UNSUPPORTED;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return SHAMPOO_ERR_UNSUPPORTED;
  unsigned char *ws = nullptr;
  {
    // every GPU holds its own copy of the array at its own address: looked up once per device
    std::lock_guard<std::mutex> lock(per_device[dev].mutex);
    if (!per_device[dev].scratch) {
      void *ptr = nullptr;
      HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
      if (!ptr) return SHAMPOO_ERR_HIP;
      per_device[dev].scratch = static_cast<unsigned char *>(ptr);
    }
    ws = per_device[dev].scratch;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (failed) {
    const int rc = launch_fill(reinterpret_cast<float *>(failed), 0.f, batch, s);   // a fill kernel, not a memset node
    if (rc) return rc;
  }
  // everything on the caller's stream: no helper streams are created on this path
  return root_inverse_batched(a, n, batch, epsilon, r, 1.f, x, lambda, failed, nullptr, ws, e, s, nullptr);
}

size_t shampoo_root_inverse_newton_workspace_bytes(int32_t n, int32_t batch) {
  if (n < 1 || batch < 1 || n > MAX_BLOCK_SIZE) return 0;
  return newton_layout(n, batch).bytes;
}

int shampoo_root_inverse_newton(const float *a, int32_t n, int32_t batch, float epsilon, int32_t p, float tolerance,
                                int32_t max_iterations, float *x, int32_t *iterations, int32_t *failed,
                                void *workspace, size_t workspace_bytes, void *stream) {
  if (!a || !x) return SHAMPOO_ERR_NULL;
  if (n < 1 || batch < 1) return SHAMPOO_ERR_SHAPE;
  if (n > MAX_BLOCK_SIZE || !newton_p_supported(p)) return SHAMPOO_ERR_UNSUPPORTED;
  if (!(epsilon >= 0.f) || !std::isfinite(epsilon) || !(tolerance > 0.f) || !std::isfinite(tolerance) ||
      max_iterations < 1 || max_iterations > 1000)
    return SHAMPOO_ERR_HYPER;
  const NewtonLayout e = newton_layout(n, batch);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % ALIGN) != 0 || workspace_bytes < e.bytes)
    return SHAMPOO_ERR_WORKSPACE;
  return newton_root_batched(a, n, batch, epsilon, p, 1.f, tolerance, max_iterations, x, iterations, failed, nullptr,
                             static_cast<unsigned char *>(workspace), e, static_cast<hipStream_t>(stream));
}

int shampoo_jacobi_pair(int32_t s, int32_t halves, int32_t round, int32_t k, int32_t *p, int32_t *q) {
  if (!p || !q) return SHAMPOO_ERR_NULL;
  if (s < 2 || (s & 1) || round < 0 || round >= s - 1 || k < 0 || k >= s / 2) return SHAMPOO_ERR_SHAPE;
  if (halves == 1 && (s < 4 || ((s / 2) & (s / 2 - 1)) != 0)) return SHAMPOO_ERR_SHAPE;
  if (halves == 2 && s % 4 != 0) return SHAMPOO_ERR_SHAPE;
  if (halves < 0 || halves > 2) return SHAMPOO_ERR_SHAPE;
  int pp, qq;
  if (halves == 2) grouped_pair(s, 2, round, k, pp, qq);
  else if (halves) halves_pair(s, round, k, pp, qq); else rr_pair(s, round, k, pp, qq);
  *p = pp; *q = qq;
  return SHAMPOO_OK;
}

const char *shampoo_strerror(int code) {
  switch (code) {
    case SHAMPOO_OK: return "success";
    case SHAMPOO_ERR_NULL: return "a required pointer is NULL";
    case SHAMPOO_ERR_SHAPE: return "bad shape, dimension count, block size, index or byte count";
    case SHAMPOO_ERR_HYPER: return "hyper-parameter out of range";
    case SHAMPOO_ERR_WORKSPACE: return "workspace NULL, misaligned or too small";
    case SHAMPOO_ERR_STEP: return "step must be non-negative and strictly increasing";
    case SHAMPOO_ERR_HIP: return "a HIP runtime call failed";
    case SHAMPOO_ERR_UNSUPPORTED: return "size outside the supported range";
    default: return "unknown error code";
  }
}

}  // extern "C"
