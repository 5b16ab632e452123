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
//    blocks are applied to A (both sides, A_kl <- J_k^T A_kl J_l; float32 MFMA in
//    the first sweeps of a cold solve, float64 MFMA afterwards) and to the rows of
//    Q^T.  When the number of block columns is a multiple of 4 the rounds are
//    ordered so that two consecutive ones stay inside four block columns
//    (grouped_pair); Q^T then takes both in one pass over memory, on the fp16
//    matrix cores with operands split into two fp16 terms, and the pivots of all
//    rounds but the first of a sweep rotate only the pairs across their two block
//    columns.  The reconstruction Q f(Lambda) Q^T reuses the batched SYRK kernel.
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
constexpr int JAC_PIV_THREADS = 256;   // workgroup of the 64 x 64 pivot solver
constexpr int JAC_NB = 32;            // block-column width of the block solver
constexpr int JAC_PIV = 2 * JAC_NB;   // pivot size
constexpr int JAC_SMALL_MAX = 128;    // largest n solved entirely in LDS
constexpr int JAC_SMALL_SWEEPS = 20;
constexpr int JAC_OUTER_SWEEPS = 24;   // float32 and float64 sweeps of the block solver together (a cap: converged matrices skip)
constexpr int JAC_INNER_SWEEPS = 1;    // 2: 256 roots of n = 1024 in 1.00 s instead of 0.80 s
// rotation thresholds |a_pq| > rel * sqrt(|a_pp a_qq|) and > abs * max|diag(input)|
constexpr double JAC_SMALL_TOL_REL = 1e-11;   // LDS solver (n <= 128), float64 copy of the factor
// Block solver: an off-diagonal element left at tau sqrt(a_ii a_jj) tilts the two
// eigenvectors by a_ij / (lambda_i - lambda_j) and changes f(A) by about |f'| |a_ij|
// <= tau f / 4, i.e. sqrt(n) tau / 4 ~ 1e-6 over a 1024-matrix: below the float32
// accuracy of the accumulated Q, and one sweep cheaper than 1e-11.
constexpr double JAC_BLOCK_TOL_REL = 1e-7;
constexpr double JAC_SMALL_TOL_ABS = 1e-15;
// The float32 sweeps of a cold block solve: as many as it takes float32 to run out of
// resolution (pairs below 1e-6 of their diagonal entries, or below 2e-7 of the largest
// diagonal entry, are left to the float64 sweeps that follow).
constexpr int JAC_F32_SWEEPS = 9;
constexpr int JAC_F32_SWEEPS_WARM = 6;     // warm start: W = Qt A Qt^T is nearly diagonal already
constexpr int JAC_F32_SWEEPS_YOUNG = 10;   // for factors known to be badly conditioned (few gradient columns so far)
constexpr double JAC_F32_TOL_REL = 1e-6;
constexpr double JAC_F32_TOL_ABS = 2e-7;

// blocks of the two-sided update per thread: s / 2 (s / 2 + 1) / 2 blocks must fit on the
// workgroup, which holds for the two uses (s <= 64 on 256 threads, s <= 128 on 1024)
constexpr int JAC_BLOCKS_PER_THREAD = 3;
static_assert((JAC_PIV / 2) * (JAC_PIV / 2 + 1) / 2 <= JAC_BLOCKS_PER_THREAD * JAC_PIV_THREADS, "pivot blocks per thread");
static_assert(32 * 33 / 2 <= JAC_BLOCKS_PER_THREAD * 256 && (JAC_SMALL_MAX / 2) * (JAC_SMALL_MAX / 2 + 1) / 2 <= JAC_BLOCKS_PER_THREAD * 1024,
              "LDS solver blocks per thread");

struct JacScratch {      // small per-workgroup LDS arrays
  // per rotation of the current round: (sin, sin / (1 + cos)) and (p, q, offset of row p, offset
  // of row q in the LDS matrix), each read with one 16-byte LDS access
  double2 st[JAC_SMALL_MAX / 2];
  int4 pq[JAC_SMALL_MAX / 2];
  int flag;
  unsigned rounds[4];     // bit r: round r of the current sweep has a pair above the threshold
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

// The pivots of the block solver are made of two index halves whose diagonal blocks were
// diagonalised by the pivots before (up to what one sweep leaves behind), so their sweeps
// take the pairs in a different order: rounds 0 .. s / 2 - 1 hold the pairs across the halves
// (index k of the first with index (k + r) mod s / 2 of the second), rounds s / 2 .. s - 2 the
// pairs within the halves (both halves play the same tournament at once).  From the second
// visit on the rounds within the halves find nothing above the threshold and are skipped whole.
// s / 2 must be a power of two.
__device__ __host__ __forceinline__ void halves_pair(int s, int r, int k, int &p, int &q) {
  const int h = s >> 1;
  if (r < h) { p = k; q = h + ((k + r) & (h - 1)); }
  else {
    rr_pair(h, r - h, k & ((h >> 1) - 1), p, q);
    if (k >= (h >> 1)) { p += h; q += h; }
  }
}
// the round in which halves_pair brings i and j together (j < i)
__device__ __forceinline__ int halves_round(int s, int i, int j) {
  const int h = s >> 1;
  if (j < h && i >= h) return (i - h - j) & (h - 1);
  const int il = i & (h - 1), jl = j & (h - 1);
  return h + ((il == h - 1) ? jl : ((il + jl) * (h >> 1)) % (h - 1));
}

// The rounds of the block solver over `cnt` block columns.  group == 1: the plain tournament.
// group == 2 (cnt a multiple of 4): block columns 2 S and 2 S + 1 form a super-column; round 0
// pairs the two members of every super-column, and the super-columns then play a tournament of
// their own in which every meeting (S, T) takes two consecutive rounds, 1 + 2 R and 2 + 2 R:
// first (2 S, 2 T) and (2 S + 1, 2 T + 1), then (2 S, 2 T + 1) and (2 S + 1, 2 T).  Every pair of
// block columns still meets exactly once per sweep, and the two rounds of a meeting stay inside
// four block columns, so the rows of Q^T they rotate can take both rotations in one pass over
// memory.  Pivot k of a round belongs to meeting k / 2.
__device__ __host__ __forceinline__ void grouped_pair(int cnt, int group, int r, int k, int &p, int &q) {
  if (group == 1) { rr_pair(cnt, r, k, p, q); return; }
  if (r == 0) { p = 2 * k; q = 2 * k + 1; return; }
  const int R = (r - 1) >> 1, sub = (r - 1) & 1, i = k & 1;
  int S, T;
  rr_pair(cnt >> 1, R, k >> 1, S, T);
  p = 2 * S + i; q = 2 * T + (i ^ sub);
}

// 1 / sqrt(x) and 1 / x for finite x > 0 (x != 0 for the reciprocal) to float64 accuracy:
// hardware estimate + three Newton steps (each squares the relative error)
__device__ __forceinline__ double rsqrt_newton(double x) {
  double y = __builtin_amdgcn_rsq(x);
#pragma unroll
  for (int it = 0; it < 3; ++it) y = y * (1.5 - 0.5 * x * y * y);
  return y;
}
__device__ __forceinline__ double rcp_newton(double x) {
  double y = __builtin_amdgcn_rcp(x);
#pragma unroll
  for (int it = 0; it < 3; ++it) y = y * (2.0 - x * y);
  return y;
}

// float32 versions (the float32 sweeps of the mixed-precision block solver): the hardware
// estimates are good to about one unit in the last place; one Newton step each
__device__ __forceinline__ float rsqrt_newton(float x) {
  float y = __builtin_amdgcn_rsqf(x);
  return y * (1.5f - 0.5f * x * y * y);
}
__device__ __forceinline__ float rcp_newton(float x) {
  float y = __builtin_amdgcn_rcpf(x);
  return y * (2.0f - x * y);
}
__device__ __forceinline__ double jac_abs(double x) { return fabs(x); }
__device__ __forceinline__ float jac_abs(float x) { return fabsf(x); }
__device__ __forceinline__ double jac_copysign(double x, double y) { return copysign(x, y); }
__device__ __forceinline__ float jac_copysign(float x, float y) { return copysignf(x, y); }

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
// SQUARE: At is instead a full square array with row stride LDA (odd): every
// LDS access of a round is then bank-conflict free, at twice the footprint; the
// mirror image of each updated block is written as well.
// Returns nonzero if any rotation was applied.  All NT threads of the workgroup must call it.
// HALVES: the pair order of halves_pair instead of the plain tournament.
// T: float64, or float32 for the first sweeps of the mixed-precision block solver.
template <bool SQUARE, int NT, bool HALVES = false, typename T = double>
__device__ int jacobi_sweeps(T *At, float *Js, int s, const int LD, const int LDA, int max_sweeps,
                             T tol_rel, T tol_abs, JacScratch *sc) {
  const int tid = threadIdx.x;
  const int half = s >> 1;
  auto at = [LDA](int i, int j) { return SQUARE ? i * LDA + j : tri(i, j); };
  // the same from row offsets (i LDA, or i (i + 1) / 2 for the packed triangle) computed once per rotation
  auto rowoff = [LDA](int i) { return SQUARE ? i * LDA : i * (i + 1) / 2; };
  auto atr = [](int i, int ri, int j, int rj) { return SQUARE ? ri + j : (i >= j ? ri + j : rj + i); };
  int any = 0;
  // this thread's blocks (k, l), l <= k, of the two-sided update: numbers tid, tid + NT, ...
  // of the half (half + 1) / 2 blocks (at most UB each: 528 on 256 threads at s = 64, 2080 on
  // 1024 at s = 128)
  constexpr int UB = JAC_BLOCKS_PER_THREAD;
  int bk[UB], bl[UB];
#pragma unroll
  for (int u = 0; u < UB; ++u) {
    const int bnum = tid + u * NT;
    bk[u] = -1; bl[u] = 0;
    if (bnum < half * (half + 1) / 2) {
      int k = (int)((sqrtf(8.f * (float)bnum + 1.f) - 1.f) * 0.5f);
      while ((k + 1) * (k + 2) / 2 <= bnum) ++k;
      while (k * (k + 1) / 2 > bnum) --k;
      bk[u] = k; bl[u] = bnum - k * (k + 1) / 2;
    }
  }
  for (int sw = 0; sw < max_sweeps; ++sw) {
    if (tid == 0) sc->flag = 0;
    if (tid < 4) sc->rounds[tid] = 0u;
    __syncthreads();
    // Which rounds of this sweep have anything to do: every pair is held against the
    // threshold once, up front, and a round without a pair above it is skipped whole (two
    // barriers and an LDS round trip each: in the late sweeps of a solve that is most rounds,
    // and in the block solver most pivots).  A pair that other rotations of this sweep push
    // over the threshold waits for the next sweep, which only ends the iteration when no
    // pair is above the threshold at its start.  Pair (p, q), p < q, meets in round
    // r = p if q = s - 1, else r with 2 r = p + q (mod s - 1), i.e. r = (p + q) (s / 2) mod (s - 1).
    {
      const int JW = s > 64 ? 128 : 64;                 // columns per row pass
      const int j = tid & (JW - 1);
      for (int i = tid / JW; i < s; i += NT / JW) {
        if (j >= i) continue;                           // j < i < s
        const T aij = jac_abs(At[at(i, j)]);
        if (aij > tol_abs && aij * aij > tol_rel * tol_rel * jac_abs(At[at(i, i)] * At[at(j, j)])) {
          const int r = HALVES ? halves_round(s, i, j) : (i == s - 1) ? j : ((i + j) * half) % (s - 1);
          atomicOr(&sc->rounds[r >> 5], 1u << (r & 31));
        }
      }
    }
    __syncthreads();
    for (int r = 0; r < s - 1; ++r) {
      if (!((sc->rounds[r >> 5] >> (r & 31)) & 1u)) continue;      // uniform
      if (tid < half) {
        int p, q;
        if (HALVES) halves_pair(s, r, tid, p, q); else rr_pair(s, r, tid, p, q);   // p < q
        const T app = At[at(p, p)], aqq = At[at(q, q)], apq = At[at(q, p)];
        T sn = 0, tp = 0;
        const T aa = jac_abs(apq);
        if (aa > tol_abs && aa * aa > tol_rel * tol_rel * jac_abs(app * aqq)) {
          // t = tan of the rotation angle, the smaller root of t^2 + 2 zeta t - 1 = 0 with
          // zeta = (a_qq - a_pp) / (2 a_pq):  t = h / (d + sign(d) sqrt(d^2 + h^2)).
          // This chain is the serial part of every round (32 lanes work, 224 wait), so the
          // square root and the reciprocals start from the hardware estimates and are
          // polished by Newton steps instead of going through the full library routines.
          const T d = aqq - app, h = (T)2 * apq;
          const T x = d * d + h * h;
          const T hyp = x * rsqrt_newton(x);
          const T t = h * rcp_newton(d + jac_copysign(hyp, d));
          const T c = rsqrt_newton((T)1 + t * t);   // cos
          sn = t * c;
          tp = sn * rcp_newton((T)1 + c);                 // sin / (1 + cos)
          if (!(jac_abs(sn) <= (T)1)) { sn = 0; tp = 0; }   // non-finite: leave the pair alone
          if (sn != (T)0) sc->flag = 1;
        }
        sc->st[tid] = make_double2((double)sn, (double)tp); sc->pq[tid] = make_int4(p, q, rowoff(p), rowoff(q));
      }
      __syncthreads();
      // A <- R^T A R on the blocks (k, l) with l <= k, dealt evenly over the threads (block
      // k (k + 1) / 2 + l to thread (that number) mod NT: a (k, l) grid with the half above the
      // diagonal switched off would cost every wavefront all of its slots).  Blocks are
      // independent, so a thread first loads all of its blocks, then rotates, then stores (the
      // loads overlap).
      {
        T a[UB], b[UB], c[UB], d[UB], sk[UB], tk[UB], sl[UB], tl[UB];
        int ia[UB], ib[UB], ic[UB], id[UB];
        int4 k4[UB], l4[UB];
        bool act[UB];
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          act[u] = bk[u] >= 0;
          if (act[u]) {
            const double2 stk = sc->st[bk[u]], stl = sc->st[bl[u]];
            sk[u] = (T)stk.x; tk[u] = (T)stk.y; sl[u] = (T)stl.x; tl[u] = (T)stl.y;
            act[u] = !(sk[u] == (T)0 && sl[u] == (T)0);
            if (act[u]) {
              k4[u] = sc->pq[bk[u]]; l4[u] = sc->pq[bl[u]];
              ia[u] = atr(k4[u].x, k4[u].z, l4[u].x, l4[u].z); ib[u] = atr(k4[u].x, k4[u].z, l4[u].y, l4[u].w);
              ic[u] = atr(k4[u].y, k4[u].w, l4[u].x, l4[u].z); id[u] = atr(k4[u].y, k4[u].w, l4[u].y, l4[u].w);
              a[u] = At[ia[u]]; b[u] = At[ib[u]]; c[u] = At[ic[u]]; d[u] = At[id[u]];
            }
          }
        }
#pragma unroll
        for (int u = 0; u < UB; ++u) {
          if (!act[u]) continue;
          // rows: (a, c) and (b, d) are (x, y) pairs of rotation k
          const T a1 = a[u] - sk[u] * (c[u] + tk[u] * a[u]), c1 = c[u] + sk[u] * (a[u] - tk[u] * c[u]);
          const T b1 = b[u] - sk[u] * (d[u] + tk[u] * b[u]), d1 = d[u] + sk[u] * (b[u] - tk[u] * d[u]);
          // columns: (a1, b1) and (c1, d1) are (x, y) pairs of rotation l
          const T a2 = a1 - sl[u] * (b1 + tl[u] * a1), b2 = b1 + sl[u] * (a1 - tl[u] * b1);
          const T c2 = c1 - sl[u] * (d1 + tl[u] * c1), d2 = d1 + sl[u] * (c1 - tl[u] * d1);
          if (bk[u] == bl[u]) {   // pivot block: (p, q) and (q, p) are the annihilated element
            At[ia[u]] = a2; At[ib[u]] = (T)0; At[id[u]] = d2;
            if (SQUARE) At[ic[u]] = (T)0;
          } else {
            At[ia[u]] = a2; At[ib[u]] = b2; At[ic[u]] = c2; At[id[u]] = d2;
            if (SQUARE) {
              At[l4[u].z + k4[u].x] = a2; At[l4[u].w + k4[u].x] = b2; At[l4[u].z + k4[u].y] = c2; At[l4[u].w + k4[u].y] = d2;
            }
          }
        }
      }
      // J <- J R (columns), same load / rotate / store batching over rows
      constexpr int V = NT >= 1024 ? 4 : 8;
      for (int l = tid & 31; l < half; l += 32) {
        const double2 stl = sc->st[l];
        const float sl = (float)stl.x;
        if (sl == 0.f) continue;
        const float tl = (float)stl.y;
        const int4 l4 = sc->pq[l];
        const int pl = l4.x, ql = l4.y;
        for (int i0 = tid >> 5; i0 < s; i0 += (NT / 32) * V) {
          float x[V], y[V];
#pragma unroll
          for (int u = 0; u < V; ++u) {
            const int i = i0 + (NT / 32) * u;
            if (i < s) { x[u] = Js[i * LD + pl]; y[u] = Js[i * LD + ql]; }
          }
#pragma unroll
          for (int u = 0; u < V; ++u) {
            const int i = i0 + (NT / 32) * u;
            if (i < s) {
              Js[i * LD + pl] = x[u] - sl * (y[u] + tl * x[u]);
              Js[i * LD + ql] = y[u] + sl * (x[u] - tl * y[u]);
            }
          }
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

// One sweep over the pairs ACROSS the two halves of a 64 x 64 pivot (index k of the first half
// with index (k + r) mod 32 of the second in round r = 0 .. 31), with the matrix and the
// accumulated rotations in registers instead of LDS.  This is what the pivots of the block
// solver run in all rounds but the first of a sweep.
//
// The pairs of a round are the same for every round if the second half is thought of as moving:
// round r pairs position k of the first half with position k of the second, where position k of
// the second half holds index (k + r) mod 32.  In that picture a thread keeps the 2 x 2 blocks
//   a = A[k][l]   b = A[k][32 + s(l)]   c = A[32 + s(k)][l]   d = A[32 + s(k)][32 + s(l)],   s(k) = (k + r) mod 32
// of fixed (k, l) for the whole sweep, rotates them with the parameters of pairs k (rows) and l
// (columns), and then lets the second half move on by one position: b comes from block
// (k, l + 1), c from (k + 1, l), d from (k + 1, l + 1); a stays.  256 threads: lane % 32 = l,
// q = 2 wave + lane / 32, blocks k = 4 q .. 4 q + 3 (all 1024 blocks: the symmetric half is computed
// too, which keeps every exchange a shift).  A shift along l is a lane rotation inside 32 lanes
// (ds_bpermute: no LDS memory involved), a shift along k is a register move for three of the
// four blocks and goes through a small LDS array for the fourth.  The accumulated rotations
// J (64 x 64) are held the same way: thread (l, q) keeps columns l and 32 + s(l) of rows
// 8 q .. 8 q + 7, and only the second of them moves.  After 32 rounds every index is back at
// its own position.  Per thread and round about 25 LDS-pipe operations and no address
// arithmetic, where the LDS version takes 100 and a third of its vector instructions on
// addresses.
template <typename T> struct JacPair { T s, t; };     // sin, sin / (1 + cos)
template <typename T> struct JacCrossScratch {
  JacPair<T> st[JAC_PIV / 2];
  T exc[8 * 32], exd[8 * 32];
  int todo, rotated;
};

__device__ __forceinline__ float lane_fetch(float v, int byte_addr) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(byte_addr, __float_as_int(v)));
}
__device__ __forceinline__ double lane_fetch(double v, int byte_addr) {
  const int lo = __builtin_amdgcn_ds_bpermute(byte_addr, __double2loint(v));
  const int hi = __builtin_amdgcn_ds_bpermute(byte_addr, __double2hiint(v));
  return __hiloint2double(hi, lo);
}

// At: the pivot, full square, row stride LDA, in LDS (read only, and only before the first
// barrier).  Js: row stride LD, in LDS; receives J if anything rotated (else it is left as it
// was); it may share the memory of At.  Returns nonzero if any rotation was applied.  All 256
// threads of the workgroup must call it.
template <typename T>
__device__ int jacobi_cross_rounds(const T *At, float *Js, const int LDA, const int LD, T tol_rel, T tol_abs,
                                   JacCrossScratch<T> *cs) {
  constexpr int H = JAC_PIV / 2;
  const int tid = threadIdx.x, lane = tid & 63, l = lane & 31, q = 2 * (tid >> 6) + (lane >> 5);
  const int nxt = 4 * ((lane & 32) | ((lane + 1) & 31));     // byte address of the lane that holds l + 1
  T a[4], b[4], c[4], d[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int k = 4 * q + p;
    a[p] = At[k * LDA + l]; b[p] = At[k * LDA + H + l];
    c[p] = At[(H + k) * LDA + l]; d[p] = At[(H + k) * LDA + H + l];
  }
  // anything above the threshold among the pairs across the halves?  b holds all of them now.
  {
    const T dl = At[(H + l) * LDA + H + l];
    int todo = 0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int k = 4 * q + p;
      const T aa = jac_abs(b[p]);
      if (aa > tol_abs && aa * aa > tol_rel * tol_rel * jac_abs(At[k * LDA + k] * dl)) todo = 1;
    }
    if (tid == 0) { cs->todo = 0; cs->rotated = 0; }
    __syncthreads();
    if (todo) cs->todo = 1;
    __syncthreads();
    if (cs->todo == 0) return 0;
  }
  float x[8], y[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { x[e] = (8 * q + e == l) ? 1.f : 0.f; y[e] = (8 * q + e == H + l) ? 1.f : 0.f; }
  const bool owner = (l >> 2) == q;      // this thread holds block (l, l), as its block l % 4
  const int ps = l & 3;
  for (int r = 0; r < H; ++r) {
    if (owner) {
      const T app = ps == 0 ? a[0] : ps == 1 ? a[1] : ps == 2 ? a[2] : a[3];
      const T aqq = ps == 0 ? d[0] : ps == 1 ? d[1] : ps == 2 ? d[2] : d[3];
      const T apq = ps == 0 ? c[0] : ps == 1 ? c[1] : ps == 2 ? c[2] : c[3];
      T sn = 0, tp = 0;
      const T aa = jac_abs(apq);
      if (aa > tol_abs && aa * aa > tol_rel * tol_rel * jac_abs(app * aqq)) {
        // tan of the rotation angle: the smaller root of t^2 + 2 zeta t - 1 = 0, zeta = (a_qq - a_pp) / (2 a_pq)
        const T dd = aqq - app, hh = (T)2 * apq;
        const T xx = dd * dd + hh * hh;
        const T hyp = xx * rsqrt_newton(xx);
        const T t = hh * rcp_newton(dd + jac_copysign(hyp, dd));
        const T cc = rsqrt_newton((T)1 + t * t);
        sn = t * cc;
        tp = sn * rcp_newton((T)1 + cc);
        if (!(jac_abs(sn) <= (T)1)) { sn = 0; tp = 0; }   // non-finite: leave the pair alone
        if (sn != (T)0) cs->rotated = 1;
      }
      cs->st[l].s = sn; cs->st[l].t = tp;
    }
    __syncthreads();
    const JacPair<T> rl = cs->st[l];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const JacPair<T> rk = cs->st[4 * q + p];
      // rows: (a, c) and (b, d) are (x, y) pairs of rotation k
      const T a1 = a[p] - rk.s * (c[p] + rk.t * a[p]), c1 = c[p] + rk.s * (a[p] - rk.t * c[p]);
      const T b1 = b[p] - rk.s * (d[p] + rk.t * b[p]), d1 = d[p] + rk.s * (b[p] - rk.t * d[p]);
      // columns: (a1, b1) and (c1, d1) are (x, y) pairs of rotation l
      a[p] = a1 - rl.s * (b1 + rl.t * a1); b[p] = b1 + rl.s * (a1 - rl.t * b1);
      c[p] = c1 - rl.s * (d1 + rl.t * c1); d[p] = d1 + rl.s * (c1 - rl.t * d1);
      if (4 * q + p == l) { b[p] = (T)0; c[p] = (T)0; }   // the annihilated element
    }
    {
      const float sl = (float)rl.s, tl = (float)rl.t;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float xe = x[e], ye = y[e];
        x[e] = xe - sl * (ye + tl * xe);
        y[e] = ye + sl * (xe - tl * ye);
      }
    }
    // the second half moves on by one position
    cs->exc[q * 32 + l] = c[0]; cs->exd[q * 32 + l] = d[0];
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 4; ++p) b[p] = lane_fetch(b[p], nxt);
    c[0] = c[1]; c[1] = c[2]; c[2] = c[3]; c[3] = cs->exc[((q + 1) & 7) * 32 + l];
    {
      const T d1 = lane_fetch(d[1], nxt), d2 = lane_fetch(d[2], nxt), d3 = lane_fetch(d[3], nxt);
      d[0] = d1; d[1] = d2; d[2] = d3; d[3] = cs->exd[((q + 1) & 7) * 32 + ((l + 1) & 31)];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) y[e] = lane_fetch(y[e], nxt);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { Js[(8 * q + e) * LD + l] = x[e]; Js[(8 * q + e) * LD + H + l] = y[e]; }
  __syncthreads();
  return cs->rotated;
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
  float scale;           // the root is taken of scale * A (bias correction, Sec. 3.1.1); 1 = off
  const int32_t *only;   // optional [batch]: matrices whose entry is 0 are left alone (x untouched)
};

// NT threads per workgroup: 256 while several matrices fit the LDS of a CU (n <= 64); 1024
// above, where only one or two do and more wavefronts are the only way to hide LDS latency.
template <int NT>
__global__ __launch_bounds__(NT) void rootinv_small_kernel(const SmallRootArgs g) {
  if (g.only && g.only[blockIdx.x] == 0) return;   // the whole workgroup, before any barrier
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NW = NT / 64;
  __shared__ float redf[NW];
  __shared__ int redi[NW];
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
  for (int i = tid >> 6; i < s; i += NW)
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
  dmax = redf[0]; bad = redi[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) { dmax = fmaxf(dmax, redf[w]); bad |= redi[w]; }
  if (bad) {   // uniform: Sec. 3.2.3, keep the previous root
    if (tid == 0) {
      if (g.failed) g.failed[b] = 1;
      if (g.fail_count) atomicAdd(g.fail_count, 1ull);
    }
    return;
  }

  jacobi_sweeps<false, NT>(At, Js, s, LD, 0, JAC_SMALL_SWEEPS, JAC_SMALL_TOL_REL, JAC_SMALL_TOL_ABS * (double)dmax, sc);
  __syncthreads();

  // lambda_min over the true eigenvalues, then f = (lambda - min(lambda_min, 0) + eps)^-r
  double lmin = 1.0e300;
  for (int i = tid; i < n; i += NT) lmin = fmin(lmin, (double)g.scale * At[i * (i + 1) / 2 + i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) lmin = fmin(lmin, __shfl_xor(lmin, off, 64));
  __syncthreads();
  double *red = reinterpret_cast<double *>(sc->st);   // rotation scratch is free now
  if (lane == 0) red[wave] = lmin;
  __syncthreads();
  lmin = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) lmin = fmin(lmin, red[w]);
  const double shift = fmin(lmin, 0.0);
  int badf = 0;
  for (int i = tid; i < s; i += NT) {
    float f = 0.f;
    if (i < n) {
      const double lam = (double)g.scale * At[i * (i + 1) / 2 + i];
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
  badf = redi[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) badf |= redi[w];
  if (tid == 0 && g.failed) g.failed[b] = badf ? 1 : 0;
  if (badf) {
    if (tid == 0 && g.fail_count) atomicAdd(g.fail_count, 1ull);
    return;
  }
  // J <- J diag(sqrt f); X = J J^T, lower triangle computed and mirrored
  for (int i = tid >> 6; i < n; i += NW)
    for (int k = lane; k < s; k += 64) Js[i * LD + k] *= fv[k];
  __syncthreads();
  float *x = g.x + (int64_t)b * g.x_stride;
  for (int i = tid >> 6; i < n; i += NW)
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
//   J  [np/64][64][64] float32 rotation blocks of the current round, and the same
//      blocks transposed as two fp16 terms (for the update of Q^T on the fp16 matrix
//      cores); two rounds' worth, because the two rounds of a meeting of
//      super-columns are applied to Q^T together
// W is float64 for the same reason as in the LDS solver: the update
// A_kl <- J_k^T A_kl J_l runs on the float64 matrix cores (v_mfma_f64_16x16x4_f64),
// so eigenvalues far below 2^-24 lambda_max survive the ~400 updates of a solve.
// J is only orthogonal to float32 accuracy; applied as a congruence this moves
// every eigenvalue by a *relative* 1e-7 per round, which is harmless.
// ---------------------------------------------------------------------------
typedef double doublex4 __attribute__((ext_vector_type(4)));

// The float32 copy of W keeps every 32 x 32 sub-block contiguous (4 KB, sub-block (br, bc) at
// (br * nblk + bc) * 1024 floats, row-major inside): the updates read and write whole sub-blocks,
// and as 128-byte row pieces 4 KB apart they reach half the memory rate that 4 KB bursts do.
__device__ __forceinline__ int w32_sub(int br, int bc, int nblk) { return (br * nblk + bc) * (JAC_NB * JAC_NB); }
__device__ __forceinline__ int w32_index(int i, int j, int nblk) {
  return w32_sub(i / JAC_NB, j / JAC_NB, nblk) + (i % JAC_NB) * JAC_NB + (j % JAC_NB);
}

// 16 bytes of a matrix that is far larger than the caches and is not touched again before the
// next round: loaded as streaming data
typedef float jac_floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load4(const float *p) {
  const jac_floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const jac_floatx4 *>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}

// Workgroups are handed to the 8 XCDs (each with an L2 of its own) round-robin in launch order.
// The update kernels of the block solver re-number them so that every XCD works through whole
// matrices: the rotation blocks of a matrix (256 KB at n = 1024), which all of its workgroups
// read, then stay in one L2 instead of being fetched into all eight.  (bx, by): what the
// workgroup takes for blockIdx.x, blockIdx.y.
__device__ __forceinline__ void xcd_order(int &bx, int &by) {
  constexpr int XCDS = 8;
  const int nx = gridDim.x, total = nx * gridDim.y;
  const int lin = blockIdx.y * nx + blockIdx.x;
  const int xcd = lin % XCDS, pos = lin / XCDS;
  const int q = total / XCDS, r = total % XCDS;        // XCDs 0 .. r - 1 get q + 1 workgroups, the others q
  const int v = xcd * q + min(xcd, r) + pos;
  by = v / nx; bx = v - by * nx;
}

struct BlockJacArgs {
  double *w;
  float *w32;            // the float32 copy of W that the first sweeps of a cold solve work on (sub-blocks contiguous: w32_index)
  float *qt;
  float *jbuf;           // [batch][np/64][64][64]: rotation blocks of the current round
  int32_t *ident;        // [batch][np/64]: pivot of the current round needed no rotation
  int32_t *ident2;       // the flags of the second round of a meeting of two super-columns (group == 2; read by
                         // the two-round Q^T update only, which finds the first round's in ident)
  uint16_t *jt16;        // [batch][np/64][2][64][64] fp16: J^T of the current round as two fp16 terms of 2^13 J^T
  uint16_t *jt16_2;      // ... and of the second round of a meeting
  int32_t group;         // 1 or 2: see grouped_pair
  int32_t cross_only;    // the pivots rotate only pairs across their two block columns
  int32_t *rot;          // [batch][JAC_OUTER_SWEEPS]: pivots that rotated, per outer sweep
  const float *dmax;     // [batch]: largest |diagonal entry| of the input
  const float *wbound;   // [batch]: largest absolute row sum of the input (bounds every entry of every orthogonal transform of it)
  const int32_t *failed; // [batch]
  const int32_t *done;   // [batch]: the float32 sweeps were all this matrix needed (blockjac_f32_verdict_kernel)
  int32_t np;            // padded size
  int32_t round, sweep;
  int32_t phase_start;   // index of the first sweep of the current phase (float32 or float64 sweeps): a sweep is
                         // skipped when the one before it, in the same phase, rotated nothing
  int32_t inner_sweeps;  // Jacobi sweeps per pivot
  double tol_rel;        // rotation threshold relative to sqrt(|a_pp a_qq|)
  double tol_abs_rel;    // ... and absolute threshold as a fraction of max |diag(input)|
  __device__ __forceinline__ bool converged(int b) const {
    return done[b] != 0 || (sweep > phase_start && rot[b * JAC_OUTER_SWEEPS + sweep - 1] == 0);
  }
  // block columns (p < q) of pivot k of the current round
  __device__ __forceinline__ void pair(int k, int &p, int &q) const { grouped_pair(np / JAC_NB, group, round, k, p, q); }
};

struct BlockInitArgs {
  const float *a; int64_t a_stride; int32_t n;
  float *w;              // the float32 copy of W (sub-blocks contiguous: w32_index)
  float *qt; int32_t np;
  float *dmax; float *wbound; int32_t *failed; int32_t *rot;
  const int32_t *only;   // optional [batch]: a matrix whose entry is 0 is marked 2 in `failed`, which
                         // every later kernel takes as "leave alone" without counting it as a failure
  int32_t warm;          // nonzero: Qt holds the eigenvectors of an earlier solve and stays; W is made
                         // from it afterwards (congruence_f64.h); only the flags and bounds are set here
};

// W = pad(sym(A)), Qt = I (unless warm), dmax, wbound, failed, rot = 0.
// grid (np / 32, batch), 256 threads: a workgroup makes the 32 rows of one block row, sub-block by
// sub-block: the 32 x 32 tile of A at (br, bc) and the one at (bc, br) come in along their rows
// (128-byte pieces) and meet in LDS, so that A is read along rows only, and a sub-block of W goes
// out as the 4 KB it occupies.  Thread t holds row t / 8, columns 4 (t % 8) .. + 3 of a tile.
__global__ __launch_bounds__(256) void blockjac_init_kernel(const BlockInitArgs g) {
  __shared__ float Xs[JAC_NB][JAC_NB + 1], Ys[JAC_NB][JAC_NB + 1];
  const int b = blockIdx.y, br = blockIdx.x, np = g.np, n = g.n, nblk = np / JAC_NB;
  const int tid = threadIdx.x, r = tid >> 3, c4 = (tid & 7) * 4;
  const float *a = g.a + (int64_t)b * g.a_stride;
  if (g.only && g.only[b] == 0) {
    if (br == 0 && tid == 0) g.failed[b] = 2;
    return;
  }
  float *w = g.w + (int64_t)b * np * np;
  float *qt = g.qt + (int64_t)b * np * np;
  const int gi = br * JAC_NB + r;           // this thread's row of the matrix
  int bad = 0;
  float rowsum = 0.f, dm = 0.f;
  for (int bc = 0; bc < nblk; ++bc) {
    const int yi = bc * JAC_NB + r;         // its row of the tile on the other side of the diagonal
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int xj = bc * JAC_NB + c4 + e, yj = br * JAC_NB + c4 + e;
      const float x = (gi < n && xj < n) ? a[(int64_t)gi * n + xj] : 0.f;
      const float y = (yi < n && yj < n) ? a[(int64_t)yi * n + yj] : 0.f;
      if (!(fabsf(x) <= 3.0e38f) || !(fabsf(y) <= 3.0e38f)) bad = 1;
      Xs[r][c4 + e] = x;
      Ys[r][c4 + e] = y;
      if (gi == xj && fabsf(x) <= 3.0e38f) dm = fmaxf(dm, fabsf(x));
    }
    __syncthreads();
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = (float)(0.5 * ((double)Xs[r][c4 + e] + (double)Ys[c4 + e][r]));
      rowsum += fabsf(v[e]);
    }
    if (!g.warm) {
      *reinterpret_cast<float4 *>(w + w32_sub(br, bc, nblk) + r * JAC_NB + c4) = make_float4(v[0], v[1], v[2], v[3]);
      const int j0 = bc * JAC_NB + c4;
      *reinterpret_cast<float4 *>(qt + (int64_t)gi * np + j0) =
          make_float4(gi == j0 ? 1.f : 0.f, gi == j0 + 1 ? 1.f : 0.f, gi == j0 + 2 ? 1.f : 0.f, gi == j0 + 3 ? 1.f : 0.f);
    }
    __syncthreads();
  }
  if (bad) g.failed[b] = 1;
  // the row sum is spread over the 8 lanes of the row; the largest of a wavefront's 8 rows goes out
#pragma unroll
  for (int off = 1; off < 8; off <<= 1) rowsum += __shfl_xor(rowsum, off, 64);
  if (!(rowsum <= 3.0e38f)) rowsum = 0.f;
#pragma unroll
  for (int off = 8; off < 64; off <<= 1) {
    rowsum = fmaxf(rowsum, __shfl_xor(rowsum, off, 64));
    dm = fmaxf(dm, __shfl_xor(dm, off, 64));
  }
#pragma unroll
  for (int off = 1; off < 8; off <<= 1) dm = fmaxf(dm, __shfl_xor(dm, off, 64));
  if ((tid & 63) == 0) {     // both are >= 0: int order = float order
    atomicMax(reinterpret_cast<int *>(g.wbound + b), __float_as_int(rowsum));
    atomicMax(reinterpret_cast<int *>(g.dmax + b), __float_as_int(dm));
  }
  if (br == 0 && tid < JAC_OUTER_SWEEPS) g.rot[b * JAC_OUTER_SWEEPS + tid] = 0;
}

typedef _Float16 jac_f16x8 __attribute__((ext_vector_type(8)));
constexpr float JAC_F16_SCALE = 8192.f;                  // 2^13

__device__ __forceinline__ uint32_t pack_f16x2(_Float16 a, _Float16 b) {
  return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}
// the two fp16 terms of JAC_F16_SCALE * x
__device__ __forceinline__ void split_scaled(float x, _Float16 &h, _Float16 &l) {
  const float sx = x * JAC_F16_SCALE;
  h = (_Float16)sx;
  l = (_Float16)(sx - (float)h);
}

constexpr int PIV_LD = JAC_PIV + 1;

// Only the lower triangle of W is kept up to date, as 32 x 32 sub-blocks (a, b)
// with a >= b (the strictly-lower ones full, the diagonal ones symmetric): every
// sub-block is then read and written by exactly one workgroup per round, along
// its rows.  A sub-block needed "the other way round" is read transposed.

// One workgroup per (pair, matrix): diagonalise the 64 x 64 pivot.
// CROSS: only the pairs across the two block columns are rotated (g.cross_only must be set:
// every round but the first of a sweep when the block columns are grouped in twos).  That solver
// keeps the pivot and the rotations in registers: it reads the LDS copy of the pivot once, and J
// comes back into the same LDS array at the end, so the kernel needs half the LDS of the general
// one and twice as many workgroups (float64) fit a CU.
template <typename T, bool CROSS> struct PivotLds;
template <typename T> struct PivotLds<T, true> {
  T At[JAC_PIV * PIV_LD];
  JacCrossScratch<T> cs;
  __device__ float *js() { return reinterpret_cast<float *>(At); }
};
template <typename T> struct PivotLds<T, false> {
  T At[JAC_PIV * PIV_LD];
  float Js[JAC_PIV * PIV_LD];
  JacScratch sc;
  __device__ float *js() { return Js; }
};

template <typename T, bool CROSS>
__global__ __launch_bounds__(JAC_PIV_THREADS) void blockjac_pivot_kernel(const BlockJacArgs g) {
  __shared__ PivotLds<T, CROSS> lds;
  T *At = lds.At;
  float *Js = lds.js();
  const int b = blockIdx.y, pair = blockIdx.x;
  if (g.failed[b]) return;
  if (g.converged(b)) return;
  const int np = g.np, nblk = np / JAC_NB;
  int pb, qb;
  g.pair(pair, pb, qb);   // pb < qb
  const T *w = (sizeof(T) == 8 ? reinterpret_cast<const T *>(g.w) : reinterpret_cast<const T *>(g.w32)) + (int64_t)b * np * np;
  const int tid = threadIdx.x;
  // A float32 pivot is solved on a copy scaled by a power of two that brings the largest diagonal
  // entry of the matrix into [0.5, 1): the rotations do not depend on the scale, and products of
  // two entries (the rotation threshold, the rotation itself) neither underflow nor overflow
  // whatever the size of the gradients (factors of gradients of size 1e-15 have entries of 1e-31).
  T psc = (T)1;
  if (sizeof(T) == 4) {
    const float dmx = g.dmax[b];
    if (dmx > 0.f && dmx < 3.0e38f) {
      int e;
      (void)frexpf(dmx, &e);
      psc = (T)ldexpf(1.f, min(max(-e, -120), 120));
    }
  }
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_PIV_THREADS / 64) {
    const int j = tid & 63;
    const int gi = (i < JAC_NB ? pb * JAC_NB + i : qb * JAC_NB + i - JAC_NB);
    const int gj = (j < JAC_NB ? pb * JAC_NB + j : qb * JAC_NB + j - JAC_NB);
    // lower triangle of W (gi >= gj when j <= i, because pb < qb), mirrored into LDS
    const int lo_r = (j <= i) ? gi : gj, lo_c = (j <= i) ? gj : gi;
    const T v = sizeof(T) == 4 ? w[w32_index(lo_r, lo_c, nblk)] * psc : w[(int64_t)lo_r * np + lo_c];
    At[i * PIV_LD + j] = v;
    if (!CROSS) Js[i * PIV_LD + j] = (i == j) ? 1.f : 0.f;
  }
  __syncthreads();
  const double dm = (double)g.dmax[b] * (double)psc;
  static_assert(JAC_PIV_THREADS == 256 && JAC_PIV == 64, "thread layout of jacobi_cross_rounds");
  int any;
  if constexpr (CROSS) {
    any = jacobi_cross_rounds<T>(At, Js, PIV_LD, PIV_LD, (T)g.tol_rel, (T)(g.tol_abs_rel * dm), &lds.cs);
    if (!any) {        // Js (the memory of At) still holds the pivot: the identity goes out instead
      __syncthreads();
      for (int i = tid >> 6; i < JAC_PIV; i += JAC_PIV_THREADS / 64) Js[i * PIV_LD + (tid & 63)] = (i == (tid & 63)) ? 1.f : 0.f;
    }
  } else {
    any = jacobi_sweeps<true, JAC_PIV_THREADS, true, T>(At, Js, JAC_PIV, PIV_LD, PIV_LD, g.inner_sweeps,
                                                        (T)g.tol_rel, (T)(g.tol_abs_rel * dm), &lds.sc);
  }
  __syncthreads();
  if (tid == 0) {
    g.ident[b * (nblk / 2) + pair] = any ? 0 : 1;
    if (any) atomicAdd(&g.rot[b * JAC_OUTER_SWEEPS + g.sweep], 1);
  }
  // written even when nothing rotated (the identity): the W update then loads rotation blocks
  // unconditionally
  float *jout = g.jbuf + ((int64_t)b * (nblk / 2) + pair) * JAC_PIV * JAC_PIV;
  for (int i = tid >> 6; i < JAC_PIV; i += JAC_PIV_THREADS / 64) jout[i * JAC_PIV + (tid & 63)] = Js[i * PIV_LD + (tid & 63)];
  // ... and transposed, as the two fp16 terms of 2^13 J^T, for the update of Q^T on the fp16
  // matrix cores: thread -> row tid / 4 of J^T, 16 consecutive k
  static_assert(JAC_PIV_THREADS == 4 * JAC_PIV, "one row of J^T per four threads");
  {
    const int i = tid >> 2, k0 = (tid & 3) * 16;
    uint32_t hw[8], lw[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      _Float16 h0, l0, h1, l1;
      split_scaled(Js[(k0 + 2 * e) * PIV_LD + i], h0, l0);
      split_scaled(Js[(k0 + 2 * e + 1) * PIV_LD + i], h1, l1);
      hw[e] = pack_f16x2(h0, h1); lw[e] = pack_f16x2(l0, l1);
    }
    uint16_t *jt = g.jt16 + (((int64_t)b * (nblk / 2) + pair) * 2 * JAC_PIV + i) * JAC_PIV + k0;
    *reinterpret_cast<uint4 *>(jt) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
    *reinterpret_cast<uint4 *>(jt + 8) = make_uint4(hw[4], hw[5], hw[6], hw[7]);
    *reinterpret_cast<uint4 *>(jt + JAC_PIV * JAC_PIV) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
    *reinterpret_cast<uint4 *>(jt + JAC_PIV * JAC_PIV + 8) = make_uint4(lw[4], lw[5], lw[6], lw[7]);
  }
}

constexpr int APP_LD = JAC_PIV + 4;

// Loads rotation block `idx` of this matrix into LDS (identity if that pivot did not rotate).
__device__ __forceinline__ void load_rotation(float *dst, const float *jb, int idx, bool ident, int tid) {
  const int r = tid >> 4, c4 = (tid & 15) * 4;
#pragma unroll
  for (int h = 0; h < 4; ++h) {
    const int i = r + 16 * h;
    float4 v;
    if (ident) v = make_float4(i == c4 ? 1.f : 0.f, i == c4 + 1 ? 1.f : 0.f, i == c4 + 2 ? 1.f : 0.f, i == c4 + 3 ? 1.f : 0.f);
    else v = *reinterpret_cast<const float4 *>(jb + ((int64_t)idx * JAC_PIV + i) * JAC_PIV + c4);
    *reinterpret_cast<float4 *>(dst + i * APP_LD + c4) = v;
  }
}

// Copies one 32 x 32 sub-block between W and the LDS tile X (64 x 64, stride APP_LD).
// (ra, cb): block row / column of the quadrant as the product sees it; (xi, xj): its
// origin inside X.  The sub-block lives in W at (max, min); when ra < cb it is accessed
// transposed.  TO_LDS: W -> X, else X -> W.  Rows of W are always walked contiguously.
template <bool TO_LDS>
__device__ __forceinline__ void copy_subblock(double *w, int np, double *X, int ra, int cb, int xi, int xj, int tid) {
  const bool tr = ra < cb;
  const int gr0 = (tr ? cb : ra) * JAC_NB, gc0 = (tr ? ra : cb) * JAC_NB;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int idx = tid + JAC_THREADS * e;
    const int ii = idx >> 5, jj = idx & 31;          // position inside the stored sub-block
    double *gp = w + (int64_t)(gr0 + ii) * np + gc0 + jj;
    double *lp = tr ? &X[(xi + jj) * APP_LD + xj + ii] : &X[(xi + ii) * APP_LD + xj + jj];
    if (TO_LDS) *lp = *gp; else *gp = *lp;
  }
}

// One 32 x 32 sub-block of W on its way to / from the LDS tile X (64 x 64, stride APP_LD),
// split into a global -> register half and a register -> LDS half so that the global loads
// of the next pair-block can be in flight while the current one is multiplied.
// (ra, cb): block row / column of the quadrant as the product sees it; (xi, xj): its origin
// inside X.  The sub-block lives in W at (max, min); when ra < cb it is used transposed.
__device__ __forceinline__ void sub_fetch(const double *w, int np, int ra, int cb, int tid, double r[4]) {
  const bool tr = ra < cb;
  const int gr0 = (tr ? cb : ra) * JAC_NB, gc0 = (tr ? ra : cb) * JAC_NB;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int idx = tid + JAC_THREADS * e;
    r[e] = __builtin_nontemporal_load(w + (int64_t)(gr0 + (idx >> 5)) * np + gc0 + (idx & 31));
  }
}
__device__ __forceinline__ void sub_stash(double *X, int ra, int cb, int xi, int xj, int tid, const double r[4]) {
  const bool tr = ra < cb;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int idx = tid + JAC_THREADS * e;
    const int ii = idx >> 5, jj = idx & 31;
    if (tr) X[(xi + jj) * APP_LD + xj + ii] = r[e]; else X[(xi + ii) * APP_LD + xj + jj] = r[e];
  }
}

constexpr int APPW_SEG = 4;   // pair-blocks of one block row handled by one workgroup

// number of workgroups per matrix: row k of the lower triangle has k + 1 pair-blocks
inline int appw_segments(int hp, int seg = APPW_SEG) {
  int s = 0;
  for (int k = 0; k < hp; ++k) s += (k + 1 + seg - 1) / seg;
  return s;
}

constexpr int APP_JLD = JAC_PIV + 4;   // LDS row stride of J_l: rows 4 apart start 16 banks apart

// W_kl <- J_k^T W_kl J_l for the pair-blocks l <= k of one matrix, in float64 on the
// matrix cores.  grid (appw_segments(hp), batch): a workgroup walks up to APPW_SEG
// consecutive pair-blocks of block row k; while one pair-block is multiplied the W tile and
// the J_l of the next one are already on their way into registers, so the HBM latency is
// paid once per workgroup rather than once per pair-block.
//
// A 16x16x4 float64 MFMA takes A(i, k) from lane (i = lane % 16, k = lane / 16), B(k, j)
// likewise (j = lane % 16), and leaves D(lane / 16 + 4 v, lane % 16) in element v of the
// lane's result.  Wavefront w owns rows 16 w .. 16 w + 15 of the result and needs no exchange
// with the others between the two products:
//   first   T^T = X^T J_k, as four 16 x 16 tiles t over the columns kk of X, restricted to the
//           wavefront's 16 columns i of J_k (16 registers, loaded once per walk):
//           element v of tile t is T[16 w + lane % 16][16 t + g + 4 v], g = lane / 16;
//   second  C = T J_l: that element is, as it stands, the A operand of a k step that covers
//           the four values kk = 16 t + g + 4 v, g = 0 .. 3 (a sum may take its terms in any
//           order as long as both operands agree); B is J_l[16 t + g + 4 v][16 u + lane % 16],
//           read from LDS, where row 16 t + g + 4 v is kept at row 16 t + 4 g + v so that the
//           four rows of a read start 16 banks apart.
// The result leaves the registers straight for W: element v of tile u is
// C[16 w + g + 4 v][16 u + lane % 16], i.e. half a row of a stored sub-block per 16 lanes (where
// the sub-block is stored transposed: 32 consecutive bytes per 4 lanes).  Only the pair-block on
// the diagonal (k = l) goes back through LDS, where it is completed from its lower half so
// that the diagonal sub-blocks stay exactly symmetric.
constexpr int APPLY_LDS_BYTES = JAC_PIV * APP_LD * 12;    // what each of the three update bodies below needs

// bx: index of the workgroup among the appw_segments(hp) of the W update
__device__ __forceinline__ void blockjac_apply_w_body(const BlockJacArgs &g, int bx, int b, unsigned char *smem) {
  double *X = reinterpret_cast<double *>(smem);                               // [JAC_PIV * APP_LD] W_kl (and the result of a diagonal pair-block)
  float *Jl = reinterpret_cast<float *>(smem + JAC_PIV * APP_LD * 8);         // [JAC_PIV * APP_JLD]
  if (g.failed[b]) return;
  if (g.converged(b)) return;
  const int np = g.np, nblk = np / JAC_NB, hp = nblk / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t *ident = g.ident + b * hp;
  const float *jb = g.jbuf + (int64_t)b * hp * JAC_PIV * JAC_PIV;
  // segment -> (k, first l)
  int seg = bx, k = 0;
  for (;;) {
    const int ns = (k + 1 + APPW_SEG - 1) / APPW_SEG;
    if (seg < ns) break;
    seg -= ns; ++k;
  }
  const int l_first = seg * APPW_SEG, l_end = min(l_first + APPW_SEG, k + 1);
  const bool idk = ident[k] != 0;
  // the flags of the walk, read once (a load inside the walk would make every pair-block wait
  // for the stores of the one before it: the counter of outstanding memory operations is one)
  unsigned idbits = 0;
#pragma unroll
  for (int e = 0; e < APPW_SEG; ++e)
    if (l_first + e < l_end && ident[l_first + e] != 0) idbits |= 1u << e;
  // the pair-blocks of this walk that rotate at all, in order (uniform across the workgroup)
  auto next_active = [&](int from) {
    int l = from;
    while (l < l_end && idk && ((idbits >> (l - l_first)) & 1u)) ++l;
    return l;
  };
  int l = next_active(l_first);
  if (l >= l_end) return;
  double *w = g.w + (int64_t)b * np * np;
  int pk, qk;
  g.pair(k, pk, qk);

  const int li = lane & 15, lg = lane >> 4;
  float jk[16];                   // J_k[4 q + lg][16 wave + li]
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    const int row = 4 * q + lg, col = 16 * wave + li;
    jk[q] = jb[((int64_t)k * JAC_PIV + row) * JAC_PIV + col];
  }
  double wt[4][4];
  float4 jn0, jn1, jn2, jn3;
  const int jr = tid >> 4, jc4 = (tid & 15) * 4;
  auto fetch = [&](int lx) {
    int pl, ql;
    g.pair(lx, pl, ql);
    sub_fetch(w, np, pk, pl, tid, wt[0]);
    sub_fetch(w, np, pk, ql, tid, wt[1]);
    sub_fetch(w, np, qk, pl, tid, wt[2]);
    sub_fetch(w, np, qk, ql, tid, wt[3]);
    const float *js = jb + ((int64_t)lx * JAC_PIV + jr) * JAC_PIV + jc4;
    jn0 = *reinterpret_cast<const float4 *>(js);
    jn1 = *reinterpret_cast<const float4 *>(js + 16 * JAC_PIV);
    jn2 = *reinterpret_cast<const float4 *>(js + 32 * JAC_PIV);
    jn3 = *reinterpret_cast<const float4 *>(js + 48 * JAC_PIV);
  };
  fetch(l);
  for (bool first = true; l < l_end; first = false) {
    const int ln = next_active(l + 1);   // l_end if this is the last one
    int pl, ql;
    g.pair(l, pl, ql);
    if (!first) __syncthreads();   // every wavefront is done with X and J_l of the pair-block before
    sub_stash(X, pk, pl, 0, 0, tid, wt[0]);
    sub_stash(X, pk, ql, 0, JAC_NB, tid, wt[1]);
    sub_stash(X, qk, pl, JAC_NB, 0, tid, wt[2]);
    sub_stash(X, qk, ql, JAC_NB, JAC_NB, tid, wt[3]);
    {
      float *jd = &Jl[(4 * (jr & 3) + (jr >> 2)) * APP_JLD + jc4];   // row i of J_l is kept at row (i & ~15) + 4 (i & 3) + ((i & 15) >> 2)
      *reinterpret_cast<float4 *>(jd) = jn0;
      *reinterpret_cast<float4 *>(jd + 16 * APP_JLD) = jn1;
      *reinterpret_cast<float4 *>(jd + 32 * APP_JLD) = jn2;
      *reinterpret_cast<float4 *>(jd + 48 * APP_JLD) = jn3;
    }
    __syncthreads();
    if (ln < l_end) fetch(ln);     // in flight during the products below

    doublex4 t1[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) t1[t] = (doublex4){0.0, 0.0, 0.0, 0.0};
    // Operands of step q + 1 are read from LDS before the four MFMAs of step q (64 cycles
    // each) are issued; the scheduling barriers keep the compiler from hoisting every read of
    // the loop to its top, which costs a workgroup per CU in registers.
    double xq[2][4];
#pragma unroll
    for (int t = 0; t < 4; ++t) xq[0][t] = X[lg * APP_LD + li + 16 * t];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      if (q + 1 < 16) {
        const double *xr = &X[(4 * (q + 1) + lg) * APP_LD + li];
#pragma unroll
        for (int t = 0; t < 4; ++t) xq[(q + 1) & 1][t] = xr[16 * t];
      }
      float f = jk[q];
      asm volatile("" : "+v"(f));          // widened at the point of use, not held as float64 across the walk
      const double bq = (double)f;
#pragma unroll
      for (int t = 0; t < 4; ++t) t1[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(xq[q & 1][t], bq, t1[t], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (k == l) __syncthreads();   // all reads of X done: the result of a diagonal pair-block is completed there
    // The second product, two of its four 16-column tiles at a time; each tile leaves as soon
    // as it is done.  (All four at once: 1 % slower.  Without the prefetch the kernel fits three
    // workgroups per CU and is 6 % slower.)
    constexpr int UW = 2;
#pragma unroll
    for (int u0 = 0; u0 < 4; u0 += UW) {
      doublex4 c2[UW];
#pragma unroll
      for (int u = 0; u < UW; ++u) c2[u] = (doublex4){0.0, 0.0, 0.0, 0.0};
      float jq[2][UW];
#pragma unroll
      for (int u = 0; u < UW; ++u) jq[0][u] = Jl[(4 * lg) * APP_JLD + li + 16 * (u0 + u)];
#pragma unroll
      for (int s = 0; s < 16; ++s) {       // step s = 4 t + v: row 16 t + lg + 4 v of J_l, kept at row 16 t + 4 lg + v
        if (s + 1 < 16) {
          const float *jrow = &Jl[(16 * ((s + 1) >> 2) + 4 * lg + ((s + 1) & 3)) * APP_JLD + li];
#pragma unroll
          for (int u = 0; u < UW; ++u) jq[(s + 1) & 1][u] = jrow[16 * (u0 + u)];
        }
        const double av = t1[s >> 2][s & 3];
#pragma unroll
        for (int u = 0; u < UW; ++u) c2[u] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, (double)jq[s & 1][u], c2[u], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (k != l) {
        const int ra = wave < 2 ? pk : qk;
        const int ii0 = (16 * wave & 31) + lg;
#pragma unroll
        for (int uu = 0; uu < UW; ++uu) {
          const int u = u0 + uu;
          const int cb = u < 2 ? pl : ql;
          const int jj = (16 * u & 31) + li;
          if (ra > cb) {
#pragma unroll
            for (int v = 0; v < 4; ++v) __builtin_nontemporal_store(c2[uu][v], w + (int64_t)(ra * JAC_NB + ii0 + 4 * v) * np + cb * JAC_NB + jj);
          } else {        // stored transposed
#pragma unroll
            for (int v = 0; v < 4; ++v) __builtin_nontemporal_store(c2[uu][v], w + (int64_t)(cb * JAC_NB + jj) * np + ra * JAC_NB + ii0 + 4 * v);
          }
        }
      } else {
#pragma unroll
        for (int uu = 0; uu < UW; ++uu) {
          const int j = 16 * (u0 + uu) + li;
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int i = 16 * wave + lg + 4 * v;
            if (j <= i) { X[i * APP_LD + j] = c2[uu][v]; X[j * APP_LD + i] = c2[uu][v]; }
          }
        }
      }
    }
    if (k == l) {
      __syncthreads();
      copy_subblock<false>(w, np, X, pk, pl, 0, 0, tid);
      copy_subblock<false>(w, np, X, qk, pl, JAC_NB, 0, tid);   // (pk, qk) is its mirror image
      copy_subblock<false>(w, np, X, qk, ql, JAC_NB, JAC_NB, tid);
    }
    l = ln;
  }
}

__device__ __forceinline__ floatx16 mfma_64(const float *At, const float *B, int wi, int wj, int lane);

// The same update on the float32 copy of W (the first sweeps of a mixed-precision cold solve):
// W_kl <- J_k^T W_kl J_l on the fp16 matrix cores.  These sweeps only have to bring the
// off-diagonal mass down to float32 level; W is formed anew in float64 afterwards, so what the
// update needs is float32-like accuracy at fp16 speed: every operand is split into two fp16
// terms (x s = h + l up to 2^-24 |x s|; s = 2^13 for the rotation blocks, a power of two per
// matrix for W, from the largest absolute row sum of the input, which bounds every entry of
// every orthogonal transform of it) and a product is three matrix-core products,
// a_h b_h + a_h b_l + a_l b_h, accumulated in float32.  W itself stays float32 in memory.
//
// v_mfma_f32_16x16x32_f16 takes 8 consecutive k of row (column) lane % 16 per lane, k block
// lane / 16, for A (B), and leaves D[4 (lane / 16) + e][lane % 16] in element e.  Wavefront w
// owns rows 16 w .. 16 w + 15 of the result and needs no exchange with the others between the
// two products:
//   first   Y^T = X^T J_k as four 16 x 16 tiles a over the columns kk of X, for the wavefront's
//           16 columns i of J_k: A is X^T, staged in LDS as [kk][m] (both planes; a thread fills
//           it with 16-byte pieces from the 8 rows x 2 columns, or the 16 consecutive values
//           of a sub-block kept transposed, that it loaded), B is J_k^T[i][m] straight from
//           memory (jt16), held in registers for the whole walk.  Element e of tile a is
//           Y^T[16 a + 4 g + e][16 w + lane % 16], g = lane / 16;
//   second  C = Y J_l: those elements are, once split again, the A operand of a k step that
//           covers kk = 16 a + 4 g + e for a = 2 t, 2 t + 1 (a sum may take its terms in any
//           order as long as both operands agree); B is J_l^T[j][kk] for the same kk, two 8-byte
//           reads from the LDS copy of jt16 of pair l.
// The result leaves the registers straight for W; only the pair-block on the diagonal (k = l)
// goes back through LDS, where it is completed from its lower half so that the diagonal
// sub-blocks stay exactly symmetric.  Same grid and walk as blockjac_apply_w_kernel.
typedef _Float16 jac_f16x8v __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int W16_XROW = JAC_PIV * 2 + 16;        // bytes of one row of X^T in LDS (64 values of m + padding)
constexpr int W16_XPLANE = JAC_PIV * W16_XROW;
constexpr int W16_JROW = JAC_PIV * 2 + 8;         // bytes of one row of J_l^T in LDS
constexpr int W16_JPLANE = JAC_PIV * W16_JROW;
constexpr int W16_LDS_BYTES = 2 * W16_XPLANE + 2 * W16_JPLANE;
constexpr int W16_SEG = 4;                       // pair-blocks of one block row handled by one workgroup (8: 2 % slower)
static_assert(2 * W16_XPLANE >= JAC_PIV * APP_LD * 4, "the float32 tile of a diagonal pair-block reuses the X^T planes");

// The power of two s with s * bound in [2^13, 2^14) (1 for a bound that is zero or not finite).
__device__ __forceinline__ float jac_pow2_scale(float bound) {
  if (!(bound > 0.f) || !(bound < 3.0e38f)) return 1.f;
  int e;
  (void)frexpf(bound, &e);               // bound = f 2^e with f in [0.5, 1)
  return ldexpf(1.f, min(max(14 - e, -100), 100));
}

__device__ __forceinline__ void blockjac_apply_w32_body(const BlockJacArgs &g, int bx, int b, unsigned char *smem) {
  unsigned char *XT = smem;                              // [2 planes][64 kk][W16_XROW]
  unsigned char *JL = smem + 2 * W16_XPLANE;             // [2 planes][64 j][W16_JROW]
  float *Ct = reinterpret_cast<float *>(smem);           // [64][APP_LD], diagonal pair-block only
  if (g.failed[b]) return;
  if (g.converged(b)) return;
  const int np = g.np, nblk = np / JAC_NB, hp = nblk / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int32_t *ident = g.ident + b * hp;
  const uint16_t *jt = g.jt16 + (int64_t)b * hp * 2 * JAC_PIV * JAC_PIV;
  int seg = bx, k = 0;
  for (;;) {
    const int ns = (k + 1 + W16_SEG - 1) / W16_SEG;
    if (seg < ns) break;
    seg -= ns; ++k;
  }
  const int l_first = seg * W16_SEG, l_end = min(l_first + W16_SEG, k + 1);
  const bool idk = ident[k] != 0;
  // the flags of the walk, read once (a load inside the walk would make every pair-block wait
  // for the stores of the one before it: the counter of outstanding memory operations is one)
  unsigned idbits = 0;
#pragma unroll
  for (int e = 0; e < W16_SEG; ++e)
    if (l_first + e < l_end && ident[l_first + e] != 0) idbits |= 1u << e;
  auto next_active = [&](int from) {
    int l = from;
    while (l < l_end && idk && ((idbits >> (l - l_first)) & 1u)) ++l;
    return l;
  };
  int l = next_active(l_first);
  if (l >= l_end) return;
  float *w = g.w32 + (int64_t)b * np * np;
  int pk, qk;
  g.pair(k, pk, qk);
  const float sw = jac_pow2_scale(g.wbound[b]);
  const float unscale = 1.f / (sw * JAC_F16_SCALE);

  // B operands of the first product: J_k^T rows 16 wave + li, m = 32 step + 8 lg .. + 7, both planes
  uint4 jk[2][2];                 // [plane][step]
#pragma unroll
  for (int pl = 0; pl < 2; ++pl)
#pragma unroll
    for (int st = 0; st < 2; ++st)
      jk[pl][st] = *reinterpret_cast<const uint4 *>(jt + ((int64_t)(2 * k + pl) * JAC_PIV + 16 * wave + li) * JAC_PIV + 32 * st + 8 * lg);

  // The next pair-block on its way: 16 values of W per thread and 64 bytes of jt16 of pair l.
  // Sub-block sb = tid / 64 of the tile: (row block, column block) = (pk, pl), (pk, ql), (qk, pl), (qk, ql).
  const int sb = tid >> 6, t6 = tid & 63;
  float wa[8], wb[8];
  uint4 jn0, jn1, jn2, jn3;
  auto fetch = [&](int lx) {
    int pl, ql;
    g.pair(lx, pl, ql);
    const int ra = (sb & 2) ? qk : pk, cb = (sb & 1) ? ql : pl;
    if (ra >= cb) {      // kept as it is: rows m = 8 (t6 / 16) .. + 7, columns 2 (t6 % 16), + 1
      const float *src = w + w32_sub(ra, cb, nblk) + 8 * (t6 >> 4) * JAC_NB + 2 * (t6 & 15);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float2 v = *reinterpret_cast<const float2 *>(src + e * JAC_NB);
        wa[e] = v.x; wb[e] = v.y;
      }
    } else {             // kept transposed: its row kk = t6 / 2, 16 consecutive m
      const float *src = w + w32_sub(cb, ra, nblk) + (t6 >> 1) * JAC_NB + 16 * (t6 & 1);
      const float4 v0 = stream_load4(src), v1 = stream_load4(src + 4), v2 = stream_load4(src + 8), v3 = stream_load4(src + 12);
      wa[0] = v0.x; wa[1] = v0.y; wa[2] = v0.z; wa[3] = v0.w; wa[4] = v1.x; wa[5] = v1.y; wa[6] = v1.z; wa[7] = v1.w;
      wb[0] = v2.x; wb[1] = v2.y; wb[2] = v2.z; wb[3] = v2.w; wb[4] = v3.x; wb[5] = v3.y; wb[6] = v3.z; wb[7] = v3.w;
    }
    // jt16 of pair lx: 2 planes x 64 rows x 128 bytes = 1024 pieces of 16 bytes, 4 per thread
    const uint4 *js = reinterpret_cast<const uint4 *>(jt + (int64_t)(2 * lx) * JAC_PIV * JAC_PIV);
    jn0 = js[tid]; jn1 = js[tid + 256]; jn2 = js[tid + 512]; jn3 = js[tid + 768];
  };
  auto pack8 = [&](const float (&x)[8], unsigned char *dst) {     // the two terms of 8 values, 16 bytes per plane
    _Float16 h[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float sx = x[e] * sw;
      h[e] = (_Float16)sx;
      lo[e] = (_Float16)(sx - (float)h[e]);
    }
    *reinterpret_cast<uint4 *>(dst) = make_uint4(pack_f16x2(h[0], h[1]), pack_f16x2(h[2], h[3]), pack_f16x2(h[4], h[5]), pack_f16x2(h[6], h[7]));
    *reinterpret_cast<uint4 *>(dst + W16_XPLANE) = make_uint4(pack_f16x2(lo[0], lo[1]), pack_f16x2(lo[2], lo[3]), pack_f16x2(lo[4], lo[5]), pack_f16x2(lo[6], lo[7]));
  };
  auto stash = [&](int lx) {
    int pl, ql;
    g.pair(lx, pl, ql);
    const int ra = (sb & 2) ? qk : pk, cb = (sb & 1) ? ql : pl;
    const int m0 = (sb & 2) ? JAC_NB : 0, kk0 = (sb & 1) ? JAC_NB : 0;     // origin of the sub-block inside the tile
    if (ra >= cb) {
      const int mg = t6 >> 4, c2 = 2 * (t6 & 15);
      pack8(wa, XT + (kk0 + c2) * W16_XROW + (m0 + 8 * mg) * 2);
      pack8(wb, XT + (kk0 + c2 + 1) * W16_XROW + (m0 + 8 * mg) * 2);
    } else {
      const int kk = t6 >> 1, mh = 16 * (t6 & 1);
      pack8(wa, XT + (kk0 + kk) * W16_XROW + (m0 + mh) * 2);
      pack8(wb, XT + (kk0 + kk) * W16_XROW + (m0 + mh + 8) * 2);
    }
    // piece tid + 256 e: plane = e / 2, row = tid / 8 + 32 (e % 2), 16-byte column = tid % 8
    unsigned char *jd = JL + (tid >> 3) * W16_JROW + (tid & 7) * 16;
    *reinterpret_cast<uint4 *>(jd) = jn0;
    *reinterpret_cast<uint4 *>(jd + 32 * W16_JROW) = jn1;
    *reinterpret_cast<uint4 *>(jd + W16_JPLANE) = jn2;
    *reinterpret_cast<uint4 *>(jd + W16_JPLANE + 32 * W16_JROW) = jn3;
  };
  fetch(l);
  for (bool first = true; l < l_end; first = false) {
    const int ln = next_active(l + 1);   // l_end if this is the last one
    int pl, ql;
    g.pair(l, pl, ql);
    if (!first) __syncthreads();         // every wavefront is done with the tile of the pair-block before
    stash(l);
    __syncthreads();
    if (ln < l_end) fetch(ln);           // in flight during the products below

    // first product: four tiles of Y^T, 2 k steps x 3 products each
    floatx4 yt[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      yt[a] = (floatx4){0.f, 0.f, 0.f, 0.f};
      const unsigned char *xr = XT + (16 * a + li) * W16_XROW + 16 * lg;
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        const jac_f16x8v xh = __builtin_bit_cast(jac_f16x8v, *reinterpret_cast<const uint4 *>(xr + 64 * st));
        const jac_f16x8v xl = __builtin_bit_cast(jac_f16x8v, *reinterpret_cast<const uint4 *>(xr + 64 * st + W16_XPLANE));
        const jac_f16x8v jh = __builtin_bit_cast(jac_f16x8v, jk[0][st]), jl = __builtin_bit_cast(jac_f16x8v, jk[1][st]);
        yt[a] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xl, jh, yt[a], 0, 0, 0);
        yt[a] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xh, jl, yt[a], 0, 0, 0);
        yt[a] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xh, jh, yt[a], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the A operands of the second product: k step t takes tiles 2 t and 2 t + 1
    jac_f16x8v ah[2], al[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      _Float16 h[8], lo[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float sx = yt[2 * t + (e >> 2)][e & 3] * unscale * sw;
        h[e] = (_Float16)sx;
        lo[e] = (_Float16)(sx - (float)h[e]);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) { ah[t][e] = h[e]; al[t][e] = lo[e]; }
    }
    if (k == l) __syncthreads();         // all reads of X^T done: the result of a diagonal pair-block is completed there
    // second product, one 16-column tile of the result at a time; each leaves as soon as it is done
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      floatx4 c = (floatx4){0.f, 0.f, 0.f, 0.f};
      const unsigned char *jr = JL + (16 * u + li) * W16_JROW + 8 * lg;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint2 h0 = *reinterpret_cast<const uint2 *>(jr + 64 * t), h1 = *reinterpret_cast<const uint2 *>(jr + 64 * t + 32);
        const uint2 l0 = *reinterpret_cast<const uint2 *>(jr + 64 * t + W16_JPLANE), l1 = *reinterpret_cast<const uint2 *>(jr + 64 * t + 32 + W16_JPLANE);
        const jac_f16x8v bh = __builtin_bit_cast(jac_f16x8v, make_uint4(h0.x, h0.y, h1.x, h1.y));
        const jac_f16x8v bl = __builtin_bit_cast(jac_f16x8v, make_uint4(l0.x, l0.y, l1.x, l1.y));
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(al[t], bh, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[t], bl, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah[t], bh, c, 0, 0, 0);
      }
      // element e is C[16 wave + 4 lg + e][16 u + li]
      if (k != l) {
        const int ra = wave < 2 ? pk : qk, cb = u < 2 ? pl : ql;
        const int ii0 = (16 * wave & 31) + 4 * lg, jj = (16 * u & 31) + li;
        if (ra > cb) {
#pragma unroll
          for (int e = 0; e < 4; ++e) __builtin_nontemporal_store(c[e] * unscale, w + w32_sub(ra, cb, nblk) + (ii0 + e) * JAC_NB + jj);
        } else {          // kept transposed: four consecutive values per lane
          __builtin_nontemporal_store(c * unscale, reinterpret_cast<floatx4 *>(w + w32_sub(cb, ra, nblk) + jj * JAC_NB + ii0));
        }
      } else {
        const int j = 16 * u + li;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 16 * wave + 4 * lg + e;
          if (j <= i) { Ct[i * APP_LD + j] = c[e] * unscale; Ct[j * APP_LD + i] = c[e] * unscale; }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (k == l) {
      __syncthreads();
      // thread -> row tid / 8 of a stored sub-block, 4 columns
      const int ii = tid >> 3, j4 = (tid & 7) * 4;
      auto sub_store = [&](int ra, int cb, int xi, int xj) {   // ra >= cb: kept as it is
        *reinterpret_cast<float4 *>(w + w32_sub(ra, cb, nblk) + ii * JAC_NB + j4) =
            *reinterpret_cast<const float4 *>(&Ct[(xi + ii) * APP_LD + xj + j4]);
      };
      sub_store(pk, pl, 0, 0);
      sub_store(qk, pl, JAC_NB, 0);                      // (pk, qk) is its mirror image and is not kept
      sub_store(qk, ql, JAC_NB, JAC_NB);
    }
    l = ln;
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

constexpr int APPQ_TILES = 4;   // 64-column tiles of Qt handled by one workgroup

// Qt rows of pair k <- J_k^T (those rows), APPQ_TILES 64-column tiles per workgroup,
// float32 MFMA.  grid (hp * ceil(np / 256), batch).
// bx: index of the workgroup among the hp * ceil(np / 256) of the Q update
__device__ __forceinline__ void blockjac_apply_q_body(const BlockJacArgs &g, int bx, int b, unsigned char *smem) {
  float *Jk = reinterpret_cast<float *>(smem);           // [JAC_PIV * APP_LD]
  float (*X)[JAC_PIV * APP_LD] = reinterpret_cast<float (*)[JAC_PIV * APP_LD]>(Jk + JAC_PIV * APP_LD);   // [2][...]
  if (g.failed[b]) return;
  if (g.converged(b)) return;
  const int np = g.np, nblk = np / JAC_NB, hp = nblk / 2, ctiles = np / JAC_PIV;
  const int groups = (ctiles + APPQ_TILES - 1) / APPQ_TILES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int k = bx / groups, grp = bx - k * groups;
  if (g.ident[b * hp + k]) return;
  float *qt = g.qt + (int64_t)b * np * np;
  int pk, qk;
  g.pair(k, pk, qk);
  const int r = tid >> 4, c4 = (tid & 15) * 4;
  const int t0 = grp * APPQ_TILES, t1 = min(t0 + APPQ_TILES, ctiles);
  float4 pre0, pre1, pre2, pre3;
  // thread (r, c4) moves rows r, r+16, r+32, r+48 of the 64-row strip, 4 columns each
  const float *src0 = qt + (int64_t)(pk * JAC_NB + r) * np + c4;
  const float *src1 = qt + (int64_t)(pk * JAC_NB + r + 16) * np + c4;
  const float *src2 = qt + (int64_t)(qk * JAC_NB + r) * np + c4;
  const float *src3 = qt + (int64_t)(qk * JAC_NB + r + 16) * np + c4;
#define APPQ_FETCH(ct)                                                        \
  pre0 = *reinterpret_cast<const float4 *>(src0 + (ct) * JAC_PIV);            \
  pre1 = *reinterpret_cast<const float4 *>(src1 + (ct) * JAC_PIV);            \
  pre2 = *reinterpret_cast<const float4 *>(src2 + (ct) * JAC_PIV);            \
  pre3 = *reinterpret_cast<const float4 *>(src3 + (ct) * JAC_PIV)
#define APPQ_STASH(dst)                                                       \
  *reinterpret_cast<float4 *>((dst) + (r) * APP_LD + c4) = pre0;              \
  *reinterpret_cast<float4 *>((dst) + (r + 16) * APP_LD + c4) = pre1;         \
  *reinterpret_cast<float4 *>((dst) + (r + 32) * APP_LD + c4) = pre2;         \
  *reinterpret_cast<float4 *>((dst) + (r + 48) * APP_LD + c4) = pre3
  APPQ_FETCH(t0);
  load_rotation(Jk, g.jbuf + (int64_t)b * hp * JAC_PIV * JAC_PIV, k, false, tid);
  APPQ_STASH(X[0]);
  __syncthreads();
  for (int t = t0; t < t1; ++t) {
    const int cur = (t - t0) & 1;
    if (t + 1 < t1) { APPQ_FETCH(t + 1); }
    const floatx16 acc = mfma_64(Jk, X[cur], wi, wj, lane);
    const int gc = t * JAC_PIV + wj * 32 + (lane & 31);
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = wi * 32 + 8 * q + 4 * (lane >> 5) + e;
        const int grow = (i < JAC_NB ? pk * JAC_NB + i : qk * JAC_NB + i - JAC_NB);
        qt[(int64_t)grow * np + gc] = acc[4 * q + e];
      }
    if (t + 1 < t1) { APPQ_STASH(X[cur ^ 1]); }
    __syncthreads();
  }
#undef APPQ_FETCH
#undef APPQ_STASH
}

// The Q^T update of both rounds of a meeting of two super-columns (group == 2) in one pass:
// the 128 rows of the four block columns a < b < c < d involved take J(a, c), J(b, d) of the
// first round and then J(a, d), J(b, c) of the second, and are read and written once.
//
// On the float32 matrix cores the update of one round already takes as long as its memory
// traffic, so one pass for two rounds would gain nothing there.  The products therefore run on
// the fp16 matrix cores with each float32 operand split into two fp16 terms (x 2^13 = h + l up
// to 2^-22 |x|: both operands are bounded by 1, rows and columns of orthogonal matrices) and
// three products per result, J_h X_h + J_h X_l + J_l X_h, accumulated in float32: 3 / 16 of the
// float32 matrix-core time, at an error of 2^-22 per update instead of 2^-24.  Q^T itself stays
// float32 in memory; the rotation blocks arrive split (jt16, written by the pivots).
//
// g.round is the first of the two rounds; g.jt16 / g.ident belong to it, g.jt16_2 / g.ident2 to
// the second.  256 threads: wavefront (piv, wi) takes pivot piv of each round and produces the
// 32 rows of its first (wi = 0) or second (wi = 1) block column, 64 columns wide.
// v_mfma_f32_32x32x16_f16 takes 8 consecutive k of row lane % 32 per lane, k block lane / 32, for
// both operands, and leaves D[8 q + 4 (lane / 32) + e][lane % 32] in element 4 q + e.  The rotation
// blocks are the A operands, straight from memory into registers (jt16 is J^T, k contiguous); the
// tile of Q^T is the B operand and is staged in LDS column by column ([column][row], both
// planes), which a thread fills from the 8 rows x 4 columns it loaded.  Between the rounds the
// accumulators go back to LDS the same way (a lane holds 4 consecutive rows of one column).
// APPQ_TILES tiles of 64 columns per workgroup, the next one on its way into registers
// meanwhile.  grid ((np / 128) * ceil(np / 256), batch).
constexpr int APPQ2_THREADS = 256;
constexpr int APPQ2_ROW = 2 * JAC_PIV * 2 + 16;          // bytes of one column of the staged tile: 128 rows + padding
constexpr int APPQ2_PLANE = JAC_PIV * APPQ2_ROW;         // one plane: 64 columns

__global__ __launch_bounds__(APPQ2_THREADS, 2) void blockjac_apply_q2_kernel(const BlockJacArgs g) {
  __shared__ __align__(16) unsigned char Xs[2 * APPQ2_PLANE];   // plane h, plane l
  int bxo, b;
  xcd_order(bxo, b);
  if (g.failed[b]) return;
  if (g.converged(b)) return;
  const int np = g.np, nblk = np / JAC_NB, hp = nblk / 2, ctiles = np / JAC_PIV;
  const int groups = (ctiles + APPQ_TILES - 1) / APPQ_TILES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int piv = wave >> 1, wi = wave & 1;
  const int K = bxo / groups, grp = bxo - K * groups;
  const bool ida0 = g.ident[b * hp + 2 * K] != 0, idb0 = g.ident[b * hp + 2 * K + 1] != 0;
  const bool ida1 = g.ident2[b * hp + 2 * K] != 0, idb1 = g.ident2[b * hp + 2 * K + 1] != 0;
  if (ida0 && idb0 && ida1 && idb1) return;
  const bool id0 = piv ? idb0 : ida0, id1 = piv ? idb1 : ida1;    // this wavefront's pivot, first and second round
  float *qt = g.qt + (int64_t)b * np * np;
  int blk_a, blk_c;               // a, c; b = a + 1, d = c + 1
  grouped_pair(nblk, 2, g.round, 2 * K, blk_a, blk_c);
  // Blocks of the staged tile: 0 = a, 1 = b, 2 = c, 3 = d.  The first round pairs block piv with
  // 2 + piv, the second with 3 - piv; this wavefront produces block out0 in the first round and
  // out1 in the second.
  const int xq0 = 2 + piv, xq1 = 3 - piv;
  const int out0 = wi ? xq0 : piv, out1 = wi ? xq1 : piv;
  // the pivot of the second round that block out0 belongs to: a, d -> 0; b, c -> 1
  const bool out0_final = (out0 == 0 || out0 == 3) ? ida1 : idb1;   // nobody touches it again: this wavefront stores it
  // A operands: J^T rows 32 wi + lane % 32, k = 16 s + 8 (lane / 32) .. + 7, both planes, both rounds
  uint4 ja[2][2][4];              // [round][plane][k step]
  {
    const int row = 32 * wi + (lane & 31), kb = lane >> 5;
    const uint16_t *j0 = g.jt16 + ((int64_t)b * hp + 2 * K + piv) * 2 * JAC_PIV * JAC_PIV + row * JAC_PIV + 8 * kb;
    const uint16_t *j1 = g.jt16_2 + ((int64_t)b * hp + 2 * K + piv) * 2 * JAC_PIV * JAC_PIV + row * JAC_PIV + 8 * kb;
#pragma unroll
    for (int pl = 0; pl < 2; ++pl)
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        ja[0][pl][st] = *reinterpret_cast<const uint4 *>(j0 + pl * JAC_PIV * JAC_PIV + 16 * st);
        ja[1][pl][st] = *reinterpret_cast<const uint4 *>(j1 + pl * JAC_PIV * JAC_PIV + 16 * st);
      }
  }
  // thread -> rows 8 rg .. 8 rg + 7 of the 128, columns c4 .. c4 + 3 of the tile
  const int rg = tid >> 4, c4 = (tid & 15) * 4;
  const int t0 = grp * APPQ_TILES, t1 = min(t0 + APPQ_TILES, ctiles);
  // offsets inside one matrix fit 32 bits (np <= 16384), which keeps addresses at one register each
  const int src = (((rg >> 2) < 2 ? blk_a + (rg >> 2) : blk_c + (rg >> 2) - 2) * JAC_NB + 8 * (rg & 3)) * np + c4;
  float4 pre[8];
  auto fetch = [&](int ct) {
#pragma unroll
    for (int e = 0; e < 8; ++e) pre[e] = stream_load4(qt + (src + e * np + ct * JAC_PIV));
  };
  auto stage = [&]() {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      _Float16 h[8], l[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = c == 0 ? pre[e].x : c == 1 ? pre[e].y : c == 2 ? pre[e].z : pre[e].w;
        split_scaled(x, h[e], l[e]);
      }
      unsigned char *dst = Xs + (c4 + c) * APPQ2_ROW + 16 * rg;
      *reinterpret_cast<uint4 *>(dst) = make_uint4(pack_f16x2(h[0], h[1]), pack_f16x2(h[2], h[3]), pack_f16x2(h[4], h[5]), pack_f16x2(h[6], h[7]));
      *reinterpret_cast<uint4 *>(dst + APPQ2_PLANE) = make_uint4(pack_f16x2(l[0], l[1]), pack_f16x2(l[2], l[3]), pack_f16x2(l[4], l[5]), pack_f16x2(l[6], l[7]));
    }
  };
  // one round of this wavefront's pivot: acc[wj] = J^T (rows of blocks xp, xq), 32 rows x 2 x 32 columns
  auto rotate = [&](const uint4 (&a)[2][4], int xq, floatx16 (&acc)[2]) {
#pragma unroll
    for (int wj = 0; wj < 2; ++wj) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[wj][v] = 0.f;
      const unsigned char *col = Xs + (32 * wj + (lane & 31)) * APPQ2_ROW + 16 * (lane >> 5);
#pragma unroll
      for (int st = 0; st < 4; ++st) {
        const unsigned char *p = col + (st < 2 ? piv : xq) * (JAC_NB * 2) + (st & 1) * 32;
        const jac_f16x8 xh = __builtin_bit_cast(jac_f16x8, *reinterpret_cast<const uint4 *>(p));
        const jac_f16x8 xl = __builtin_bit_cast(jac_f16x8, *reinterpret_cast<const uint4 *>(p + APPQ2_PLANE));
        const jac_f16x8 jh = __builtin_bit_cast(jac_f16x8, a[0][st]), jl = __builtin_bit_cast(jac_f16x8, a[1][st]);
        acc[wj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(jl, xh, acc[wj], 0, 0, 0);
        acc[wj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(jh, xl, acc[wj], 0, 0, 0);
        acc[wj] = __builtin_amdgcn_mfma_f32_32x32x16_f16(jh, xh, acc[wj], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);     // or every operand read of the round is hoisted to its top, which costs a workgroup per CU in registers
      }
    }
  };
  constexpr float UNSCALE = 1.f / (JAC_F16_SCALE * JAC_F16_SCALE);
  // rows of block `blk` (0 .. 3) of the tile at columns ct: the accumulators, unscaled, to Q^T
  auto store = [&](const floatx16 (&acc)[2], int blk, int ct) {
    int dst = ((blk < 2 ? blk_a + blk : blk_c + blk - 2) * JAC_NB + 4 * (lane >> 5)) * np + ct * JAC_PIV + (lane & 31);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        __builtin_nontemporal_store(acc[0][4 * q + e] * UNSCALE, qt + dst);
        __builtin_nontemporal_store(acc[1][4 * q + e] * UNSCALE, qt + dst + 32);
        dst += np;
      }
      dst += 4 * np;
    }
  };
  fetch(t0);
  for (int t = t0; t < t1; ++t) {
    stage();
    __syncthreads();
    if (t + 1 < t1) fetch(t + 1);
    floatx16 acc[2];
    if (!id0) rotate(ja[0], xq0, acc);
    __syncthreads();               // every wavefront has read what it needs of the tile
    if (!id0) {
      if (out0_final) store(acc, out0, t);
      else {
        // back into the tile for the second round: element 4 q + e is row 8 q + 4 (lane / 32) + e
#pragma unroll
        for (int wj = 0; wj < 2; ++wj) {
          unsigned char *dst = Xs + (32 * wj + (lane & 31)) * APPQ2_ROW + (out0 * JAC_NB + 4 * (lane >> 5)) * 2;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            _Float16 h[4], l[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) split_scaled(acc[wj][4 * q + e] * UNSCALE, h[e], l[e]);
            *reinterpret_cast<uint2 *>(dst + 16 * q) = make_uint2(pack_f16x2(h[0], h[1]), pack_f16x2(h[2], h[3]));
            *reinterpret_cast<uint2 *>(dst + 16 * q + APPQ2_PLANE) = make_uint2(pack_f16x2(l[0], l[1]), pack_f16x2(l[2], l[3]));
          }
        }
      }
    }
    __syncthreads();
    if (!id1) {
      rotate(ja[1], xq1, acc);
      store(acc, out1, t);
    }
    __syncthreads();               // the tile is free for the next one
  }
}

// The three updates as kernels of their own (one launch for W and Q^T together measured 3 %
// slower: the two bodies then share one register allocation and one occupancy limit).
__global__ __launch_bounds__(JAC_THREADS, 2) void blockjac_apply_w_kernel(const BlockJacArgs g) {
  __shared__ __align__(32) unsigned char smem[APPLY_LDS_BYTES];
  int bx, b;
  xcd_order(bx, b);
  blockjac_apply_w_body(g, bx, b, smem);
}
__global__ __launch_bounds__(JAC_THREADS, 3) void blockjac_apply_w32_kernel(const BlockJacArgs g) {
  __shared__ __align__(32) unsigned char smem[W16_LDS_BYTES];
  int bx, b;
  xcd_order(bx, b);
  blockjac_apply_w32_body(g, bx, b, smem);
}
__global__ __launch_bounds__(JAC_THREADS, 2) void blockjac_apply_q_kernel(const BlockJacArgs g) {
  __shared__ __align__(32) unsigned char smem[APPLY_LDS_BYTES];
  int bx, b;
  xcd_order(bx, b);
  blockjac_apply_q_body(g, bx, b, smem);
}

// After the float32 sweeps: does this matrix need the float64 phase at all?
// What converged float32 sweeps leave behind is an absolute error of about 1e-7 of the largest
// eigenvalue, in the eigenvalues and in the off-diagonal elements alike.  For a well-conditioned
// matrix that is a relative 1e-6 of every eigenvalue, and the congruence plus the float64 sweeps
// (a quarter of such a solve: their first sweep finds every pivot above the float64 threshold
// and costs more than a float32 one) would change nothing that can be seen in the result.
// Two tests on the float32 W = D + E (D its diagonal, lo and hi the smallest and largest entry
// of D):
//   lo >= JAC_F32_ONLY_RATIO * hi                      the spectrum is narrow, and
//   ||E||_F <= JAC_F32_ONLY_OFF * sqrt(n) * lo         the sweeps did converge.
// The second bounds what stopping here costs: to first order f(D + E) - f(D) has the entries
// E_ij (f(d_i) - f(d_j)) / (d_i - d_j), at most |f'| |E_ij| = |E_ij| f / (4 lo) for
// f = lambda^(-1/4), so the relative error of the root in the Frobenius norm is at most
// ||E||_F / (4 sqrt(n) lo) <= JAC_F32_ONLY_OFF / 4.
// A matrix that passes gets done[b] = 1 (every later kernel of the solve returns at once for it)
// and its diagonal copied to d32 (an array of its own: the float64 W of one matrix lies over the
// float32 copies of two others, which their workgroups may not have read yet), where the last
// kernel of the solve looks for the eigenvalues; skip[b] = failed[b] | done[b] is what the
// congruence takes.  One workgroup of 256 threads per matrix.
constexpr float JAC_F32_ONLY_RATIO = 0.1f;
constexpr float JAC_F32_ONLY_OFF = 6.0e-5f;

struct BlockVerdictArgs {
  float *d32;            // [batch][np]
  const float *w32; int32_t np, n;
  const int32_t *failed; int32_t *done; int32_t *skip;
};

__global__ __launch_bounds__(256) void blockjac_f32_verdict_kernel(const BlockVerdictArgs g) {
  __shared__ float redlo[4], redhi[4];
  __shared__ double redss[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int np = g.np, n = g.n, nblk = np / JAC_NB;
  if (g.failed[b]) {
    if (tid == 0) { g.done[b] = 0; g.skip[b] = 1; }
    return;
  }
  const float *w32 = g.w32 + (int64_t)b * np * np;
  float *d32 = g.d32 + (int64_t)b * np;
  float lo = 3.0e38f, hi = -3.0e38f;
  for (int i = tid; i < np; i += 256) {
    const float d = w32[w32_index(i, i, nblk)];
    d32[i] = d;
    if (i < n) { lo = fminf(lo, d); hi = fmaxf(hi, d); }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { lo = fminf(lo, __shfl_xor(lo, off, 64)); hi = fmaxf(hi, __shfl_xor(hi, off, 64)); }
  if (lane == 0) { redlo[wave] = lo; redhi[wave] = hi; }
  __syncthreads();
  lo = fminf(fminf(redlo[0], redlo[1]), fminf(redlo[2], redlo[3]));
  hi = fmaxf(fmaxf(redhi[0], redhi[1]), fmaxf(redhi[2], redhi[3]));
  bool ok = lo > 0.f && hi < 3.0e38f && lo >= JAC_F32_ONLY_RATIO * hi;     // uniform over the workgroup
  if (ok) {
    // ||E||_F^2 / hi^2: the sub-blocks below the diagonal count twice, those on it hold both halves.
    // The elements are scaled by a power of two near 1 / hi first (their squares would leave the
    // float32 range for factors of very small or very large gradients).
    const float sc = jac_pow2_scale(hi);
    double ss = 0.0;
    for (int br = 0; br < nblk; ++br)
      for (int bc = 0; bc <= br; ++bc) {
        const float *sub = w32 + w32_sub(br, bc, nblk);
        float acc = 0.f;
        for (int e = tid; e < JAC_NB * JAC_NB / 4; e += 256) {
          const float4 q = stream_load4(sub + 4 * e);
          float v[4] = {q.x, q.y, q.z, q.w};
          if (br == bc) {           // element 4 e + c is (row, col) = (e / 8, 4 (e % 8) + c)
            const int row = e >> 3, col0 = 4 * (e & 7);
#pragma unroll
            for (int c = 0; c < 4; ++c) if (col0 + c == row) v[c] = 0.f;
          }
#pragma unroll
          for (int c = 0; c < 4; ++c) { v[c] *= sc; acc += v[c] * v[c]; }
        }
        ss += (double)acc * (br == bc ? 1.0 : 2.0);
      }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if (lane == 0) redss[wave] = ss;
    __syncthreads();
    ss = redss[0] + redss[1] + redss[2] + redss[3];
    const double bound = (double)JAC_F32_ONLY_OFF * (double)(lo * sc);
    ok = ss <= bound * bound * (double)n;
  }
  if (tid == 0) { g.done[b] = ok ? 1 : 0; g.skip[b] = ok ? 1 : 0; }
}

struct BlockFinalArgs {
  const double *w; const float *qt; int32_t np; int32_t n;
  float epsilon, r;
  float scale;           // the root is taken of scale * A; 1 = off
  float *fvals;          // [batch][np]: lambda'^-r / ||q||^2 (0 on padding)
  float *lambda;         // optional [batch][n]
  int32_t *failed;       // [batch] in/out
  int32_t *failed_out;   // optional user-visible copy
  unsigned long long *fail_count;
  const int32_t *rot;    // [batch][JAC_OUTER_SWEEPS] pivots that rotated per sweep
  int32_t *sweeps_out;   // optional [batch]: number of sweeps in which anything rotated
  const int32_t *done;   // optional [batch]: nonzero = the eigenvalues are in d32, not on the diagonal of w
  const float *d32;      // [batch][np]
};

// fvals[i] <- ||row i of Qt||^2 for the n eigenvectors of every matrix that has not failed.
// grid (ceil(n / 4), batch), 256 threads: one wavefront per row.
struct BlockRowNormArgs {
  const float *qt; float *fvals; const int32_t *failed; int32_t np, n;
};
__global__ __launch_bounds__(256) void blockjac_rownorm_kernel(const BlockRowNormArgs g) {
  const int b = blockIdx.y, lane = threadIdx.x & 63, i = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (g.failed[b] || i >= g.n) return;
  const float *row = g.qt + (int64_t)b * g.np * g.np + (int64_t)i * g.np;
  double ss = 0.0;
  for (int j = 4 * lane; j < g.np; j += 256) {
    const float4 v = stream_load4(row + j);
    ss += (double)v.x * (double)v.x + (double)v.y * (double)v.y + (double)v.z * (double)v.z + (double)v.w * (double)v.w;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if (lane == 0) g.fvals[(int64_t)b * g.np + i] = (float)ss;
}

// One workgroup per matrix: eigenvalues, shift, f(lambda); fvals holds the squared row norms of Qt
// on entry (blockjac_rownorm_kernel).
// The rotation blocks are orthogonal to float32 accuracy only, so after a few
// hundred rounds the accumulated columns q_i have drifted off unit length by ~1e-5
// (and the diagonal of W, q_i^T A q_i, with them).  Both are put right here: the
// eigenvalue is the Rayleigh quotient W_ii / ||q_i||^2 and the weight handed to the
// reconstruction sum_i f_i q_i q_i^T is f_i / ||q_i||^2.
__global__ __launch_bounds__(256) void blockjac_final_kernel(const BlockFinalArgs g) {
  __shared__ double redf[4];
  __shared__ int redi[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int np = g.np, n = g.n;
  const double *w = g.w + (int64_t)b * np * np;
  float *fv = g.fvals + (int64_t)b * np;
  const int bad = g.failed[b];
  const float *d32 = (g.done && g.done[b]) ? g.d32 + (int64_t)b * np : nullptr;
  auto diag = [&](int i) { return d32 ? (double)d32[i] : w[(int64_t)i * np + i]; };
  // fv[i] holds ||row i of Qt||^2 (blockjac_rownorm_kernel)
  double lmin = 1.0e300;
  if (!bad)
    for (int i = tid; i < n; i += 256) lmin = fmin(lmin, (double)g.scale * diag(i) / (double)fv[i]);
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
      const double nrm2 = (double)fv[i];
      const double lam = (double)g.scale * diag(i) / nrm2;
      f = (float)(pow(lam - shift + (double)g.epsilon, -(double)g.r) / nrm2);
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
  if (tid == 0 && g.sweeps_out && bad != 2) {
    int cnt = 0;
    for (int sw = 0; sw < JAC_OUTER_SWEEPS; ++sw) cnt += g.rot[b * JAC_OUTER_SWEEPS + sw] != 0;
    g.sweeps_out[b] = cnt;
  }
  if (tid == 0 && bad != 2) {   // 2: not this call's matrix (see BlockInitArgs::only)
    g.failed[b] = badf;
    if (g.failed_out) g.failed_out[b] = badf;
    if (badf && g.fail_count) atomicAdd(g.fail_count, 1ull);
  }
}

}  // namespace shampoo
