/*
 * shampoo.h -- C ABI of the MI355X (gfx950) per-block Shampoo optimizer step.
 *
 * The library computes, entirely in hand-written HIP kernels, the optimizer
 * step of Shi et al., "A Distributed Data-Parallel PyTorch Implementation of
 * the Distributed Shampoo Optimizer for Training Neural Networks At-Scale"
 * (arXiv 2309.06497), restricted to one GPU: blocked Kronecker-factor
 * accumulation (matrices, and tensors of order one, three and four after merging
 * of small dimensions), periodic inverse-root refresh by batched symmetric
 * eigendecomposition (or the coupled inverse Newton iteration), preconditioning
 * by the roots, AdaGrad / SGD / RMSprop / Adam grafting, gradient filtering,
 * bias correction, weight decay, (Nesterov) momentum and the parameter update.
 * The multi-GPU distribution of the paper (Sec. 4.1) is not part of this library.
 *
 * Conventions for every entry point
 *   - "device pointer": memory of the GPU the optimizer was created on,
 *     owned by the caller and never freed by the library.
 *   - "host pointer": ordinary process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it; calls return without waiting unless stated.
 *   - Return value: 0 on success, negative error code otherwise (see
 *     shampoo_strerror).  Argument errors (every code except SHAMPOO_ERR_HIP)
 *     are detected before any work is enqueued: nothing has been modified.
 *   - No entry point throws; none is safe to call concurrently on the same
 *     shampoo_opt from several threads.
 */
#ifndef SHAMPOO_H
#define SHAMPOO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct shampoo_opt shampoo_opt; /* opaque, owned by the library */

enum {
  SHAMPOO_OK = 0,
  SHAMPOO_ERR_NULL = -1,      /* a required pointer is NULL                      */
  SHAMPOO_ERR_SHAPE = -2,     /* bad n_params / ndim / shape / block_size / index */
  SHAMPOO_ERR_HYPER = -3,     /* hyper-parameter out of range                     */
  SHAMPOO_ERR_WORKSPACE = -4, /* workspace NULL, misaligned or too small          */
  SHAMPOO_ERR_STEP = -5,      /* step not strictly increasing                     */
  SHAMPOO_ERR_HIP = -6,       /* a HIP runtime call failed                        */
  SHAMPOO_ERR_UNSUPPORTED = -7 /* size outside what the kernels support           */
};

enum { SHAMPOO_GRAD_F32 = 0, SHAMPOO_GRAD_BF16 = 1 };
enum { SHAMPOO_GRAFT_ADAGRAD = 0, SHAMPOO_GRAFT_SGD = 1, SHAMPOO_GRAFT_RMSPROP = 2, SHAMPOO_GRAFT_ADAM = 3 };
enum { SHAMPOO_ROOT_EIGH = 0, SHAMPOO_ROOT_NEWTON = 1 };
enum { SHAMPOO_MATRIX_CORES_AUTO = 0, SHAMPOO_MATRIX_CORES_FP32 = 1 };
enum { SHAMPOO_LARGE_DIM_BLOCKING = 0, SHAMPOO_LARGE_DIM_ADAGRAD = 1, SHAMPOO_LARGE_DIM_DIAGONAL = 2 };
#define SHAMPOO_MAX_NDIM 4

/*
 * Optimizer configuration (copied at create; the arrays need not outlive the call).
 * Hyper-parameters are those of the paper's complete pseudocode (Sec. 3,
 * "Complete Distributed Shampoo Pseudocode").
 */
typedef struct {
  int32_t n_params;       /* number of parameters (tensors), >= 1                          */
  const int32_t *ndim;    /* host [n_params]: 1 (diagonal AdaGrad path, Sec. 4.2.2), 2, 3 or 4.
                             A parameter of 3 or 4 dimensions first has its small dimensions
                             merged (Sec. 4.2.1: from the left, a dimension joins the current
                             group while the product stays <= block_size, a dimension of size 1
                             always; only a view, no data moves).  Two dimensions left: the matrix case on the merged shape.
                             Three or four left, or one (all merged): Shampoo for a tensor of that
                             order w (Sec. 2.3), one factor per dimension, root exponent
                             2 * root_exponent / w, blocks of at most block_size per dimension
                             (a block of more than 2^30 elements: SHAMPOO_ERR_UNSUPPORTED)   */
  const int64_t *shape;   /* host [SHAMPOO_MAX_NDIM * n_params]: the ndim[i] dimensions of
                             parameter i, slowest first, at shape[SHAMPOO_MAX_NDIM * i ...];
                             the remaining entries are ignored                               */
  int32_t block_size;     /* b: max_preconditioner_dim of Sec. 4.2.1, >= 1                  */
  float beta2;            /* in (0,1]; 1 = plain sum of G G^T, < 1 = EMA (Sec. 3.1.1)       */
  float epsilon;          /* > 0: added to the eigenvalues in the root inverse (Sec. 3.2.1) */
  float root_exponent;    /* r > 0: factors are raised to the power -r (0.25 for matrices)  */
  int32_t precondition_frequency;     /* f >= 1: roots refreshed when step % f == 0 (Sec. 4.3) */
  int32_t start_preconditioning_step; /* >= 0: before it the grafted direction is used alone   */
  float graft_epsilon;    /* >= 0: P_graft = G / (sqrt(A) + graft_epsilon) (Sec. 2.4)        */
  float momentum;         /* mu in [0,1): 0 disables the momentum state (Sec. 3.1.3)         */
  float beta1;            /* in [0,1): > 0 filters the gradient, Gf <- beta1 Gf + (1-beta1) G;
                             grafting state and factors use G, directions use Gf (Sec. 3.1.1) */
  float weight_decay;     /* >= 0 (Sec. 3.1.2)                                               */
  int32_t use_decoupled_weight_decay; /* != 0: P <- P - wd W after grafting; 0: G <- G + wd W  */
  int32_t use_nesterov;   /* != 0: W += lr (mu M + P) instead of lr M (Sec. 3.1.3)            */
  int32_t grafting_type;  /* SHAMPOO_GRAFT_ADAGRAD (A <- A + G.^2), SHAMPOO_GRAFT_SGD (P_graft = G, no
                             state), SHAMPOO_GRAFT_RMSPROP / _ADAM (A <- beta_g A + (1-beta_g) G.^2;
                             Adam divides A by 1 - beta_g^(step+1) when bias correction is on).
                             1-D parameters run that diagonal method itself (AdaGrad under SGD) */
  float grafting_beta2;   /* beta_g in (0,1] of RMSprop / Adam grafting; ignored otherwise   */
  int32_t use_bias_correction; /* != 0: directions use Gf / (1 - beta1^(step+1)) and roots are
                             taken of L / (1 - beta2^(step+1)) (beta2 < 1), epsilon added after
                             the division; stored state stays uncorrected (Sec. 3.1.1)        */
  int32_t large_dim_method; /* what happens to a 2-D parameter with a dimension above block_size (Sec. 4.2):
                             SHAMPOO_LARGE_DIM_BLOCKING (default): cut into blocks (Sec. 4.2.1);
                             SHAMPOO_LARGE_DIM_ADAGRAD: the diagonal method on its entries, as for a
                             1-D parameter (Sec. 4.2.2);
                             SHAMPOO_LARGE_DIM_DIAGONAL: kept whole, the factor of each such
                             dimension replaced by its diagonal (Sec. 4.2.3).
                             Tensors of order 1, 3 or 4 (after merging) are always blocked;
                             more than 65535 whole parameters or tensor blocks of one shape:
                             SHAMPOO_ERR_UNSUPPORTED                                          */
  int32_t root_method;    /* SHAMPOO_ROOT_EIGH: eigendecomposition (framed box of Sec. 3.2.1, default);
                             SHAMPOO_ROOT_NEWTON: coupled inverse Newton iteration of the same
                             section on L + epsilon I, in float32; needs 1/root_exponent in
                             {1, 2, 4, 8} (else SHAMPOO_ERR_UNSUPPORTED; for a tensor parameter
                             the exponent in question is 2 * root_exponent / w).  A factor whose
                             iterates do not stay finite (condition number beyond float32) is
                             handed to the eigendecomposition instead (the guard of Sec. 3.2.3);
                             to learn whether any did, a refresh step under this method waits
                             for `stream` once per batch of factors                          */
  float newton_tolerance; /* stop when ||M_k - I||_inf < this; 0 selects 1e-6 (Sec. 3.2.1)     */
  int32_t newton_max_iterations; /* iteration cap, <= 1000; 0 selects 100                     */
  int32_t precond_matrix_cores; /* SHAMPOO_MATRIX_CORES_AUTO (default): with bf16 gradients and blocks
                             whose shape and alignment allow it, Lbar G Rbar runs on the fp16 matrix
                             cores from float32 operands split into two fp16 planes each, scaled
                             per block by a power of two (three exact products accumulated in
                             float32: float32 accuracy at 3/16 of the float32-MFMA time; elements
                             below 2^-16 of a block's largest keep absolute, not relative,
                             accuracy); SHAMPOO_MATRIX_CORES_FP32: always the float32 MFMA          */
  int32_t warm_start_roots; /* != 0: the eigendecomposition of a refresh starts from the eigenvectors of
                             the previous one (Sec. 3.2.1, 4.3: between refreshes a factor changes
                             little) instead of from the identity: W = Q^T L Q is formed (float64
                             sums) and the Jacobi sweeps begin there.  Factors of dimension <= 128 (solved
                             inside one workgroup) and the coupled Newton iteration ignore it.  Costs
                             one more float32 matrix per factor in the workspace.  Every 16th refresh
                             starts cold, which bounds the drift of the accumulated float32
                             eigenvectors away from orthogonality.  0 (default): every refresh cold */
  int32_t grad_dtype;     /* SHAMPOO_GRAD_F32 or SHAMPOO_GRAD_BF16; parameters are float32   */
  int32_t device;         /* HIP device ordinal                                              */
} shampoo_config;

/*
 * Block planner (host only, touches no GPU).  Sec. 4.2.1: a rows x cols
 * parameter is cut into ceil(rows/b) x ceil(cols/b) blocks, all b x b except
 * in the last block row / column.  Blocks of equal (m, n) form a bucket and
 * are numbered (slot) in parameter order, row-major inside a parameter.
 * Writes up to `cap` rows of 12 int64
 * {param, row0, col0, m, n, bucket, slot, flags, s3, d3, s4, d4}
 * into `table` (host, may be NULL when cap == 0) and the total number of
 * blocks / buckets into *n_blocks / *n_buckets (host, may be NULL).
 * A block of a tensor parameter (flags bit 2, and the order 1, 3 or 4 of the merged tensor
 * in flags bits 4..6) starts at (row0, col0, s3, s4) of the merged
 * shape and measures m x n x d3 x d4 (sizes 1 for the dimensions it does not have); matrix
 * blocks have s3 = s4 = 0, d3 = d4 = 1.  Tensor blocks are numbered in row-major order of
 * their block indices.
 * Under SHAMPOO_LARGE_DIM_DIAGONAL a parameter with a dimension above b is one row
 * (m, n = its shape) with flags bit 0 / bit 1 set where the left / right factor is
 * diagonal; under SHAMPOO_LARGE_DIM_ADAGRAD such a parameter has no row (it is handled
 * like a 1-D parameter).
 */
int shampoo_plan(const shampoo_config *cfg, int64_t *table, int64_t cap,
                 int64_t *n_blocks, int64_t *n_buckets);

/* Bytes of device workspace shampoo_create needs for cfg; 0 if cfg is invalid. */
size_t shampoo_workspace_bytes(const shampoo_config *cfg);

/*
 * Create an optimizer.  `workspace` is a device pointer, 256-byte aligned, of
 * at least shampoo_workspace_bytes(cfg) bytes; it holds all optimizer state
 * (factors L, R, roots, grafting state A, momentum M) and scratch, and must
 * stay allocated until shampoo_destroy.  State is initialised (L = R = 0,
 * roots = I, A = M = 0) on `stream`, which is synchronised before returning.
 * *out (host) receives the handle.
 */
int shampoo_create(const shampoo_config *cfg, void *workspace, size_t workspace_bytes,
                   void *stream, shampoo_opt **out);

/*
 * One optimizer iteration t = `step` (0-based, strictly increasing between
 * calls) of the complete pseudocode for every block of every parameter:
 *   G <- G + wd W   (l2 weight decay only)               (Sec. 3.1.2)
 *   L <- beta2 L + (1-beta2) G G^T, R likewise          (Sec. 3.1.1)
 *   A <- A + G.^2   (AdaGrad grafting; EMA for RMSprop / Adam)   (Sec. 2.4, 2.2)
 *   if step >= start and step % f == 0: roots refreshed  (Sec. 3.2.1 box, 4.3)
 *   Gf <- beta1 Gf + (1-beta1) G  (Gf = G when beta1 = 0) (Sec. 3.1.1)
 *       (with bias correction the lines below read Gf / (1 - beta1^(step+1)))
 *   P_graft = Gf/(sqrt(A)+eps_g)  or  Gf (SGD grafting)
 *   P = -||P_graft||_F * Lbar Gf Rbar / ||Lbar Gf Rbar||_F           (Sec. 2.4)
 *       (P = -P_graft while step < start; 1-D parameters: -Gf/(sqrt(A)+eps_g))
 *   P <- P - wd W   (decoupled weight decay only)        (Sec. 3.1.2)
 *   M <- mu M + P ; W <- W + lr M  (Nesterov: lr (mu M + P))          (Sec. 3.1.3)
 * A block of a tensor parameter has one factor per dimension k,
 *   L_k <- beta2 L_k + (1-beta2) G_(k) G_(k)^T  (G_(k): mode-k unfolding),
 * and P_shampoo = G x_1 Lbar_1 x_2 Lbar_2 ... x_w Lbar_w (mode products, Sec. 2.3); the
 * other lines apply unchanged.
 * params: host array [n_params] of device pointers, float32, contiguous
 *         row-major with the shapes given at create; updated in place.
 * grads:  host array [n_params] of device pointers, float32 or bfloat16 per
 *         grad_dtype, same shapes; read only.
 * Asynchronous on `stream` (except refresh steps under SHAMPOO_ROOT_NEWTON, see
 * root_method, and a call that follows a change of the params / grads pointers, which first
 * waits for `stream`: the tables it sends replace those an earlier call may still be copying).
 * With bf16 gradients the factor update of the first steps, while a factor has summed fewer than
 * four times as many gradient columns as it has rows, adds up in float64 (the later ones in the
 * float32 accumulators of the matrix cores): a root taken from such a young factor weights its
 * smallest eigenvalues most.  If a launch fails (SHAMPOO_ERR_HIP) the state is partly updated
 * and `step` does not count as taken.  A factor whose eigendecomposition is not finite keeps its
 * previous root (Sec. 3.2.3); such events are counted, see shampoo_status.
 */
int shampoo_step(shampoo_opt *opt, void *const *params, const void *const *grads,
                 float lr, int64_t step, void *stream);

/* State selectors for shampoo_get. */
enum {
  SHAMPOO_GET_L = 0,      /* m x m float32 (m floats, the diagonal, where that factor is diagonal) */
  SHAMPOO_GET_R = 1,      /* n x n (n)       */
  SHAMPOO_GET_LINV = 2,   /* m x m (m)       */
  SHAMPOO_GET_RINV = 3,   /* n x n (n)       */
  SHAMPOO_GET_A = 4,      /* m x n (block) or len (1-D parameter, block = 0) */
  SHAMPOO_GET_M = 5,      /* same shape as A; error if momentum == 0         */
  SHAMPOO_GET_PSH = 6,    /* m x n: last Lbar G Rbar                         */
  SHAMPOO_GET_NORMS = 7,  /* 2 floats: ||P_graft||_F^2, ||P_shampoo||_F^2 of the last step */
  SHAMPOO_GET_GF = 8,     /* same shape as A: filtered gradient; error if beta1 == 0       */
  SHAMPOO_GET_L2 = 9,     /* tensor blocks of order 3 or 4: the factor of the second dimension, n x n */
  SHAMPOO_GET_L2INV = 10, /* and its root                                                    */
  SHAMPOO_GET_L3 = 11,    /* tensor blocks of order 4: the factor of the third dimension, d3 x d3 */
  SHAMPOO_GET_L3INV = 12  /* and its root                                                    */
};
/* For a block m x n x d3 (x d4) of a tensor parameter: L / LINV belong to the first dimension
 * (m x m), R / RINV to the last one, L2 / L2INV and L3 / L3INV to those between; A, M, PSH,
 * GF are the dense block. */

/*
 * Copy one piece of state of block `block` (row-major index inside parameter
 * `param`) into dst (device pointer, dense row-major float32, `bytes` must
 * equal the size listed above).  Asynchronous on `stream`.
 */
int shampoo_get(shampoo_opt *opt, int32_t param, int32_t block, int32_t which,
                void *dst, size_t bytes, void *stream);

/*
 * Synchronises `stream` and reports (host pointers, each may be NULL):
 * the number of root refreshes performed, and the total number of factors
 * whose refresh was skipped because the factor or its spectrum was not finite.
 */
int shampoo_status(shampoo_opt *opt, void *stream, int64_t *n_refreshes,
                   int64_t *n_failed_roots);

/* Per-stage device timing (HIP events on the step's stream). */
enum {
  SHAMPOO_STAGE_FACTOR = 0,   /* both symmetric rank-k factor updates       */
  SHAMPOO_STAGE_GRAFT = 1,    /* grafting state + graft norm                */
  SHAMPOO_STAGE_ROOT = 2,     /* root-inverse refresh                       */
  SHAMPOO_STAGE_PRECOND = 3,  /* T = Lbar G (diagonal Shampoo: the whole Lbar G Rbar) */
  SHAMPOO_STAGE_UPDATE = 4,   /* rescale + momentum + parameter update      */
  SHAMPOO_STAGE_DIAG = 5,     /* 1-D parameters                             */
  SHAMPOO_STAGE_FUSED = 6,    /* blocks <= 128 x 128 on steps without refresh: factor update,
                                 grafting, preconditioning and update in one kernel */
  SHAMPOO_STAGE_PRECOND2 = 7, /* P = T Rbar, with the sums of squares of P  */
  SHAMPOO_STAGE_COUNT = 8
};
/* enable != 0: later steps record events around each stage (small overhead). */
int shampoo_set_timing(shampoo_opt *opt, int32_t enable);
/*
 * Synchronises the recorded events and returns, for `stage`, the summed
 * milliseconds and the number of timed intervals since the last call for that
 * stage (host pointers).  Resets that stage's record.
 */
int shampoo_get_timing(shampoo_opt *opt, int32_t stage, double *ms_total, int64_t *intervals);

/* Frees the host-side handle only (the workspace belongs to the caller). */
int shampoo_destroy(shampoo_opt *opt);

/*
 * Stand-alone batched root inverse (the framed box of Sec. 3.2.1):
 *   lambda, Q = eigh(A_i);  lambda' = lambda - min(lambda_min, 0) + epsilon;
 *   X_i = Q diag(lambda'^(-r)) Q^T               for i = 0 .. batch-1.
 * a:      device, batch dense row-major symmetric n x n float32 matrices (read only)
 * x:      device, batch n x n float32 outputs (may not alias a)
 * lambda: device, batch x n float32 eigenvalues in the solver's order
 *         (unsorted), or NULL
 * workspace: device, 256-byte aligned, at least
 *         shampoo_root_inverse_workspace_bytes(n, batch) bytes
 * failed: device int32[batch] set to 1 where A_i or its spectrum is not
 *         finite (X_i is then left untouched), else 0; or NULL
 * Asynchronous on `stream`.
 */
size_t shampoo_root_inverse_workspace_bytes(int32_t n, int32_t batch);
int shampoo_root_inverse(const float *a, int32_t n, int32_t batch, float epsilon, float r,
                         float *x, float *lambda, int32_t *failed,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * shampoo_root_inverse with a warm start (n > 128 only, else SHAMPOO_ERR_UNSUPPORTED): the
 * eigenvectors are kept in the caller's array qt between calls.
 * qt:     device, batch x np x np float32, np = n rounded up to a multiple of 64, aligned to 16
 *         bytes (else SHAMPOO_ERR_WORKSPACE); rows are eigenvectors.  start == 0: a cold solve (qt is overwritten).  start != 0: qt holds the
 *         result of an earlier call on matrices close to a (the same factors some steps
 *         earlier): the solve starts from W = qt a qt^T (float64 sums), and qt is updated.
 *         A matrix that fails (see `failed`) leaves its part of qt as it was.
 * sweeps: device int32[batch] or NULL: the number of Jacobi sweeps in which anything rotated
 *         (the last one of a solve never does: it finds every pair below the threshold).
 * Everything else as shampoo_root_inverse; the workspace is larger by the float64 panel.
 */
size_t shampoo_root_inverse_warm_workspace_bytes(int32_t n, int32_t batch);
int shampoo_root_inverse_warm(const float *a, int32_t n, int32_t batch, float epsilon, float r,
                              float *x, float *lambda, int32_t *failed, float *qt, int32_t start,
                              int32_t *sweeps, void *workspace, size_t workspace_bytes, void *stream);

/*
 * shampoo_root_inverse for callers that cannot allocate device memory or must not see an
 * allocation happen: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments and results as shampoo_root_inverse without the
 * workspace: the solver's working arrays live in a fixed array of
 * SHAMPOO_STATIC_SCRATCH_BYTES inside the library's device image (one copy per GPU, held
 * until the process ends), and matrices are processed as many at a time as fit there
 * (n = 2048: one, n = 1024: four; n <= 128 needs no scratch at all).  The call allocates
 * nothing, creates no streams and enqueues kernels only (no memset nodes), all on `stream`.
 * n > SHAMPOO_STATIC_MAX_N: SHAMPOO_ERR_UNSUPPORTED, nothing enqueued.
 * Every call on a GPU uses that GPU's one array: calls whose work overlaps on one GPU (two
 * streams, two threads) race; the caller orders them.
 */
#define SHAMPOO_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
#define SHAMPOO_STATIC_MAX_N 2048
int shampoo_root_inverse_static(const float *a, int32_t n, int32_t batch, float epsilon, float r,
                                float *x, float *lambda, int32_t *failed, void *stream);

/*
 * Stand-alone batched coupled inverse Newton iteration (Sec. 3.2.1, item 2):
 *   A_i = a_i + epsilon I,  c = (2 ||A_i||_F / (p + 1))^(1/p),  X_0 = I / c,  M_0 = A_i / c^p,
 *   X_{k+1} = X_k T_k,  M_{k+1} = T_k^p M_k,  T_k = ((p + 1) I - M_k) / p,
 * ended per matrix at the first k with ||M_k - I||_inf < tolerance, at k = max_iterations,
 * or when the norm has reached the floor of float32 arithmetic (below 0.1 and no longer
 * halving).  x_i = X_k approximates A_i^(-1/p).
 * a:          device, batch dense row-major symmetric n x n float32 matrices (read only)
 * p:          1, 2, 4 or 8 (else SHAMPOO_ERR_UNSUPPORTED)
 * x:          device, batch n x n float32 outputs (may not alias a)
 * iterations: device int32[batch], the k at which each matrix ended, or NULL
 * failed:     device int32[batch] set to 1 where A_i or an iterate is not finite (x_i is
 *             then left untouched), else 0; or NULL
 * workspace:  device, 256-byte aligned, at least
 *             shampoo_root_inverse_newton_workspace_bytes(n, batch) bytes
 * Asynchronous on `stream`; no host synchronisation inside.
 */
size_t shampoo_root_inverse_newton_workspace_bytes(int32_t n, int32_t batch);
int shampoo_root_inverse_newton(const float *a, int32_t n, int32_t batch, float epsilon, int32_t p,
                                float tolerance, int32_t max_iterations, float *x,
                                int32_t *iterations, int32_t *failed,
                                void *workspace, size_t workspace_bytes, void *stream);

/* The order in which the Jacobi eigensolver of the refresh (Sec. 3.2.1: the root inverse by
 * symmetric eigendecomposition) visits index pairs: pair `k` (0 <= k < s / 2) of round `round`
 * (0 <= round < s - 1) of a sweep over s indices, written to *p < *q.  Every round is a
 * perfect matching and the s - 1 rounds cover every pair once.  halves = 0: the plain
 * tournament (any even s >= 2, the solver for n <= 128).  halves = 1: the order of the
 * 64 x 64 pivots of the blocked solver (s / 2 a power of two, s >= 4): rounds 0 .. s / 2 - 1
 * pair the first half of the indices with the second, the remaining rounds pair within the
 * halves.  halves = 2: the order of the block columns of the blocked solver when their number
 * s is a multiple of 4: indices 2 S and 2 S + 1 form a super-column, round 0 pairs the members
 * of every super-column, and rounds 1 + 2 R, 2 + 2 R are the two rounds of the meetings (S, T)
 * of round R of the super-columns' own tournament: (2 S, 2 T), (2 S + 1, 2 T + 1), then
 * (2 S, 2 T + 1), (2 S + 1, 2 T); pairs 2 K and 2 K + 1 of both rounds belong to meeting K.
 * Host only, no device work; SHAMPOO_ERR_NULL / SHAMPOO_ERR_SHAPE on bad arguments. */
int shampoo_jacobi_pair(int32_t s, int32_t halves, int32_t round, int32_t k, int32_t *p, int32_t *q);

/* Static, NUL-terminated description of a return code. */
const char *shampoo_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SHAMPOO_H */
