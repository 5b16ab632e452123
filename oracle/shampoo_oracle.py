"""fp64 CPU oracle for the per-block Shampoo optimizer step.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP path is checked against.  Only the test-suite, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does, and
this module imports nothing from the product package.  It shares no code,
tables or helpers with the HIP kernels.

Everything is numpy float64.  Inputs given as float32 (or bf16 bits decoded
to float32 by the caller) are widened exactly.  No blocking, fusion or
reordering beyond what the paper's algorithm states.

What is computed (paper: "Complete Distributed Shampoo Pseudocode"; identical to
"Shampoo Pseudocode (with AdaGrad Grafting)" when beta2 = 1, beta1 = 0, no
weight decay, no momentum):

  for every block (m x n) of every 2-D parameter, at iteration t (0-based):
    0. if weight_decay > 0 and not decoupled: G <- G + weight_decay * W   [Sec. 3.1.2]
    1. L <- beta2 L + (1-beta2) G G^T,  R <- beta2 R + (1-beta2) G^T G
       (plain sums when beta2 == 1; L = R = 0 initially)      [Sec. 3.1.1 EMA eqs]
    2. AdaGrad grafting: A <- A + G*G elementwise (SGD grafting has no state)  [Sec. 2.4]
       RMSprop / Adam grafting: A <- beta_g A + (1 - beta_g) G*G           [Sec. 2.2 EMA eq.]
    3. if t >= start and t % f == 0:
         Lbar <- rootinv(L), Rbar <- rootinv(R)                [Sec. 3.2.1 framed box;
         or, on request, the coupled inverse Newton iteration of the same section]
         (with bias correction and beta2 < 1: of L / (1 - beta2^(t+1)), likewise R)
    4. if beta1 > 0: Gf <- beta1 Gf + (1-beta1) G (Gf = 0 initially), else Gf = G.
       The grafting state above uses G, every direction below uses Gf
       (with bias correction and beta1 > 0: Gf / (1 - beta1^(t+1)))      [Sec. 3.1.1]
    5. P_graft = Gf / (sqrt(A) + eps_graft)  (AdaGrad, RMSprop)  or  Gf  (SGD)    [Sec. 2.4]
       Adam grafting with bias correction: A / (1 - beta_g^(t+1)) under the root
    6. if t >= start: P = -||P_graft||_F * Lbar Gf Rbar / ||Lbar Gf Rbar||_F
       else:          P = -P_graft                             [Sec. 2.4 grafting eq.]
    7. if weight_decay > 0 and decoupled: P <- P - weight_decay * W      [Sec. 3.1.2 eqs]
    8. if mu > 0: M <- mu M + P ; P <- mu M + P (Nesterov) or P <- M     [Sec. 3.1.3 eqs]
    9. W <- W + lr * P
  1-D parameters take steps 0, 2 (always AdaGrad), 4, P = -Gf / (sqrt(A) + eps_graft),
  7, 8, 9 (diagonal AdaGrad, Sec. 2.2 / Sec. 4.2.2).

  A 2-D parameter with a dimension above the block size is, by large_dim_method (Sec. 4.2):
    "blocking"  cut into blocks as above (Sec. 4.2.1);
    "adagrad"   handled like a 1-D parameter, i.e. by the diagonal method (Sec. 4.2.2);
    "diagonal"  kept whole, with the factor of every dimension above the block size
                replaced by its diagonal: l_i <- beta2 l_i + (1-beta2) sum_j G_ij^2 (likewise
                r_j), root inverse elementwise by the same framed box (Sec. 4.2.3).

  A parameter of order 3 or more first has its small dimensions merged (Sec. 4.2.1): going
  from the left, a dimension is multiplied into the current group while the product stays
  within the block size (a dimension of size 1 always is).  If two dimensions remain it is the matrix case above on the merged
  shape.  Otherwise (three or more remain, or one: everything merged) it is Shampoo for a
  tensor of order w (Sec. 2.3 / 3, "root 2w"): every dimension is cut into pieces of at most
  the block size; each sub-tensor block keeps one factor per dimension k,
      L_k <- beta2 L_k + (1-beta2) G_(k) G_(k)^T      (G_(k): the mode-k unfolding),
  its root inverse is taken with exponent 2 * root_exponent / w (1/(2w) for root_exponent =
  1/4; w = 1 is full-matrix AdaGrad with exponent 1/2), and
      P_shampoo = G x_1 Lbar_1 x_2 Lbar_2 ... x_w Lbar_w     (mode products);
  grafting, decay, momentum and the update are those of the matrix case.

Readings of the paper taken here (each also listed in the design notes):
  * Factors start at zero and epsilon enters only inside the root-inverse
    routine (the complete pseudocode + framed box), not as L_{-1} = eps*I.
  * The EMA weight in the factor update is beta2 (the complete pseudocode
    prints beta1 there while guarding on beta2 < 1; the text equations use
    beta2).
  * Bias correction is optional and off by default (the workloads do not list it).
    When on, the corrected factor is what the root routine receives, so epsilon is
    added after the division; the stored factors and the filtered gradient stay
    uncorrected, as in Adam.
  * Grafting norms are taken per block (each block owns its grafting object,
    App. E class structure).
  * The grafting branch before start_preconditioning_step uses P = -P_graft
    (sign consistent with W <- W + lr P).
  * Momentum recursion is M_t = mu M_{t-1} + P_t.
  * If ||P_shampoo||_F == 0 or ||P_graft||_F == 0 the block's P is zero.
  * Decoupled weight decay enters as P <- P - weight_decay * W: the complete
    pseudocode prints a plus sign, but its P already carries the minus sign of the
    step (W <- W + lr P), and the text equations give W_{t+1} = (1 - lr wd) W_t - ....
  * 1-D parameters run the diagonal method that the blocks graft from (AdaGrad, RMSprop or
    Adam; Sec. 4.2.2 offers exactly these in place of Shampoo), and AdaGrad under SGD grafting.
  * root_exponent is the matrix value (1/4); a tensor of order w uses 2 * root_exponent / w,
    i.e. the paper's exponent multiplier applied to the default 1/(2w).  Merging applies to
    parameters given with three or more dimensions; a matrix is taken as the caller shaped it
    (the workloads reshape convolution weights to matrices themselves).  The large-dimension
    methods other than blocking apply to matrices only.
  * RMSprop and Adam grafting differ only in the bias correction of the second moment,
    which Adam applies when bias correction is on; gradient filtering (beta1) is the
    optimizer-wide heuristic of Sec. 3.1.1 for every grafting type.

Pins: see tests/test_oracle_pins.py (Kronecker brute force, X^4 (L+eps I) = I,
diagonal closed forms, polar factor at t = 0, textbook AdaGrad, geometric
momentum and Nesterov sums, trace identities, independent Jacobi eigensolver,
geometric weight decay, l2 as a shifted gradient, constant-gradient filtering,
SGD-graft step length, bias correction under a constant gradient, coupled Newton against
the spectral definition and scalar closed forms, RMSprop / Adam grafting against textbook
RMSprop and Adam on 1-D parameters, merging against the paper's worked example, the
order-3 direction against the explicit Kronecker product and against closed forms on rank-one
tensors and fully merged vectors).
"""
import numpy as np


# ----------------------------------------------------------------------------
# Blocking (Sec. 4.2.1 "Merging and Blocking": k_m = ceil(m/b), k_n = ceil(n/b),
# full b x b blocks except the last block row / column, which hold the rest).
# ----------------------------------------------------------------------------
def block_partition(rows, cols, b):
    """Return the list of (row0, col0, m, n) blocks of a rows x cols matrix."""
    if rows <= 0 or cols <= 0 or b <= 0:
        raise ValueError("bad shape or block size")
    km = -(-rows // b)
    kn = -(-cols // b)
    blocks = []
    for i in range(km):
        for j in range(kn):
            r0 = i * b
            c0 = j * b
            blocks.append((r0, c0, min(b, rows - r0), min(b, cols - c0)))
    return blocks


def merge_dims(shape, b):
    """Merging small dimensions (Sec. 4.2.1): consecutive dimensions are merged, from the
    left, while the product stays within b.  (10, 2, 2, 4) with b = 8 gives (10, 4, 4).
    A dimension of size 1 always merges (it changes no product; the paper names the removal
    of unit dimensions as a purpose of merging): (512, 256, 1, 1) with b = 128 is (512, 256)."""
    shape = [int(d) for d in shape]
    if not shape or any(d <= 0 for d in shape) or b <= 0:
        raise ValueError("bad shape or block size")
    merged, cur = [], shape[0]
    for d in shape[1:]:
        if cur * d <= b or d == 1 or cur == 1:
            cur *= d
        else:
            merged.append(cur)
            cur = d
    merged.append(cur)
    return tuple(merged)


def tensor_block_partition(shape, b):
    """Blocks of an order-w tensor: every dimension cut into pieces of at most b (full pieces
    except the last).  Returns a list of (starts, dims), block indices in row-major order."""
    pieces = []
    for d in shape:
        k = -(-d // b)
        pieces.append([(i * b, min(b, d - i * b)) for i in range(k)])
    blocks = [((), ())]
    for dim_pieces in pieces:
        blocks = [(st + (s0,), dm + (dd,)) for (st, dm) in blocks for (s0, dd) in dim_pieces]
    return blocks


def unfold(G, k):
    """Mode-k unfolding G_(k): dimension k becomes the rows, all others the columns."""
    G = np.asarray(G, dtype=np.float64)
    return np.moveaxis(G, k, 0).reshape(G.shape[k], -1)


def tensor_factor_update(Ls, G, beta2):
    """L_k <- beta2 L_k + (1 - beta2) G_(k) G_(k)^T for every dimension k (plain sums when
    beta2 == 1): the tensor form of the Kronecker factors (Sec. 2.3, Sec. 3.1.1)."""
    out = []
    for k, L in enumerate(Ls):
        Gk = unfold(G, k)
        S = Gk @ Gk.T
        out.append(beta2 * L + (1.0 - beta2) * S if beta2 < 1.0 else L + S)
    return out


def mode_product(G, X, k):
    """G x_k X: every mode-k fibre of G is multiplied by the matrix X."""
    return np.moveaxis(np.tensordot(X, G, axes=(1, k)), 0, k)


def tensor_shampoo_direction(Xs, G):
    """P_shampoo = G x_1 X_1 x_2 X_2 ... x_w X_w (Sec. 2.3, tensor case)."""
    P = np.asarray(G, dtype=np.float64)
    for k, X in enumerate(Xs):
        P = mode_product(P, X, k)
    return P


# ----------------------------------------------------------------------------
# Stage functions
# ----------------------------------------------------------------------------
def factor_update(L, R, G, beta2):
    """Kronecker factor accumulation, Sec. 3.1.1 EMA equations / pseudocode."""
    G = np.asarray(G, dtype=np.float64)
    GGt = G @ G.T
    GtG = G.T @ G
    if beta2 < 1.0:
        return beta2 * L + (1.0 - beta2) * GGt, beta2 * R + (1.0 - beta2) * GtG
    return L + GGt, R + GtG


def graft_state_update(A, G):
    """AdaGrad grafting state: running sum of squared gradients (Sec. 2.4)."""
    G = np.asarray(G, dtype=np.float64)
    return A + G * G


def graft_state_update_ema(A, G, beta_g):
    """RMSprop / Adam second moment: exponential moving average of squared gradients (Sec. 2.2)."""
    G = np.asarray(G, dtype=np.float64)
    return beta_g * A + (1.0 - beta_g) * G * G


def graft_direction(G, A, eps_graft):
    """P_graft = G / (A^{1/2} + eps_graft), elementwise (Sec. 2.4)."""
    G = np.asarray(G, dtype=np.float64)
    return G / (np.sqrt(A) + eps_graft)


def root_inverse(F, epsilon, r):
    """Framed box "Symmetric Eigendecomposition Approach for Computing Root
    Inverse" (Sec. 3.2.1):
        lambda, Q = eigh(F)
        lambda_new = lambda - min(lambda_min, 0) + epsilon
        return Q diag(lambda_new^{-r}) Q^T
    Returns (root inverse, lambda).  numpy's LAPACK eigh is the library step.
    """
    F = np.asarray(F, dtype=np.float64)
    lam, Q = np.linalg.eigh(F)
    lam_min = lam.min()
    lam_new = lam - min(lam_min, 0.0) + epsilon
    X = (Q * lam_new ** (-r)) @ Q.T
    return X, lam


def root_inverse_newton(F, epsilon, p, tol=1e-6, max_iterations=100):
    """Coupled inverse Newton iteration of Sec. 3.2.1 (item 2) for (F + epsilon I)^(-1/p):
        c   = (2 ||A||_F / (p + 1))^(1/p),  A = F + epsilon I
        X_0 = I / c,   M_0 = A / c^p
        X_{k+1} = X_k T_k,   M_{k+1} = T_k^p M_k,   T_k = ((p + 1) I - M_k) / p
    stopped at the first k with ||M_k - I||_inf < tol (maximum absolute row sum), or after
    max_iterations steps.  Returns (X_k, k, ||M_k - I||_inf).  The paper leaves open how
    epsilon enters this variant and the iteration cap; the readings taken are: epsilon is
    added to the matrix before the iteration, and the cap is a parameter."""
    F = np.asarray(F, dtype=np.float64)
    n = F.shape[0]
    I = np.eye(n)
    A = F + epsilon * I
    c = (2.0 * np.sqrt(np.sum(A * A)) / (p + 1.0)) ** (1.0 / p)
    X = I / c
    M = A / c ** p
    k = 0
    while True:
        err = np.max(np.sum(np.abs(M - I), axis=1))
        if err < tol or k >= max_iterations:
            return X, k, err
        T = ((p + 1.0) * I - M) / p
        X = X @ T
        M = np.linalg.matrix_power(T, p) @ M
        k += 1


def shampoo_direction(Lbar, G, Rbar):
    """P_shampoo = Lbar G Rbar (Sec. 2.3 Shampoo update)."""
    return Lbar @ np.asarray(G, dtype=np.float64) @ Rbar


def grafted_direction(P_sh, P_graft):
    """P = -||P_graft||_F P_sh / ||P_sh||_F (Sec. 2.4); zero if either norm is zero."""
    n_sh = np.sqrt(np.sum(P_sh * P_sh))
    n_g = np.sqrt(np.sum(P_graft * P_graft))
    if n_sh == 0.0 or n_g == 0.0:
        return np.zeros_like(P_sh)
    return -(n_g / n_sh) * P_sh


# ----------------------------------------------------------------------------
# Whole optimizer
# ----------------------------------------------------------------------------
class ShampooOracle:
    """State and step of the optimizer for a list of 1-D / 2-D parameters.

    shapes: list of tuples, (len,) or (rows, cols).
    State per 2-D block: L, R, Lbar, Rbar; per element: A, M.  All float64.
    """

    def __init__(self, shapes, block_size, beta2, epsilon, root_exponent,
                 precondition_frequency, start_preconditioning_step=0,
                 graft_epsilon=1e-10, momentum=0.0, beta1=0.0, weight_decay=0.0,
                 use_decoupled_weight_decay=True, use_nesterov=False, grafting="adagrad",
                 use_bias_correction=False, root_method="eigh", newton_tolerance=1e-6,
                 newton_max_iterations=100, grafting_beta2=0.999, large_dim_method="blocking"):
        self.shapes = [tuple(int(x) for x in s) for s in shapes]
        self.b = int(block_size)
        self.beta2 = float(beta2)
        self.epsilon = float(epsilon)
        self.r = float(root_exponent)
        self.f = int(precondition_frequency)
        self.start = int(start_preconditioning_step)
        self.eps_g = float(graft_epsilon)
        self.mu = float(momentum)
        self.beta1 = float(beta1)
        self.wd = float(weight_decay)
        self.decoupled = bool(use_decoupled_weight_decay)
        self.nesterov = bool(use_nesterov)
        self.bias_correction = bool(use_bias_correction)
        if root_method not in ("eigh", "newton"):
            raise ValueError("root_method must be 'eigh' or 'newton'")
        self.root_method = root_method
        self.newton_tol = float(newton_tolerance)
        self.newton_max_iter = int(newton_max_iterations)
        if grafting not in ("adagrad", "sgd", "rmsprop", "adam"):
            raise ValueError("grafting must be 'adagrad', 'sgd', 'rmsprop' or 'adam'")
        self.grafting = grafting
        self.beta_g = float(grafting_beta2)
        if large_dim_method not in ("blocking", "adagrad", "diagonal"):
            raise ValueError("large_dim_method must be 'blocking', 'adagrad' or 'diagonal'")
        self.large_dim_method = large_dim_method
        # per 2-D parameter: None (blocked / small), "adagrad", or (L is diagonal, R is diagonal)
        self.whole = []
        self.blocks = []      # per param: list of (r0, c0, m, n) (empty for 1-D)
        self.L, self.R, self.Lbar, self.Rbar = [], [], [], []
        self.A, self.M, self.Gf = [], [], []
        self.P_sh = []        # last Shampoo direction per block (for inspection)
        self.s_g, self.s_sh = [], []   # last squared norms per block
        # the shape each parameter is worked on (after merging); state arrays have this shape
        self.view_shapes = [merge_dims(s, self.b) if len(s) >= 3 else s for s in self.shapes]
        # tensor parameters (order 1 after merging, or >= 3): per block the list of factors / roots
        self.tblocks, self.TL, self.TLbar = {}, {}, {}
        for i, s in enumerate(self.view_shapes):
            if len(self.shapes[i]) >= 3 and len(s) != 2:
                blks = tensor_block_partition(s, self.b)
                self.tblocks[i] = blks
                self.TL[i] = [[np.zeros((d, d)) for d in dims] for (_, dims) in blks]
                self.TLbar[i] = [[np.eye(d) for d in dims] for (_, dims) in blks]
                self.A.append(np.zeros(s)); self.M.append(np.zeros(s)); self.Gf.append(np.zeros(s))
                self.whole.append(None)
                self.blocks.append([])
                for lst in (self.L, self.R, self.Lbar, self.Rbar):
                    lst.append([])
                self.P_sh.append([None] * len(blks))
                self.s_g.append([0.0] * len(blks))
                self.s_sh.append([0.0] * len(blks))
                continue
            self._init_matrix_or_vector(s)

    def _init_matrix_or_vector(self, s):
        """State of a vector or matrix parameter of (merged) shape s."""
        large_dim_method = self.large_dim_method
        self.A.append(np.zeros(s))
        self.M.append(np.zeros(s))
        self.Gf.append(np.zeros(s))
        big = len(s) == 2 and (s[0] > self.b or s[1] > self.b)
        if len(s) == 2 and big and large_dim_method == "adagrad":
            self.whole.append("adagrad")
            self.blocks.append([])
            for lst in (self.L, self.R, self.Lbar, self.Rbar, self.P_sh, self.s_g, self.s_sh):
                lst.append([])
        elif len(s) == 2 and big and large_dim_method == "diagonal":
            dl, dr = s[0] > self.b, s[1] > self.b
            self.whole.append((dl, dr))
            self.blocks.append([(0, 0, s[0], s[1])])
            # a diagonalised factor is stored as the vector of its diagonal
            self.L.append([np.zeros(s[0]) if dl else np.zeros((s[0], s[0]))])
            self.R.append([np.zeros(s[1]) if dr else np.zeros((s[1], s[1]))])
            self.Lbar.append([np.ones(s[0]) if dl else np.eye(s[0])])
            self.Rbar.append([np.ones(s[1]) if dr else np.eye(s[1])])
            self.P_sh.append([None])
            self.s_g.append([0.0])
            self.s_sh.append([0.0])
        elif len(s) == 2:
            self.whole.append(None)
            blks = block_partition(s[0], s[1], self.b)
            self.blocks.append(blks)
            self.L.append([np.zeros((m, m)) for (_, _, m, n) in blks])
            self.R.append([np.zeros((n, n)) for (_, _, m, n) in blks])
            # before the first refresh the previous root is the identity
            self.Lbar.append([np.eye(m) for (_, _, m, n) in blks])
            self.Rbar.append([np.eye(n) for (_, _, m, n) in blks])
            self.P_sh.append([None] * len(blks))
            self.s_g.append([0.0] * len(blks))
            self.s_sh.append([0.0] * len(blks))
        elif len(s) == 1:
            self.whole.append(None)
            self.blocks.append([])
            for lst in (self.L, self.R, self.Lbar, self.Rbar, self.P_sh,
                        self.s_g, self.s_sh):
                lst.append([])
        else:
            raise ValueError("bad parameter shape")

    def _root(self, F, r=None):
        r = self.r if r is None else r
        if self.root_method == "newton":
            with np.errstate(over="ignore", invalid="ignore"):
                X, _, err = root_inverse_newton(F, self.epsilon, int(round(1.0 / r)), self.newton_tol,
                                                self.newton_max_iter)
            # guard of Sec. 3.2.3: a failed root computation is retried by the other, more
            # accurate routine (here: the eigendecomposition) before the previous root is kept
            if np.isfinite(err) and np.all(np.isfinite(X)):
                return X
        return root_inverse(F, self.epsilon, r)[0]

    def _graft_state(self, A, G):
        if self.grafting in ("rmsprop", "adam"):
            return graft_state_update_ema(A, G, self.beta_g)
        return graft_state_update(A, G)

    def _second_moment(self, A, t):
        """What goes under the square root of the grafted direction."""
        if self.grafting == "adam" and self.bias_correction and self.beta_g < 1.0:
            return A / (1.0 - self.beta_g ** (t + 1))
        return A

    def _diag_root(self, d):
        """The framed box of Sec. 3.2.1 on a diagonal matrix: its eigenvalues are its entries."""
        lam_new = d - min(d.min(), 0.0) + self.epsilon
        return lam_new ** (-self.r)

    def _finish(self, i, sl, P, W, lr):
        """Steps 7-9 on one block / vector: decoupled decay, momentum, update."""
        if self.wd > 0.0 and self.decoupled:
            P = P - self.wd * W[sl]
        if self.mu > 0.0:
            self.M[i][sl] = self.mu * self.M[i][sl] + P
            P = self.mu * self.M[i][sl] + P if self.nesterov else self.M[i][sl]
        W[sl] += lr * P

    def step(self, params, grads, lr, t):
        """One iteration t.  params: list of float64 arrays, updated in place.
        grads: list of arrays (any float dtype; widened exactly)."""
        refresh = (t >= self.start) and (t % self.f == 0)
        # Sec. 3.1.1 bias correction: G^ = Gf / (1 - beta1^(t+1)), L^ = L / (1 - beta2^(t+1))
        c1 = c2 = 1.0
        if self.bias_correction and self.beta1 > 0.0:
            c1 = 1.0 / (1.0 - self.beta1 ** (t + 1))
        if self.bias_correction and self.beta2 < 1.0:
            c2 = 1.0 / (1.0 - self.beta2 ** (t + 1))
        for i, s in enumerate(self.view_shapes):
            G = np.asarray(grads[i], dtype=np.float64).reshape(s)
            W = params[i].reshape(s)      # a view: merging moves no data (Sec. 4.2.1)
            if W.base is None and W is not params[i]:
                raise ValueError("parameters must be C-contiguous")
            if self.wd > 0.0 and not self.decoupled:
                G = G + self.wd * W
            if self.beta1 > 0.0:
                self.Gf[i] = self.beta1 * self.Gf[i] + (1.0 - self.beta1) * G
                Gf = c1 * self.Gf[i]
            else:
                Gf = G
            if i in self.tblocks:
                self._tensor_blocks(i, G, Gf, W, lr, t, refresh, c2)
                continue
            if len(s) == 1 or self.whole[i] == "adagrad":
                self.A[i] = self._graft_state(self.A[i], G)
                P = -graft_direction(Gf, self._second_moment(self.A[i], t), self.eps_g)
                self._finish(i, slice(None), P, W, lr)
                continue
            for k, (r0, c0, m, n) in enumerate(self.blocks[i]):
                sl = (slice(r0, r0 + m), slice(c0, c0 + n))
                Gb, Gfb = G[sl], Gf[sl]
                if self.whole[i] is not None:
                    P = self._diagonal_shampoo(i, Gb, Gfb, t, refresh, c2)
                    self._finish(i, sl, P, W, lr)
                    continue
                self.L[i][k], self.R[i][k] = factor_update(
                    self.L[i][k], self.R[i][k], Gb, self.beta2)
                if self.grafting != "sgd":
                    self.A[i][sl] = self._graft_state(self.A[i][sl], Gb)
                if refresh:
                    self.Lbar[i][k] = self._root(c2 * self.L[i][k])
                    self.Rbar[i][k] = self._root(c2 * self.R[i][k])
                if self.grafting != "sgd":
                    Pg = graft_direction(Gfb, self._second_moment(self.A[i][sl], t), self.eps_g)
                else:
                    Pg = Gfb.copy()
                self.s_g[i][k] = float(np.sum(Pg * Pg))
                if t >= self.start:
                    Psh = shampoo_direction(self.Lbar[i][k], Gfb, self.Rbar[i][k])
                    self.P_sh[i][k] = Psh
                    self.s_sh[i][k] = float(np.sum(Psh * Psh))
                    P = grafted_direction(Psh, Pg)
                else:
                    P = -Pg
                self._finish(i, sl, P, W, lr)

    def _tensor_blocks(self, i, G, Gf, W, lr, t, refresh, c2):
        """Shampoo for a tensor of order w (Sec. 2.3 / 3): one factor per dimension, roots with
        exponent 2 r / w, mode products; everything else as for a matrix block."""
        w = len(self.view_shapes[i])
        rw = 2.0 * self.r / w
        for k, (starts, dims) in enumerate(self.tblocks[i]):
            sl = tuple(slice(s0, s0 + d) for s0, d in zip(starts, dims))
            Gb, Gfb = G[sl], Gf[sl]
            self.TL[i][k] = tensor_factor_update(self.TL[i][k], Gb, self.beta2)
            if self.grafting != "sgd":
                self.A[i][sl] = self._graft_state(self.A[i][sl], Gb)
            if refresh:
                self.TLbar[i][k] = [self._root(c2 * L, rw) for L in self.TL[i][k]]
            if self.grafting != "sgd":
                Pg = graft_direction(Gfb, self._second_moment(self.A[i][sl], t), self.eps_g)
            else:
                Pg = Gfb.copy()
            self.s_g[i][k] = float(np.sum(Pg * Pg))
            if t >= self.start:
                Psh = tensor_shampoo_direction(self.TLbar[i][k], Gfb)
                self.P_sh[i][k] = Psh
                self.s_sh[i][k] = float(np.sum(Psh * Psh))
                P = grafted_direction(Psh, Pg)
            else:
                P = -Pg
            self._finish(i, sl, P, W, lr)

    def _diagonal_shampoo(self, i, G, Gf, t, refresh, c2):
        """Sec. 4.2.3 on a whole parameter: factors of the large dimensions are diagonal."""
        dl, dr = self.whole[i]
        a, b = (self.beta2, 1.0 - self.beta2) if self.beta2 < 1.0 else (1.0, 1.0)
        GGt_diag = np.sum(G * G, axis=1)           # diag(G G^T)
        GtG_diag = np.sum(G * G, axis=0)           # diag(G^T G)
        self.L[i][0] = a * self.L[i][0] + b * (GGt_diag if dl else G @ G.T)
        self.R[i][0] = a * self.R[i][0] + b * (GtG_diag if dr else G.T @ G)
        if self.grafting != "sgd":
            self.A[i] = self._graft_state(self.A[i], G)
        if refresh:
            self.Lbar[i][0] = self._diag_root(c2 * self.L[i][0]) if dl else self._root(c2 * self.L[i][0])
            self.Rbar[i][0] = self._diag_root(c2 * self.R[i][0]) if dr else self._root(c2 * self.R[i][0])
        Pg = graft_direction(Gf, self._second_moment(self.A[i], t), self.eps_g) if self.grafting != "sgd" else Gf.copy()
        self.s_g[i][0] = float(np.sum(Pg * Pg))
        if t < self.start:
            return -Pg
        T = self.Lbar[i][0][:, None] * Gf if dl else self.Lbar[i][0] @ Gf
        Psh = T * self.Rbar[i][0][None, :] if dr else T @ self.Rbar[i][0]
        self.P_sh[i][0] = Psh
        self.s_sh[i][0] = float(np.sum(Psh * Psh))
        return grafted_direction(Psh, Pg)
