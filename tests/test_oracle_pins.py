"""Pins for the fp64 oracle: each test ties one part of oracle/shampoo_oracle.py
to something fixed by the paper or by mathematics, written independently of the
oracle's own formulae.  CPU only."""
import numpy as np
import pytest

from oracle import shampoo_oracle as so
from paper_2309_06497_amd import workloads as wl


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------------------
# an eigensolver that is not LAPACK: cyclic Jacobi, plain loops (tiny n only)
# ---------------------------------------------------------------------------
def jacobi_eigh(A, sweeps=30):
    A = np.array(A, dtype=np.float64)
    n = A.shape[0]
    V = np.eye(n)
    for _ in range(sweeps):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                if abs(A[p, q]) < 1e-150:
                    continue
                off += A[p, q] ** 2
                tau = (A[q, q] - A[p, p]) / (2.0 * A[p, q])
                t = (1.0 if tau >= 0 else -1.0) / (abs(tau) + np.sqrt(1.0 + tau * tau))
                c = 1.0 / np.sqrt(1.0 + t * t)
                s = t * c
                Rm = np.eye(n)
                Rm[p, p] = c; Rm[q, q] = c; Rm[p, q] = s; Rm[q, p] = -s
                A = Rm.T @ A @ Rm
                V = V @ Rm
        if off < 1e-300:
            break
    return np.diag(A).copy(), V


# ---------------------------------------------------------------------------
# Blocking  (Sec. 4.2.1)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("rows,cols,b", [(256, 128, 64), (64, 147, 128), (2048, 1000, 128),
                                         (5, 7, 3), (1, 1, 4), (130, 130, 128)])
def test_block_partition_covers_once(rows, cols, b):
    blks = so.block_partition(rows, cols, b)
    assert len(blks) == -(-rows // b) * -(-cols // b)
    cover = np.zeros((rows, cols), dtype=np.int32)
    for (r0, c0, m, n) in blks:
        assert 1 <= m <= b and 1 <= n <= b
        # full blocks except in the last block row / column
        if r0 + m < rows:
            assert m == b
        if c0 + n < cols:
            assert n == b
        cover[r0:r0 + m, c0:c0 + n] += 1
    assert (cover == 1).all()


def test_resnet50_block_histogram():
    shapes = wl.resnet50_shapes()
    two_d = [s for s in shapes if len(s) == 2]
    one_d = [s for s in shapes if len(s) == 1]
    assert len(two_d) == 54 and len(one_d) == 107
    assert sum(wl.numel(s) for s in shapes) == 25_557_032
    hist = {}
    for (r, c) in two_d:
        for (_, _, m, n) in so.block_partition(r, c, 128):
            hist[(m, n)] = hist.get((m, n), 0) + 1
    assert hist == {(128, 128): 1530, (64, 128): 17, (128, 104): 16, (128, 64): 8,
                    (64, 64): 4, (64, 19): 1}


def test_transformer_shapes():
    shapes = wl.transformer_shapes()
    two_d = [s for s in shapes if len(s) == 2]
    assert sum(wl.numel(s) for s in two_d) == 1_207_959_552
    nblk = sum(len(so.block_partition(r, c, 1024)) for (r, c) in two_d)
    assert nblk == 1152
    assert sum(wl.numel(s) for s in shapes if len(s) == 1) == 98 * 2048


# ---------------------------------------------------------------------------
# Root inverse  (Sec. 2.2 definition via eigendecomposition; Sec. 3.2.1 box)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,r", [(1, 0.25), (2, 0.25), (7, 0.25), (33, 0.25), (12, 0.5)])
def test_root_inverse_power_identity(n, r):
    g = rng(n).standard_normal((n, n + 3))
    F = g @ g.T
    eps = 1e-12
    X, lam = so.root_inverse(F, eps, r)
    assert np.allclose(X, X.T, rtol=0, atol=1e-12 * np.abs(X).max())
    assert np.linalg.eigvalsh(X).min() > 0
    p = int(round(1.0 / r))
    Xp = np.linalg.matrix_power(X, p)
    err = np.linalg.norm(Xp @ (F + eps * np.eye(n)) - np.eye(n)) / np.sqrt(n)
    assert err < 1e-9
    assert np.all(np.diff(lam) >= 0)


def test_root_inverse_diagonal_closed_form():
    d = np.array([4.0, 0.25, 9.0, 1e-3, 0.0])
    eps = 1e-12
    X, _ = so.root_inverse(np.diag(d), eps, 0.25)
    assert np.allclose(X, np.diag((d + eps) ** -0.25), rtol=1e-13, atol=0)


def test_root_inverse_negative_eigenvalue_shift():
    # the box shifts by -min(lambda_min, 0): diag(-1, 3) -> lambda_new = (eps, 4 + eps)
    eps = 1e-6
    X, lam = so.root_inverse(np.diag([-1.0, 3.0]), eps, 0.25)
    assert np.allclose(lam, [-1.0, 3.0])
    assert np.allclose(X, np.diag([eps ** -0.25, (4.0 + eps) ** -0.25]), rtol=1e-12)
    # and a non-negative spectrum is not shifted at all
    X2, _ = so.root_inverse(np.diag([1.0, 3.0]), eps, 0.25)
    assert np.allclose(X2, np.diag([(1 + eps) ** -0.25, (3 + eps) ** -0.25]), rtol=1e-12)


def test_root_inverse_matches_independent_jacobi():
    g = rng(5).standard_normal((9, 11))
    F = g @ g.T
    eps = 1e-9
    X, lam = so.root_inverse(F, eps, 0.25)
    lam_j, V = jacobi_eigh(F)
    Xj = (V * (lam_j + eps) ** -0.25) @ V.T
    assert np.allclose(np.sort(lam_j), lam, rtol=1e-11)
    assert np.allclose(X, Xj, rtol=1e-9, atol=1e-12)


def test_root_inverse_orthogonal_equivariance():
    g = rng(6).standard_normal((8, 8))
    F = g @ g.T
    U, _ = np.linalg.qr(rng(7).standard_normal((8, 8)))
    X, _ = so.root_inverse(F, 1e-9, 0.25)
    XU, _ = so.root_inverse(U @ F @ U.T, 1e-9, 0.25)
    assert np.allclose(XU, U @ X @ U.T, rtol=1e-9, atol=1e-11)


# ---------------------------------------------------------------------------
# Two-sided preconditioning vs the explicit Kronecker product (Sec. 1.2 vec
# identities, Sec. 2.3): (L (x) R)^(-1/4) vec(G) = vec(L^(-1/4) G R^(-1/4)),
# vec taken row-wise.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("m,n", [(3, 4), (5, 5), (4, 2), (1, 6)])
def test_kronecker_brute_force(m, n):
    r = rng(100 * m + n)
    eps = 1e-3
    L = np.zeros((m, m)); R = np.zeros((n, n))
    for _ in range(3):
        G = r.standard_normal((m, n))
        L, R = so.factor_update(L, R, G, 1.0)
    Lbar, _ = so.root_inverse(L, eps, 0.25)
    Rbar, _ = so.root_inverse(R, eps, 0.25)
    P = so.shampoo_direction(Lbar, G, Rbar)
    # brute force with an eigensolver that is not LAPACK, on the mn x mn matrix
    K = np.kron(L + eps * np.eye(m), R + eps * np.eye(n))
    lam, V = jacobi_eigh(K)
    Kroot = (V * lam ** -0.25) @ V.T
    assert np.allclose(Kroot @ G.reshape(-1), P.reshape(-1), rtol=1e-8, atol=1e-10)


def test_factor_update_definition_and_trace():
    r = rng(3)
    m, n = 6, 9
    beta2 = 0.9
    L = np.zeros((m, m)); R = np.zeros((n, n))
    Ls = np.zeros((m, m)); Rs = np.zeros((n, n))
    tr = 0.0; trs = 0.0
    for t in range(5):
        G = r.standard_normal((m, n)).astype(np.float32)
        L, R = so.factor_update(L, R, G, beta2)
        Ls, Rs = so.factor_update(Ls, Rs, G, 1.0)
        g2 = float(np.sum(G.astype(np.float64) ** 2))
        tr = beta2 * tr + (1 - beta2) * g2
        trs += g2
        # elementwise definition: L_ij = sum_k G_ik G_jk, R_ij = sum_k G_ki G_kj
        assert np.isclose(np.trace(L), tr, rtol=1e-13)
        assert np.isclose(np.trace(R), tr, rtol=1e-13)
        assert np.isclose(np.trace(Ls), trs, rtol=1e-13)
        assert np.isclose(np.trace(Rs), trs, rtol=1e-13)
    assert L.shape == (m, m) and R.shape == (n, n)
    assert np.allclose(L, L.T) and np.allclose(R, R.T)
    assert np.linalg.eigvalsh(L).min() > -1e-12 * np.linalg.eigvalsh(L).max()
    Gd = G.astype(np.float64)
    L1, R1 = so.factor_update(np.zeros((m, m)), np.zeros((n, n)), G, 1.0)
    ref_L = np.array([[sum(Gd[i, k] * Gd[j, k] for k in range(n)) for j in range(m)] for i in range(m)])
    ref_R = np.array([[sum(Gd[k, i] * Gd[k, j] for k in range(m)) for j in range(n)] for i in range(n)])
    assert np.allclose(L1, ref_L, rtol=1e-13) and np.allclose(R1, ref_R, rtol=1e-13)


# ---------------------------------------------------------------------------
# Whole-step closed forms
# ---------------------------------------------------------------------------
def make_opt(shapes, **kw):
    args = dict(block_size=64, beta2=1.0, epsilon=1e-12, root_exponent=0.25,
                precondition_frequency=1, start_preconditioning_step=0,
                graft_epsilon=1e-10, momentum=0.0)
    args.update(kw)
    return so.ShampooOracle(shapes, **args)


@pytest.mark.parametrize("m,n", [(6, 4), (4, 6), (5, 5)])
def test_first_step_is_polar_factor(m, n):
    """beta2 = 1, t = 0, full-rank G = U S V^T: L^(-1/4) G R^(-1/4) = U V^T, the
    AdaGrad graft is sign(G), so W_1 = W_0 - lr sqrt(max(m, n)) U V^T."""
    G = rng(m * 10 + n).standard_normal((m, n))
    U, S, Vt = np.linalg.svd(G, full_matrices=False)
    # rank-deficient side: the null space gets eps^(-1/4) but G has no component there
    opt = make_opt([(m, n)], epsilon=1e-14)
    W = [np.zeros((m, n))]
    lr = 0.1
    opt.step(W, [G], lr, 0)
    expect = -lr * np.sqrt(max(m, n)) * (U @ Vt)
    assert np.allclose(W[0], expect, rtol=1e-6, atol=1e-8)
    assert np.isclose(opt.s_g[0][0], m * n, rtol=1e-8)
    assert np.isclose(opt.s_sh[0][0], min(m, n), rtol=1e-6)


def test_diagonal_gradients_reduce_to_adagrad():
    """If every G_s is diagonal, L = R = diag(sum d^2) and Shampoo's direction is
    d / sqrt(sum d^2), i.e. diagonal AdaGrad (App. B algebra)."""
    n = 6
    r = rng(11)
    opt = make_opt([(n, n)], epsilon=1e-30, graft_epsilon=1e-30)
    W = [np.zeros((n, n))]
    w_ref = np.zeros(n); acc = np.zeros(n)
    lr = 0.05
    for t in range(6):
        d = r.standard_normal(n) + 0.1
        opt.step(W, [np.diag(d)], lr, t)
        acc += d * d
        w_ref -= lr * d / np.sqrt(acc)
        assert np.allclose(np.diag(W[0]), w_ref, rtol=1e-9, atol=1e-12)
        assert np.allclose(W[0] - np.diag(np.diag(W[0])), 0.0, atol=1e-12)


def test_one_d_path_is_textbook_adagrad_with_momentum():
    n = 37
    r = rng(12)
    mu, lr, eg = 0.9, 0.01, 1e-10
    opt = make_opt([(n,)], momentum=mu, graft_epsilon=eg, precondition_frequency=10)
    W = [r.standard_normal(n)]
    w = W[0].copy(); a = np.zeros(n); mom = np.zeros(n)
    for t in range(12):
        g = (r.standard_normal(n) * 0.01).astype(np.float32)
        opt.step(W, [g], lr, t)
        for i in range(n):          # textbook loop, scalar by scalar
            gi = float(g[i])
            a[i] += gi * gi
            mom[i] = mu * mom[i] - gi / (np.sqrt(a[i]) + eg)
            w[i] += lr * mom[i]
        assert np.array_equal(W[0], w)


def test_grafting_norm_and_block_independence():
    """||P||_F equals the AdaGrad direction's norm per block; blocks of one
    parameter behave exactly like separate parameters."""
    r = rng(13)
    shape = (10, 7); b = 4
    G_seq = [r.standard_normal(shape) * 0.01 for _ in range(4)]
    lr = 0.3
    opt = make_opt([shape], block_size=b, beta2=0.9, precondition_frequency=2)
    W = [np.zeros(shape)]
    blks = so.block_partition(*shape, b)
    subs = [make_opt([(m, n)], block_size=b, beta2=0.9, precondition_frequency=2) for (_, _, m, n) in blks]
    Wsub = [[np.zeros((m, n))] for (_, _, m, n) in blks]
    acc = np.zeros(shape)
    for t, G in enumerate(G_seq):
        before = W[0].copy()
        opt.step(W, [G], lr, t)
        acc += G * G
        for k, (r0, c0, m, n) in enumerate(blks):
            sl = (slice(r0, r0 + m), slice(c0, c0 + n))
            delta = (W[0] - before)[sl]
            pg = G[sl] / (np.sqrt(acc[sl]) + 1e-10)
            assert np.isclose(np.linalg.norm(delta), lr * np.linalg.norm(pg), rtol=1e-10)
            subs[k].step(Wsub[k], [G[sl]], lr, t)
            assert np.allclose(W[0][sl], Wsub[k][0], rtol=1e-12, atol=1e-15)


def test_momentum_is_geometric_sum_of_directions():
    """Gradients do not depend on W here, so the directions P_s are the same with
    and without momentum and W_T = W_0 + lr sum_t sum_{s<=t} mu^(t-s) P_s."""
    r = rng(14)
    shapes = [(6, 5), (9,)]
    grads = [[r.standard_normal(s) * 0.1 for s in shapes] for _ in range(7)]
    lr, mu = 0.02, 0.8
    plain = make_opt(shapes, precondition_frequency=3)
    W = [np.zeros(s) for s in shapes]
    P = []
    for t, g in enumerate(grads):
        before = [w.copy() for w in W]
        plain.step(W, g, lr, t)
        P.append([(w - b0) / lr for w, b0 in zip(W, before)])
    mom = make_opt(shapes, precondition_frequency=3, momentum=mu)
    Wm = [np.zeros(s) for s in shapes]
    for t, g in enumerate(grads):
        mom.step(Wm, g, lr, t)
    for i in range(len(shapes)):
        expect = np.zeros(shapes[i])
        for t in range(len(grads)):
            for s_ in range(t + 1):
                expect += lr * mu ** (t - s_) * P[s_][i]
        assert np.allclose(Wm[i], expect, rtol=1e-10, atol=1e-14)


def test_refresh_schedule_and_warmup_branch():
    r = rng(15)
    shape = (5, 4)
    opt = make_opt([shape], precondition_frequency=3, start_preconditioning_step=2)
    W = [np.zeros(shape)]
    acc = np.zeros(shape)
    roots = []
    for t in range(8):
        G = r.standard_normal(shape)
        before = W[0].copy()
        opt.step(W, [G], 0.1, t)
        acc += G * G
        roots.append(opt.Lbar[0][0].copy())
        if t < 2:   # grafting direction only, with a minus sign
            assert np.allclose(W[0] - before, -0.1 * G / (np.sqrt(acc) + 1e-10), rtol=1e-12)
            assert np.array_equal(opt.Lbar[0][0], np.eye(5))
    # refresh at t = 3 and t = 6 only (t >= start and t % f == 0); stale otherwise
    assert np.array_equal(roots[2], np.eye(5))
    assert not np.array_equal(roots[3], roots[2])
    assert np.array_equal(roots[4], roots[3]) and np.array_equal(roots[5], roots[3])
    assert not np.array_equal(roots[6], roots[5])
    assert np.array_equal(roots[7], roots[6])
    # the refreshed root uses the factor that already contains G_t
    X, _ = so.root_inverse(opt.L[0][0], 1e-12, 0.25)
    assert not np.allclose(roots[6], X)   # L has moved on at t = 7 ...
    opt2 = make_opt([shape], precondition_frequency=1)
    W2 = [np.zeros(shape)]
    G = r.standard_normal(shape)
    opt2.step(W2, [G], 0.1, 0)
    X0, _ = so.root_inverse(G @ G.T, 1e-12, 0.25)
    assert np.allclose(opt2.Lbar[0][0], X0, rtol=1e-12)   # ... and at t = 0 it is rootinv(G0 G0^T)


def test_gradient_scale_invariance():
    """Scaling every gradient by c leaves the trajectory unchanged (grafting
    normalises the direction, AdaGrad's direction is scale-free) up to epsilon
    effects.  Roots are refreshed every step so that each G_t lies in the range
    of its own factors and epsilon (which does not scale) stays negligible."""
    r = rng(16)
    shapes = [(12, 9), (5,)]
    grads = [[r.standard_normal(s) for s in shapes] for _ in range(5)]
    outs = []
    for c in (1.0, 64.0):
        opt = make_opt(shapes, block_size=8, beta2=0.99, precondition_frequency=1, momentum=0.9,
                       epsilon=1e-20, graft_epsilon=1e-20)
        W = [np.zeros(s) for s in shapes]
        for t, g in enumerate(grads):
            opt.step(W, [c * x for x in g], 0.01, t)
        outs.append(W)
    for a, b in zip(*outs):
        assert np.allclose(a, b, rtol=1e-7, atol=1e-12)


def test_zero_gradient_block_is_safe():
    opt = make_opt([(4, 4)], momentum=0.9)
    W = [np.ones((4, 4))]
    opt.step(W, [np.zeros((4, 4))], 0.1, 0)
    assert np.array_equal(W[0], np.ones((4, 4)))
    assert np.all(np.isfinite(opt.Lbar[0][0]))


def test_bf16_helpers_roundtrip():
    x = rng(17).standard_normal(1000).astype(np.float32)
    bits = wl.f32_to_bf16_bits(x)
    y = wl.bf16_bits_to_f32(bits)
    assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(wl.f32_to_bf16_bits(y), bits)
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> rounds to 1
    assert wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32)))[0] == 1.0
    assert wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32)))[0] == 1.0 + 2.0 ** -6


# ---------------------------------------------------------------------------
# Heuristics of the complete pseudocode (Sec. 3.1): weight decay, gradient
# filtering, Nesterov, SGD grafting
# ---------------------------------------------------------------------------
def test_decoupled_weight_decay_is_geometric_shrink():
    """Zero gradients: W_{t+1} = (1 - lr wd) W_t (Sec. 3.1.2 decoupled equations)."""
    shapes = [(6, 5), (7,)]
    opt = make_opt(shapes, weight_decay=0.1, use_decoupled_weight_decay=True)
    r = rng(20)
    W0 = [r.standard_normal(s) for s in shapes]
    W = [w.copy() for w in W0]
    lr = 0.05
    for t in range(6):
        opt.step(W, [np.zeros(s) for s in shapes], lr, t)
    for w, w0 in zip(W, W0):
        assert np.allclose(w, w0 * (1 - lr * 0.1) ** 6, rtol=1e-13)


def test_decoupled_weight_decay_adds_to_the_grafted_step():
    """W_{t+1} = (1 - lr wd) W_t + lr P_t with P_t the step of the undecayed optimizer
    (weight decay sits outside the preconditioner and the grafting, Sec. 3.1.2)."""
    r = rng(21)
    shapes = [(8, 6)]
    grads = [[r.standard_normal(s) for s in shapes] for _ in range(4)]
    lr, wd = 0.1, 0.3
    plain = make_opt(shapes, precondition_frequency=2)
    Wp = [np.zeros(s) for s in shapes]
    P = []
    for t, g in enumerate(grads):
        before = Wp[0].copy()
        plain.step(Wp, g, lr, t)
        P.append((Wp[0] - before) / lr)
    dec = make_opt(shapes, precondition_frequency=2, weight_decay=wd)
    W = [r.standard_normal(shapes[0])]
    w_ref = W[0].copy()
    for t, g in enumerate(grads):
        dec.step(W, g, lr, t)
        w_ref = (1 - lr * wd) * w_ref + lr * P[t]
        assert np.allclose(W[0], w_ref, rtol=1e-12, atol=1e-14)


def test_l2_regularisation_is_a_shifted_gradient():
    """l2: the optimizer sees G + wd W everywhere (Sec. 3.1.2): same trajectory as the
    plain optimizer fed those gradients by hand."""
    r = rng(22)
    shapes = [(9, 7), (5,)]
    grads = [[r.standard_normal(s) * 0.1 for s in shapes] for _ in range(5)]
    wd, lr = 0.2, 0.05
    a = make_opt(shapes, block_size=4, beta2=0.9, precondition_frequency=2, momentum=0.5,
                 weight_decay=wd, use_decoupled_weight_decay=False)
    b = make_opt(shapes, block_size=4, beta2=0.9, precondition_frequency=2, momentum=0.5)
    Wa = [r.standard_normal(s) for s in shapes]
    Wb = [w.copy() for w in Wa]
    for t, g in enumerate(grads):
        a.step(Wa, g, lr, t)
        b.step(Wb, [gi + wd * wi for gi, wi in zip(g, Wb)], lr, t)
        for x, y in zip(Wa, Wb):
            assert np.allclose(x, y, rtol=1e-12, atol=1e-14)


def test_nesterov_is_geometric_sum_plus_current_direction():
    """W_{t+1} = W_t + lr (mu M_t + P_t), M_t = sum_{s<=t} mu^(t-s) P_s (Sec. 3.1.3)."""
    r = rng(23)
    shapes = [(6, 5), (9,)]
    grads = [[r.standard_normal(s) * 0.1 for s in shapes] for _ in range(6)]
    lr, mu = 0.02, 0.7
    plain = make_opt(shapes, precondition_frequency=3)
    W = [np.zeros(s) for s in shapes]
    P = []
    for t, g in enumerate(grads):
        before = [w.copy() for w in W]
        plain.step(W, g, lr, t)
        P.append([(w - b0) / lr for w, b0 in zip(W, before)])
    nes = make_opt(shapes, precondition_frequency=3, momentum=mu, use_nesterov=True)
    Wn = [np.zeros(s) for s in shapes]
    for t, g in enumerate(grads):
        nes.step(Wn, g, lr, t)
    for i in range(len(shapes)):
        expect = np.zeros(shapes[i])
        for t in range(len(grads)):
            M = sum(mu ** (t - s_) * P[s_][i] for s_ in range(t + 1))
            expect += lr * (mu * M + P[t][i])
        assert np.allclose(Wn[i], expect, rtol=1e-10, atol=1e-14)


def test_gradient_filtering_with_a_constant_gradient():
    """Constant full-rank G, beta2 = 1, roots refreshed every step: the filtered gradient is
    (1 - beta1^(t+1)) G, the Shampoo direction of any multiple of G is U V^T, the AdaGrad state
    is (t+1) G^2, so W_T = -lr sqrt(max(m,n)) U V^T sum_t (1 - beta1^(t+1)) / sqrt(t+1)."""
    m, n, b1, lr = 5, 4, 0.8, 0.1
    G = rng(24).standard_normal((m, n))
    U, S, Vt = np.linalg.svd(G, full_matrices=False)
    opt = make_opt([(m, n)], epsilon=1e-14, graft_epsilon=0.0, beta1=b1)
    W = [np.zeros((m, n))]
    coeff = 0.0
    for t in range(5):
        opt.step(W, [G], lr, t)
        coeff += (1 - b1 ** (t + 1)) / np.sqrt(t + 1)
        assert np.allclose(W[0], -lr * np.sqrt(max(m, n)) * coeff * (U @ Vt), rtol=1e-6, atol=1e-9)


def test_gradient_filtering_one_d_textbook():
    """1-D: A from the raw gradient, direction from the filtered one (Sec. 3.1.1)."""
    n, b1, lr, eg = 11, 0.9, 0.01, 1e-10
    r = rng(25)
    opt = make_opt([(n,)], beta1=b1, graft_epsilon=eg)
    W = [np.zeros(n)]
    w = np.zeros(n); a = np.zeros(n); gf = np.zeros(n)
    for t in range(7):
        g = r.standard_normal(n)
        opt.step(W, [g], lr, t)
        for i in range(n):
            a[i] += g[i] * g[i]
            gf[i] = b1 * gf[i] + (1 - b1) * g[i]
            w[i] -= lr * gf[i] / (np.sqrt(a[i]) + eg)
        assert np.allclose(W[0], w, rtol=1e-13, atol=1e-16)


def test_sgd_grafting_step_length_and_polar_first_step():
    """SGD grafting: ||P||_F = ||G||_F per block (Sec. 2.4); at t = 0 with beta2 = 1 the step is
    -lr ||G||_F U V^T / sqrt(min(m, n))."""
    m, n, lr = 6, 4, 0.2
    G = rng(26).standard_normal((m, n))
    U, S, Vt = np.linalg.svd(G, full_matrices=False)
    opt = make_opt([(m, n)], epsilon=1e-14, grafting="sgd")
    W = [np.zeros((m, n))]
    opt.step(W, [G], lr, 0)
    assert np.allclose(W[0], -lr * np.linalg.norm(G) / np.sqrt(min(m, n)) * (U @ Vt), rtol=1e-6, atol=1e-9)
    G2 = rng(27).standard_normal((m, n))
    before = W[0].copy()
    opt.step(W, [G2], lr, 1)
    assert np.isclose(np.linalg.norm(W[0] - before), lr * np.linalg.norm(G2), rtol=1e-10)
    assert np.array_equal(opt.A[0], np.zeros((m, n)))     # no grafting state


def test_bias_correction_undoes_filtering_of_a_constant_gradient():
    """Sec. 3.1.1: Gf / (1 - beta1^(t+1)) of a constant gradient is that gradient, so the
    closed form of the filtering pin loses its (1 - beta1^(t+1)) weights."""
    m, n, b1, lr = 5, 4, 0.8, 0.1
    G = rng(28).standard_normal((m, n))
    U, S, Vt = np.linalg.svd(G, full_matrices=False)
    opt = make_opt([(m, n)], epsilon=1e-14, graft_epsilon=0.0, beta1=b1, use_bias_correction=True)
    W = [np.zeros((m, n))]
    coeff = 0.0
    for t in range(5):
        opt.step(W, [G], lr, t)
        coeff += 1.0 / np.sqrt(t + 1)
        assert np.allclose(W[0], -lr * np.sqrt(max(m, n)) * coeff * (U @ Vt), rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("bc", [False, True])
def test_bias_correction_of_the_factors_diagonal_closed_form(bc):
    """Constant diagonal G = diag(d), beta2 < 1: L_t = (1 - beta2^(t+1)) diag(d^2).  With bias
    correction the root routine sees diag(d^2) at every t, and epsilon (large here, so that the
    order matters) is added after the division."""
    d = np.array([0.5, 1.0, 2.0, 3.0])
    b2, eps = 0.9, 0.5
    opt = make_opt([(4, 4)], beta2=b2, epsilon=eps, use_bias_correction=bc)
    W = [np.zeros((4, 4))]
    for t in range(4):
        opt.step(W, [np.diag(d)], 0.1, t)
        scale = 1.0 if bc else 1.0 - b2 ** (t + 1)
        expect = np.diag((scale * d * d + eps) ** -0.25)
        assert np.allclose(opt.Lbar[0][0], expect, rtol=1e-12, atol=1e-14)
        assert np.allclose(opt.Rbar[0][0], expect, rtol=1e-12, atol=1e-14)
        assert np.allclose(np.diag(opt.L[0][0]), (1.0 - b2 ** (t + 1)) * d * d, rtol=1e-12)   # stored uncorrected


def test_bias_correction_one_d_textbook():
    n, b1, lr, eg = 9, 0.9, 0.01, 1e-10
    r = rng(29)
    opt = make_opt([(n,)], beta1=b1, graft_epsilon=eg, use_bias_correction=True)
    W = [np.zeros(n)]
    w = np.zeros(n); a = np.zeros(n); gf = np.zeros(n)
    for t in range(6):
        g = r.standard_normal(n)
        opt.step(W, [g], lr, t)
        for i in range(n):
            a[i] += g[i] * g[i]
            gf[i] = b1 * gf[i] + (1 - b1) * g[i]
            w[i] -= lr * (gf[i] / (1 - b1 ** (t + 1))) / (np.sqrt(a[i]) + eg)
        assert np.allclose(W[0], w, rtol=1e-13, atol=1e-16)


# ---------------------------------------------------------------------------
# Coupled inverse Newton iteration (Sec. 3.2.1, item 2)
# ---------------------------------------------------------------------------
def wishart(n, k, seed):
    g = rng(seed).standard_normal((n, k))
    return g @ g.T / k


@pytest.mark.parametrize("p", [1, 2, 4])
def test_newton_converges_to_the_spectral_root_inverse(p):
    """On a well-conditioned SPD matrix the iteration ends below its tolerance and X equals
    (A + eps I)^(-1/p) from the eigendecomposition to about tol / p."""
    A = wishart(24, 96, 40 + p)
    eps = 1e-3
    X, k, err = so.root_inverse_newton(A, eps, p, tol=1e-10, max_iterations=200)
    lam, Q = np.linalg.eigh(A)
    exact = (Q * (lam + eps) ** (-1.0 / p)) @ Q.T
    assert err < 1e-10 and 0 < k < 60
    assert np.linalg.norm(X - exact) <= 1e-9 * np.linalg.norm(exact)
    # X^p (A + eps I) = I
    assert np.allclose(np.linalg.matrix_power(X, p) @ (A + eps * np.eye(24)), np.eye(24), atol=1e-8)


def test_newton_scalar_recursion_by_hand():
    """n = 1: c = (2 a / (p + 1))^(1/p), m_0 = (p + 1) / 2 ... the scalar recursion written out."""
    a, p, eps = 3.7, 4, 0.05
    X, k, err = so.root_inverse_newton(np.array([[a]]), eps, p, tol=1e-12, max_iterations=50)
    A = a + eps
    c = (2 * A / (p + 1)) ** (1 / p)
    x, m = 1 / c, A / c ** p
    assert np.isclose(m, (p + 1) / 2)
    steps = 0
    while abs(m - 1) >= 1e-12:
        t = ((p + 1) - m) / p
        x, m = x * t, t ** p * m
        steps += 1
    assert steps == k and np.isclose(X[0, 0], x, rtol=1e-14) and np.isclose(x, A ** (-1 / p), rtol=1e-11)


def test_newton_iteration_cap_and_diagonal_input():
    """A diagonal matrix stays diagonal and every entry follows its own scalar recursion from the
    common c; with a cap of 3 steps exactly 3 are taken."""
    d = np.array([0.2, 1.0, 5.0])
    p = 2
    X, k, err = so.root_inverse_newton(np.diag(d), 0.0, p, tol=1e-30, max_iterations=3)
    assert k == 3
    c = (2 * np.sqrt(np.sum(d * d)) / (p + 1)) ** (1 / p)
    x, m = np.full(3, 1 / c), d / c ** p
    for _ in range(3):
        t = ((p + 1) - m) / p
        x, m = x * t, t ** p * m
    assert np.allclose(X, np.diag(x), rtol=1e-14, atol=1e-300)
    assert np.isclose(err, np.max(np.abs(m - 1)))


def test_optimizer_with_newton_roots_matches_eigh_roots_when_well_conditioned():
    """Same optimizer, two root routines: on well-conditioned factors (wide blocks, visible
    epsilon) the trajectories agree to the Newton tolerance."""
    shapes = [(8, 40), (12,)]
    kw = dict(block_size=64, beta2=0.99, epsilon=1e-3, precondition_frequency=2, momentum=0.9)
    a = make_opt(shapes, **kw)
    b = make_opt(shapes, root_method="newton", newton_tolerance=1e-10, **kw)
    Wa = [np.zeros(s) for s in shapes]
    Wb = [np.zeros(s) for s in shapes]
    for t in range(5):
        g = [rng(50 + t).standard_normal(s) for s in shapes]
        a.step(Wa, g, 0.1, t)
        b.step(Wb, g, 0.1, t)
    assert np.allclose(Wa[0], Wb[0], rtol=1e-7, atol=1e-10)
    assert np.allclose(a.Rbar[0][0], b.Rbar[0][0], rtol=1e-7, atol=1e-9)


# ---------------------------------------------------------------------------
# RMSprop / Adam grafting (Sec. 2.2 EMA equation, Sec. 2.4)
# ---------------------------------------------------------------------------
def test_adam_grafting_on_a_vector_is_textbook_adam():
    """1-D parameter, Adam grafting, beta1 filtering, bias correction: the update is Adam's,
    w -= lr * mhat / (sqrt(vhat) + eps), written out with scalars."""
    n, b1, b2, lr, eg = 7, 0.9, 0.99, 0.01, 1e-8
    r = rng(70)
    opt = make_opt([(n,)], beta1=b1, graft_epsilon=eg, grafting="adam", grafting_beta2=b2,
                   use_bias_correction=True)
    W = [np.zeros(n)]
    w = np.zeros(n); m = np.zeros(n); v = np.zeros(n)
    for t in range(6):
        g = r.standard_normal(n)
        opt.step(W, [g], lr, t)
        for i in range(n):
            m[i] = b1 * m[i] + (1 - b1) * g[i]
            v[i] = b2 * v[i] + (1 - b2) * g[i] * g[i]
            w[i] -= lr * (m[i] / (1 - b1 ** (t + 1))) / (np.sqrt(v[i] / (1 - b2 ** (t + 1))) + eg)
        assert np.allclose(W[0], w, rtol=1e-13, atol=1e-16)


def test_rmsprop_grafting_on_a_vector_is_textbook_rmsprop():
    n, b2, lr, eg = 5, 0.9, 0.05, 1e-8
    r = rng(71)
    opt = make_opt([(n,)], graft_epsilon=eg, grafting="rmsprop", grafting_beta2=b2, use_bias_correction=True)
    W = [np.zeros(n)]
    w = np.zeros(n); v = np.zeros(n)
    for t in range(5):
        g = r.standard_normal(n)
        opt.step(W, [g], lr, t)
        v = b2 * v + (1 - b2) * g * g          # no bias correction for RMSprop
        w = w - lr * g / (np.sqrt(v) + eg)
        assert np.allclose(W[0], w, rtol=1e-13, atol=1e-16)


def test_rmsprop_grafting_sets_the_block_step_length():
    """2-D block: the step has the Frobenius norm of the RMSprop direction of that block and the
    orientation of the Shampoo direction (Sec. 2.4); at t = 0 with beta2 = 1: U V^T."""
    m, n, b2, lr = 5, 4, 0.5, 0.3
    G = rng(72).standard_normal((m, n))
    U, S, Vt = np.linalg.svd(G, full_matrices=False)
    opt = make_opt([(m, n)], epsilon=1e-14, graft_epsilon=0.0, grafting="rmsprop", grafting_beta2=b2)
    W = [np.zeros((m, n))]
    opt.step(W, [G], lr, 0)
    # A_0 = (1 - b2) G^2, so P_graft = sign(G) / sqrt(1 - b2) and ||P_graft||_F = sqrt(m n / (1 - b2))
    expect = -lr * np.sqrt(m * n / (1 - b2)) / np.sqrt(min(m, n)) * (U @ Vt)
    assert np.allclose(W[0], expect, rtol=1e-6, atol=1e-9)
    assert np.allclose(opt.A[0], (1 - b2) * G * G)


# ---------------------------------------------------------------------------
# Large-dimension methods other than blocking (Sec. 4.2.2, 4.2.3)
# ---------------------------------------------------------------------------
def test_adagrad_large_dim_method_is_the_flattened_diagonal_method():
    """A matrix with a dimension above the block size under "adagrad" steps exactly like the
    1-D parameter made of its entries; a matrix within the block size is untouched by the option."""
    shapes = [(6, 3), (3, 3)]
    a = make_opt(shapes, block_size=4, large_dim_method="adagrad", momentum=0.5)
    b = make_opt([(18,), (3, 3)], block_size=4, momentum=0.5)
    Wa = [np.zeros(s) for s in shapes]
    Wb = [np.zeros(18), np.zeros((3, 3))]
    for t in range(4):
        g = [rng(90 + t).standard_normal(s) for s in shapes]
        a.step(Wa, g, 0.1, t)
        b.step(Wb, [g[0].reshape(-1), g[1]], 0.1, t)
    assert np.array_equal(Wa[0].reshape(-1), Wb[0]) and np.array_equal(Wa[1], Wb[1])


def test_diagonal_shampoo_both_dimensions_by_hand():
    """Both dimensions above the block size, beta2 = 1, one step: l_i = sum_j G_ij^2,
    r_j = sum_i G_ij^2, P_sh_ij = (l_i + eps)^(-1/4) G_ij (r_j + eps)^(-1/4); loops written out."""
    m, n, eps, lr = 5, 6, 1e-3, 0.1
    G = rng(95).standard_normal((m, n))
    opt = make_opt([(m, n)], block_size=4, epsilon=eps, large_dim_method="diagonal")
    W = [np.zeros((m, n))]
    opt.step(W, [G], lr, 0)
    l = [sum(G[i, j] ** 2 for j in range(n)) for i in range(m)]
    r = [sum(G[i, j] ** 2 for i in range(m)) for j in range(n)]
    P = np.array([[(l[i] + eps) ** -0.25 * G[i, j] * (r[j] + eps) ** -0.25 for j in range(n)] for i in range(m)])
    graft = np.sqrt(m * n)            # AdaGrad graft of the first step is sign(G) (eps_g tiny)
    assert np.allclose(W[0], -lr * graft * P / np.linalg.norm(P), rtol=1e-8)
    assert np.allclose(opt.L[0][0], l) and np.allclose(opt.R[0][0], r)


@pytest.mark.parametrize("shape,dl,dr", [((7, 3), True, False), ((3, 7), False, True)])
def test_diagonal_shampoo_mixed_equals_full_shampoo_on_diagonalised_factor(shape, dl, dr):
    """One dimension above the block size: the step equals the full two-factor formula with that
    factor replaced by its diagonal (Sec. 4.2.3), the other factor being the usual full one."""
    m, n = shape
    eps = 1e-4
    opt = make_opt([shape], block_size=4, epsilon=eps, beta2=0.9, large_dim_method="diagonal", precondition_frequency=1)
    W = [np.zeros(shape)]
    L = np.zeros((m, m)); R = np.zeros((n, n)); A = np.zeros(shape)
    for t in range(3):
        G = rng(96 + t).standard_normal(shape)
        before = W[0].copy()
        opt.step(W, [G], 0.1, t)
        L = 0.9 * L + 0.1 * G @ G.T
        R = 0.9 * R + 0.1 * G.T @ G
        A = A + G * G
        Lm = np.diag(np.diag(L)) if dl else L
        Rm = np.diag(np.diag(R)) if dr else R
        lam, Q = np.linalg.eigh(Lm); Li = (Q * (lam + eps) ** -0.25) @ Q.T
        lam, Q = np.linalg.eigh(Rm); Ri = (Q * (lam + eps) ** -0.25) @ Q.T
        Psh = Li @ G @ Ri
        Pg = G / (np.sqrt(A) + 1e-10)
        expect = -0.1 * np.linalg.norm(Pg) * Psh / np.linalg.norm(Psh)
        assert np.allclose(W[0] - before, expect, rtol=1e-9, atol=1e-12)


def test_diagonal_method_leaves_small_matrices_alone():
    shapes = [(4, 3)]
    a = make_opt(shapes, block_size=4, large_dim_method="diagonal")
    b = make_opt(shapes, block_size=4)
    Wa, Wb = [np.zeros((4, 3))], [np.zeros((4, 3))]
    for t in range(3):
        g = [rng(99 + t).standard_normal((4, 3))]
        a.step(Wa, g, 0.1, t); b.step(Wb, g, 0.1, t)
    assert np.array_equal(Wa[0], Wb[0])


# ---------------------------------------------------------------------------
# merging and tensors of order w (Sec. 2.3, Sec. 4.2.1)
# ---------------------------------------------------------------------------
def test_merging_worked_example_of_the_paper():
    """Sec. 4.2.1: with maximum dimension 8 a 10 x 2 x 2 x 4 tensor becomes 10 x 4 x 4
    (tests/golden/merge_dims.txt holds the example and a few consequences of the rule)."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "merge_dims.txt")
    rows = [ln.split("#")[0].split() for ln in open(path) if ln.split("#")[0].strip()]
    assert len(rows) >= 5
    for b, shape, merged in rows:
        shape = tuple(int(x) for x in shape.split("x"))
        merged = tuple(int(x) for x in merged.split("x"))
        assert so.merge_dims(shape, int(b)) == merged, (b, shape)
        assert int(np.prod(merged)) == int(np.prod(shape))      # a view: no element added or lost


def test_tensor_blocks_tile_the_tensor_exactly_once():
    shape, b = (5, 3, 7), 3
    seen = np.zeros(shape, dtype=int)
    blks = so.tensor_block_partition(shape, b)
    assert len(blks) == 2 * 1 * 3
    for starts, dims in blks:
        assert all(1 <= d <= b for d in dims)
        seen[tuple(slice(s0, s0 + d) for s0, d in zip(starts, dims))] += 1
    assert (seen == 1).all()
    # row-major order of the block indices: the last dimension moves fastest
    assert [st for st, _ in blks[:3]] == [(0, 0, 0), (0, 0, 3), (0, 0, 6)]


def test_order3_factors_and_direction_against_explicit_loops_and_kronecker():
    """L_k = G_(k) G_(k)^T written as explicit sums, and the mode products against the
    Kronecker form: vec(G x_1 X1 x_2 X2 x_3 X3) = (X1 kron X2 kron X3) vec(G), row-major vec."""
    r = rng(70)
    d = (3, 4, 2)
    G = r.standard_normal(d)
    Ls = so.tensor_factor_update([np.zeros((n, n)) for n in d], G, 1.0)
    L1 = np.zeros((3, 3)); L2 = np.zeros((4, 4)); L3 = np.zeros((2, 2))
    for i in range(3):
        for j in range(4):
            for k in range(2):
                for a in range(3):
                    L1[i, a] += G[i, j, k] * G[a, j, k]
                for a in range(4):
                    L2[j, a] += G[i, j, k] * G[i, a, k]
                for a in range(2):
                    L3[k, a] += G[i, j, k] * G[i, j, a]
    for got, want in zip(Ls, (L1, L2, L3)):
        assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    # EMA form
    Ls2 = so.tensor_factor_update(Ls, G, 0.9)
    assert np.allclose(Ls2[1], 0.9 * L2 + 0.1 * L2, rtol=1e-13)
    Xs = [r.standard_normal((n, n)) for n in d]
    Xs = [x + x.T for x in Xs]
    P = so.tensor_shampoo_direction(Xs, G)
    K = np.kron(np.kron(Xs[0], Xs[1]), Xs[2])
    assert np.allclose(P.reshape(-1), K @ G.reshape(-1), rtol=1e-12, atol=1e-12)
    # and the inverse-root form of the preconditioner: (L1 kron L2 kron L3)^(-1/6) vec(G)
    eps = 1e-3
    roots = [so.root_inverse(L, eps, 1.0 / 6.0)[0] for L in Ls]
    big = np.kron(np.kron(Ls[0] + eps * np.eye(3), Ls[1] + eps * np.eye(4)), Ls[2] + eps * np.eye(2))
    lam, Q = np.linalg.eigh(big)
    want = (Q * lam ** (-1.0 / 6.0)) @ Q.T @ G.reshape(-1)
    assert np.allclose(so.tensor_shampoo_direction(roots, G).reshape(-1), want, rtol=1e-9, atol=1e-12)


def test_order3_step_on_a_rank_one_tensor_has_a_closed_form():
    """G = a o b o c: every factor is ||G||^2 times a projector, so with exponent 1/(2w) = 1/6
    per dimension the Shampoo direction is G / sqrt(||G||^2 + eps): any other exponent shows."""
    r = rng(71)
    a, b_, c = r.standard_normal(5), r.standard_normal(4), r.standard_normal(6)
    G = np.einsum("i,j,k->ijk", a, b_, c)
    eps = 1e-4
    o = so.ShampooOracle([(5, 4, 6)], 8, 1.0, eps, 0.25, 1, momentum=0.0, grafting="sgd")
    assert 0 in o.tblocks and o.view_shapes[0] == (5, 4, 6)
    W = [np.zeros((5, 4, 6))]
    o.step(W, [G], 1.0, 0)
    g2 = float(np.sum(G * G))
    assert np.allclose(o.P_sh[0][0], G / np.sqrt(g2 + eps), rtol=1e-9, atol=1e-12)
    # SGD grafting: the step has the length of the gradient, the direction of P_shampoo (= that of G)
    assert np.allclose(W[0], -G, rtol=1e-9, atol=1e-12)
    # the three roots individually: (L_k + eps I)^(-1/6) a_k = (||G||^2 + eps)^(-1/6) a_k
    for k, v in enumerate((a, b_, c)):
        assert np.allclose(o.TLbar[0][0][k] @ v, (g2 + eps) ** (-1.0 / 6.0) * v, rtol=1e-9)


def test_order4_step_on_a_rank_one_tensor_has_a_closed_form():
    """G = a o b o c o d (order w = 4): every factor is ||G||^2 times a projector, so with the
    exponent 2 r / w = 1 / (2 w) = 1/8 per dimension (Sec. 2.3: "root 2w") the four roots together
    give G / sqrt(||G||^2 + eps), and each root alone scales its own vector by
    (||G||^2 + eps)^(-1/8).  An exponent of 1/6 or 1/4 per dimension shows in both."""
    r = rng(75)
    vs = [r.standard_normal(n) for n in (3, 4, 2, 5)]
    G = np.einsum("i,j,k,l->ijkl", *vs)
    eps = 1e-4
    o = so.ShampooOracle([(3, 4, 2, 5)], 5, 1.0, eps, 0.25, 1, momentum=0.0, grafting="sgd")
    assert 0 in o.tblocks and o.view_shapes[0] == (3, 4, 2, 5)     # nothing merges at block size 5
    W = [np.zeros((3, 4, 2, 5))]
    o.step(W, [G], 1.0, 0)
    g2 = float(np.sum(G * G))
    assert np.allclose(o.P_sh[0][0], G / np.sqrt(g2 + eps), rtol=1e-9, atol=1e-12)
    assert not np.allclose(o.P_sh[0][0], G * (g2 + eps) ** (-4.0 / 6.0), rtol=1e-3)
    for k, v in enumerate(vs):
        assert np.allclose(o.TLbar[0][0][k] @ v, (g2 + eps) ** (-1.0 / 8.0) * v, rtol=1e-9)
    assert np.allclose(W[0], -G, rtol=1e-9, atol=1e-12)


def test_order4_factors_and_direction_against_explicit_loops_and_kronecker():
    """Order 4: L_k = G_(k) G_(k)^T as explicit sums for every mode, and the direction of a full
    step against ((L1 + eps I) kron ... kron (L4 + eps I))^(-1/8) vec(G), row-major vec."""
    r = rng(76)
    d = (2, 3, 2, 3)
    G = r.standard_normal(d)
    Ls = so.tensor_factor_update([np.zeros((n, n)) for n in d], G, 1.0)
    want = [np.zeros((n, n)) for n in d]
    for idx in np.ndindex(*d):
        for mode in range(4):
            for a in range(d[mode]):
                jdx = list(idx); jdx[mode] = a
                want[mode][idx[mode], a] += G[idx] * G[tuple(jdx)]
    for got, w_ in zip(Ls, want):
        assert np.allclose(got, w_, rtol=1e-13, atol=1e-13)
    eps = 1e-3
    o = so.ShampooOracle([d], 3, 1.0, eps, 0.25, 1, momentum=0.0, grafting="sgd")
    o.step([np.zeros(d)], [G], 1.0, 0)
    big = np.eye(1)
    for L in want:
        big = np.kron(big, L + eps * np.eye(L.shape[0]))
    lam, Q = np.linalg.eigh(big)
    direction = (Q * lam ** (-1.0 / 8.0)) @ Q.T @ G.reshape(-1)
    assert np.allclose(o.P_sh[0][0].reshape(-1), direction, rtol=1e-9, atol=1e-12)


def test_fully_merged_tensor_is_full_matrix_adagrad():
    """Everything merged: Shampoo on a vector, one factor sum g g^T with exponent 1/2
    (Sec. 4.2.1).  After one gradient (L + eps I)^(-1/2) g = g / sqrt(||g||^2 + eps); after two,
    the direction is checked against the explicit matrix inverse square root."""
    r = rng(72)
    shape = (2, 3, 2)                    # 12 <= b = 16: merges to a vector of 12
    eps = 1e-6
    o = so.ShampooOracle([shape], 16, 1.0, eps, 0.25, 1, momentum=0.0, grafting="sgd")
    assert o.view_shapes[0] == (12,) and 0 in o.tblocks
    W = [np.zeros(shape)]
    g0 = r.standard_normal(shape)
    o.step(W, [g0], 1.0, 0)
    assert np.allclose(o.P_sh[0][0].reshape(-1), g0.reshape(-1) / np.sqrt(np.sum(g0 * g0) + eps), rtol=1e-9)
    g1 = r.standard_normal(shape)
    o.step(W, [g1], 1.0, 1)
    L = np.outer(g0.reshape(-1), g0.reshape(-1)) + np.outer(g1.reshape(-1), g1.reshape(-1)) + eps * np.eye(12)
    lam, Q = np.linalg.eigh(L)
    want = (Q / np.sqrt(lam)) @ Q.T @ g1.reshape(-1)
    assert np.allclose(o.P_sh[0][0].reshape(-1), want, rtol=1e-8, atol=1e-12)


def test_tensor_that_merges_to_a_matrix_runs_the_matrix_case():
    """(6, 5, 2) with b = 10 merges to (6, 10) and must follow exactly the trajectory of the
    6 x 10 matrix (merging is only a view); (6, 2, 2, 5) merges to (6, 4, 5) and stays a tensor."""
    assert so.merge_dims((6, 2, 2, 5), 10) == (6, 4, 5)
    r = rng(73)
    kw = dict(momentum=0.9, beta1=0.9, weight_decay=0.01, use_nesterov=True)
    o3 = so.ShampooOracle([(6, 5, 2)], 10, 0.99, 1e-8, 0.25, 2, **kw)
    o2 = so.ShampooOracle([(6, 10)], 10, 0.99, 1e-8, 0.25, 2, **kw)
    assert o3.view_shapes[0] == (6, 10) and 0 not in o3.tblocks
    w0 = r.standard_normal((6, 5, 2))
    W3, W2 = [w0.copy()], [w0.reshape(6, 10).copy()]
    for t in range(4):
        g = r.standard_normal((6, 5, 2))
        o3.step(W3, [g], 0.05, t)
        o2.step(W2, [g.reshape(6, 10)], 0.05, t)
    assert np.array_equal(W3[0].reshape(6, 10), W2[0])


def test_order3_blocks_are_independent_and_heuristics_apply_per_block():
    """A 4 x 6 x 4 tensor cut with b = 4 into two blocks along the middle dimension behaves as
    the separate 4 x 4 x 4 and 4 x 2 x 4 tensors (same hyper-parameters)."""
    r = rng(74)
    kw = dict(momentum=0.5, weight_decay=0.02, grafting="adagrad")
    whole = so.ShampooOracle([(4, 6, 4)], 4, 0.9, 1e-6, 0.25, 1, **kw)
    parts = so.ShampooOracle([(4, 4, 4), (4, 2, 4)], 4, 0.9, 1e-6, 0.25, 1, **kw)
    assert [d for _, d in whole.tblocks[0]] == [(4, 4, 4), (4, 2, 4)]
    w0 = r.standard_normal((4, 6, 4))
    Ww = [w0.copy()]
    Wp = [np.ascontiguousarray(w0[:, :4, :]), np.ascontiguousarray(w0[:, 4:, :])]
    for t in range(3):
        g = r.standard_normal((4, 6, 4))
        whole.step(Ww, [g], 0.1, t)
        parts.step(Wp, [np.ascontiguousarray(g[:, :4, :]), np.ascontiguousarray(g[:, 4:, :])], 0.1, t)
    assert np.allclose(Ww[0][:, :4, :], Wp[0], rtol=1e-12, atol=1e-14)
    assert np.allclose(Ww[0][:, 4:, :], Wp[1], rtol=1e-12, atol=1e-14)
