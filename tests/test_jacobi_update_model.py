"""A numpy model of the index algebra of the blocked eigensolver's W update
(blockjac_apply_w_kernel): each wavefront carries 16 rows of C = J_k^T X J_l through two chained
16x16x4 float64 matrix-core products without exchanging data with the other wavefronts.  The
model states the operand and result layout of the instruction as the kernel uses it and checks
that the kernel's choice of operands, its order of the k index in the second product and its
placement of the results give J_k^T X J_l.  CPU only: the kernel itself is checked on the GPU
through the root-inverse parity tests."""
import numpy as np


def mfma_f64_16x16x4(a, b, c):
    """D = A B + C for one wavefront: lane l supplies A(l % 16, l // 16) and B(l // 16, l % 16);
    element v of lane l of the result is D(l // 16 + 4 v, l % 16)."""
    A = np.zeros((16, 4)); B = np.zeros((4, 16))
    for lane in range(64):
        A[lane % 16, lane // 16] = a[lane]
        B[lane // 16, lane % 16] = b[lane]
    D = A @ B
    out = c.copy()
    for lane in range(64):
        for v in range(4):
            out[lane, v] += D[lane // 16 + 4 * v, lane % 16]
    return out


def jl_row_in_lds(i):
    """Row i of J_l is kept at this row of the LDS copy (within its group of 16 rows)."""
    return (i & ~15) + 4 * (i & 3) + ((i & 15) >> 2)


def w_update_by_wavefronts(X, Jk, Jl):
    Jl_lds = np.zeros_like(Jl)
    for i in range(64):
        Jl_lds[jl_row_in_lds(i)] = Jl[i]
    C = np.zeros((64, 64))
    for wave in range(4):
        li = np.arange(64) % 16
        lg = np.arange(64) // 16
        # first product: T^T = X^T J_k on the wavefront's 16 columns of J_k, four tiles t over kk
        t1 = [np.zeros((64, 4)) for _ in range(4)]
        for q in range(16):
            b = Jk[4 * q + lg, 16 * wave + li]
            for t in range(4):
                a = X[4 * q + lg, 16 * t + li]
                t1[t] = mfma_f64_16x16x4(a, b, t1[t])
        # second product: the accumulators are the A operand as they stand; step (t, v) reads
        # LDS row 16 t + 4 g + v of J_l, which holds row 16 t + g + 4 v
        c2 = [np.zeros((64, 4)) for _ in range(4)]
        for t in range(4):
            for v in range(4):
                a = t1[t][:, v]
                for u in range(4):
                    b = Jl_lds[16 * t + 4 * lg + v, 16 * u + li]
                    c2[u] = mfma_f64_16x16x4(a, b, c2[u])
        for u in range(4):
            for lane in range(64):
                for v in range(4):
                    C[16 * wave + lane // 16 + 4 * v, 16 * u + lane % 16] = c2[u][lane, v]
    return C


def test_chained_products_give_the_two_sided_rotation():
    rng = np.random.default_rng(5)
    X, Jk, Jl = (rng.standard_normal((64, 64)) for _ in range(3))
    C = w_update_by_wavefronts(X, Jk, Jl)
    ref = Jk.T @ X @ Jl
    assert np.abs(C - ref).max() <= 1e-12 * np.abs(ref).max()


def test_lds_row_permutation_is_an_involution_within_groups_of_16():
    rows = [jl_row_in_lds(i) for i in range(64)]
    assert sorted(rows) == list(range(64))
    assert all(jl_row_in_lds(r) == i for i, r in enumerate(rows))
    assert all(r // 16 == i // 16 for i, r in enumerate(rows))


def test_a_wrong_result_layout_is_caught():
    """With the rows of the result taken as 4 (lane // 16) + v instead of lane // 16 + 4 v (the
    layout of the 32-bit instruction of the same shape) the chained form does not give the
    product: the model tells the two apart."""
    rng = np.random.default_rng(6)
    X, Jk, Jl = (rng.standard_normal((64, 64)) for _ in range(3))
    C = w_update_by_wavefronts(X, Jk, Jl)
    wrong = np.zeros_like(C)
    for wave in range(4):
        for g in range(4):
            for v in range(4):
                wrong[16 * wave + 4 * g + v] = C[16 * wave + g + 4 * v]
    ref = Jk.T @ X @ Jl
    assert np.abs(wrong - ref).max() > 1e-3
