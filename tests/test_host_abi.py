"""Host-side tests of libshampoo (no GPU): the library loads, exports every
symbol the header declares, validates configurations, and its block planner
agrees with the blocking rule of Sec. 4.2.1 as written out in the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import shampoo_oracle as so
from paper_2309_06497_amd import binding as B
from paper_2309_06497_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def cfg_for(shapes, b, **kw):
    args = dict(beta2=0.999, epsilon=1e-12, root_exponent=0.25, precondition_frequency=10)
    args.update(kw)
    return B.make_config(shapes, b, **args)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "shampoo.h")).read()
    declared = set(re.findall(r"\b(shampoo_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert L.shampoo_strerror(0) == b"success"
    assert L.shampoo_strerror(-4).startswith(b"workspace")


@pytest.mark.parametrize("name,shapes,b", [
    ("tiny", wl.tiny_shapes(), 64),
    ("uniform", wl.uniform_shapes(), 128),
    ("resnet50", wl.resnet50_shapes(), 128),
    ("transformer", wl.transformer_shapes(), 1024),
    ("ragged", [(5, 7), (3,), (130, 257), (1, 1)], 128),
])
def test_planner_matches_blocking_rule(name, shapes, b):
    cfg = cfg_for(shapes, b)
    table, n_buckets = B.shampoo_plan(cfg)
    expect = []
    for i, s in enumerate(shapes):
        if len(s) == 2:
            expect += [(i, r0, c0, m, n) for (r0, c0, m, n) in so.block_partition(s[0], s[1], b)]
    assert [tuple(int(x) for x in row[:5]) for row in table] == expect
    # buckets: equal (m, n) share a bucket, slots count up inside it in table order
    seen = {}
    for row in table:
        key = (int(row[3]), int(row[4]))
        bucket, slot = int(row[5]), int(row[6])
        if key not in seen:
            seen[key] = [bucket, 0]
        assert seen[key][0] == bucket and seen[key][1] == slot
        seen[key][1] += 1
    assert len(seen) == n_buckets
    assert len({v[0] for v in seen.values()}) == n_buckets


def test_planner_histograms_of_the_named_workloads():
    t, nb = B.shampoo_plan(cfg_for(wl.tiny_shapes(), 64))
    assert len(t) == 8 and nb == 1 and set(map(tuple, t[:, 3:5])) == {(64, 64)}
    t, nb = B.shampoo_plan(cfg_for(wl.uniform_shapes(), 128))
    assert len(t) == 512 and nb == 1
    t, nb = B.shampoo_plan(cfg_for(wl.resnet50_shapes(), 128))
    assert len(t) == 1576 and nb == 6
    t, nb = B.shampoo_plan(cfg_for(wl.transformer_shapes(), 1024))
    assert len(t) == 1152 and nb == 1


def test_workspace_holds_the_state_of_the_memory_rule():
    """Sec. 4.2.1: blocked Shampoo on a matrix stores 4 d1 d2 numbers (factors and
    roots) when b divides both dimensions; plus A, M, the direction scratch."""
    d1, d2, b = 512, 384, 128
    cfg = cfg_for([(d1, d2)], b, momentum=0.9)
    nbytes = B.shampoo_workspace_bytes(cfg)
    state = 4 * d1 * d2 + 2 * d1 * d2      # factors + roots, A + M
    scratch = 2 * d1 * d2                   # P and T
    assert nbytes >= 4 * (state + scratch)
    assert nbytes < 4 * (state + scratch) * 1.02 + (1 << 16)
    # the transformer workload fits one MI355X (288 GB) with room to spare
    big = B.shampoo_workspace_bytes(cfg_for(wl.transformer_shapes(), 1024, momentum=0.9))
    assert 35e9 < big < 60e9


@pytest.mark.parametrize("kw,code", [
    (dict(beta2=0.0), -3), (dict(beta2=1.5), -3), (dict(epsilon=0.0), -3), (dict(epsilon=-1.0), -3),
    (dict(root_exponent=0.0), -3), (dict(precondition_frequency=0), -3),
    (dict(start_preconditioning_step=-1), -3), (dict(graft_epsilon=-1.0), -3),
    (dict(momentum=1.0), -3), (dict(momentum=-0.1), -3), (dict(grad_dtype=7), -3),
    (dict(beta1=1.0), -3), (dict(beta1=-0.5), -3), (dict(weight_decay=-1.0), -3), (dict(grafting_type=5), -3),
    (dict(grafting_type=B.GRAFT_ADAM, grafting_beta2=0.0), -3), (dict(grafting_type=B.GRAFT_RMSPROP, grafting_beta2=1.5), -3),
    (dict(large_dim_method=3), -3), (dict(precond_matrix_cores=2), -3), (dict(root_method=3), -3), (dict(root_method=B.ROOT_NEWTON, newton_tolerance=-1.0), -3),
    (dict(root_method=B.ROOT_NEWTON, newton_max_iterations=5000), -3),
    (dict(root_method=B.ROOT_NEWTON, root_exponent=1.0 / 3.0), -7),
])
def test_bad_hyperparameters_are_rejected(kw, code):
    cfg = cfg_for([(8, 8)], 4, **kw)
    assert B.lib().shampoo_plan(ctypes.byref(cfg), None, 0, None, None) == code
    assert B.shampoo_workspace_bytes(cfg) == 0


def test_bad_shapes_are_rejected():
    L = B.lib()
    assert L.shampoo_plan(None, None, 0, None, None) == -1
    assert L.shampoo_plan(ctypes.byref(cfg_for([(8, 0)], 4)), None, 0, None, None) == -2
    assert L.shampoo_plan(ctypes.byref(cfg_for([(0,)], 4)), None, 0, None, None) == -2
    assert L.shampoo_plan(ctypes.byref(cfg_for([(8, 8)], 0)), None, 0, None, None) == -2
    assert L.shampoo_plan(ctypes.byref(cfg_for([(8, 8)], 100000)), None, 0, None, None) == -7
    cfg = cfg_for([(8, 8)], 4)
    cfg.n_params = 0
    assert L.shampoo_plan(ctypes.byref(cfg), None, 0, None, None) == -2
    cfg = cfg_for([(8, 8)], 4)
    cfg._keep[0][0] = 5             # ndim 5
    assert L.shampoo_plan(ctypes.byref(cfg), None, 0, None, None) == -2
    assert L.shampoo_plan(ctypes.byref(cfg_for([(8, 8, 0)], 4)), None, 0, None, None) == -2
    # four dimensions that do not merge are planned as a tensor of order 4 ...
    assert L.shampoo_plan(ctypes.byref(cfg_for([(8, 8, 8, 8)], 4)), None, 0, None, None) == 0
    # ... unless one block would pass 2^30 elements
    assert L.shampoo_plan(ctypes.byref(cfg_for([(256, 256, 256, 256)], 200)), None, 0, None, None) == -7
    # coupled Newton needs 1 / exponent in {1, 2, 4, 8}: an order-3 tensor would need 6
    assert L.shampoo_plan(ctypes.byref(cfg_for([(8, 8, 8)], 4, root_method=B.ROOT_NEWTON)), None, 0, None, None) == -7
    # a table pointer is required when cap > 0
    assert L.shampoo_plan(ctypes.byref(cfg_for([(8, 8)], 4)), None, 3, None, None) == -1
    # null handles
    assert L.shampoo_step(None, None, None, 0.1, 0, None) == -1
    assert L.shampoo_destroy(None) == -1
    assert L.shampoo_get(None, 0, 0, 0, None, 0, None) == -1
    assert L.shampoo_root_inverse_workspace_bytes(0, 1) == 0
    assert L.shampoo_root_inverse_workspace_bytes(1024, 4) > 2 * 4 * 1024 * 1024 * 4
    assert L.shampoo_root_inverse_newton_workspace_bytes(0, 1) == 0
    assert L.shampoo_root_inverse_newton_workspace_bytes(1024, 4) >= 7 * 4 * 1024 * 1024 * 4
    assert L.shampoo_root_inverse_newton(None, 8, 1, 1e-6, 4, 1e-6, 10, None, None, None, None, 0, None) == -1
    out = ctypes.c_void_p()
    # create checks the workspace before touching any device
    assert L.shampoo_create(ctypes.byref(cfg_for([(8, 8)], 4)), None, 0, None, ctypes.byref(out)) == -4
    assert L.shampoo_create(ctypes.byref(cfg_for([(8, 8)], 4)), None, 0, None, None) == -1


def test_planner_large_dimension_methods():
    """Sec. 4.2.2 / 4.2.3: under "adagrad" a matrix above the block size leaves the block table,
    under "diagonal" it stays whole with flags for its diagonalised sides."""
    shapes = [(600, 48), (40, 264), (300, 200), (64, 64), (9,)]
    t, nb = B.shampoo_plan(cfg_for(shapes, 128, large_dim_method=B.LARGE_DIM_ADAGRAD))
    assert [tuple(int(x) for x in r[:5]) for r in t] == [(3, 0, 0, 64, 64)] and nb == 1
    t, nb = B.shampoo_plan(cfg_for(shapes, 128, large_dim_method=B.LARGE_DIM_DIAGONAL))
    assert [(int(r[0]), int(r[3]), int(r[4]), int(r[7])) for r in t] == [
        (0, 600, 48, 1), (1, 40, 264, 2), (2, 300, 200, 3), (3, 64, 64, 0)]
    assert nb == 4
    # diagonal Shampoo stores d1 + d2 numbers per factor pair instead of d1^2 + d2^2 (Sec. 4.2.3)
    big = [(100000, 64)]
    blocked = B.shampoo_workspace_bytes(cfg_for(big, 1024, momentum=0.9))
    diag = B.shampoo_workspace_bytes(cfg_for(big, 1024, momentum=0.9, large_dim_method=B.LARGE_DIM_DIAGONAL))
    assert diag < blocked - 2 * 97 * 1024 * 1024 * 4


def test_planner_merges_small_dimensions_and_blocks_tensors():
    """Sec. 4.2.1: merging (the same cases as tests/golden/merge_dims.txt, seen through the
    planner) and blocking of what stays a tensor; block order and the oracle's partition agree."""
    from oracle import shampoo_oracle as so
    # merges to a matrix: blocked like the matrix
    t, nb = B.shampoo_plan(cfg_for([(256, 64, 1, 1)], 128))
    assert [tuple(int(x) for x in r[:5]) for r in t] == [(0, 0, 0, 128, 64), (0, 128, 0, 128, 64)]
    assert all(int(r[7]) == 0 and int(r[9]) == 1 for r in t)
    # stays of order 3: (64, 64, 3, 3) -> (64, 64, 9), one block
    t, nb = B.shampoo_plan(cfg_for([(64, 64, 3, 3)], 128))
    assert [tuple(int(x) for x in r) for r in t] == [(0, 0, 0, 64, 64, 0, 0, 4 | 3 << 4, 0, 9, 0, 1)]
    # everything merges: one factor (full-matrix AdaGrad), block len x 1 x 1
    t, nb = B.shampoo_plan(cfg_for([(2, 3, 2)], 16))
    assert [tuple(int(x) for x in r) for r in t] == [(0, 0, 0, 12, 1, 0, 0, 4 | 1 << 4, 0, 1, 0, 1)]
    # blocking of a tensor, against the oracle's partition (row-major order of block indices)
    shape, b = (10, 7, 5), 4
    t, nb = B.shampoo_plan(cfg_for([shape], b))
    want = so.tensor_block_partition(so.merge_dims(shape, b), b)
    got = [((int(r[1]), int(r[2]), int(r[8])), (int(r[3]), int(r[4]), int(r[9]))) for r in t]
    assert got == want and all(int(r[7]) == 4 | 3 << 4 for r in t)
    # order 4: four dimensions that do not merge, cut in every dimension
    shape, b = (9, 6, 5, 7), 4
    t, nb = B.shampoo_plan(cfg_for([shape], b))
    assert so.merge_dims(shape, b) == shape
    want = so.tensor_block_partition(shape, b)
    got = [((int(r[1]), int(r[2]), int(r[8]), int(r[10])), (int(r[3]), int(r[4]), int(r[9]), int(r[11]))) for r in t]
    assert got == want and all(int(r[7]) == 4 | 4 << 4 for r in t)
    assert nb == len({sz for _, sz in want})
    # buckets: equal (d1, d2, d3) share one; slots count up inside it
    shape, b = (10, 7, 5), 4
    t, nb = B.shampoo_plan(cfg_for([shape], b))
    keys = {}
    for r in t:
        k = (int(r[3]), int(r[4]), int(r[9]))
        assert keys.setdefault(k, int(r[5])) == int(r[5])
    assert nb == len(keys)
    # a tensor block needs three factors and roots: workspace grows accordingly
    assert B.shampoo_workspace_bytes(cfg_for([(64, 64, 9)], 128)) > 2 * 4 * (64 * 64 * 2 + 81)


@pytest.mark.parametrize("s,halves", [(2, 0), (6, 0), (64, 0), (128, 0), (4, 1), (16, 1), (64, 1),
                                      (4, 2), (8, 2), (12, 2), (32, 2), (64, 2), (256, 2)])
def test_jacobi_pair_schedule_is_a_tournament(s, halves):
    """Every round of the eigensolver's sweep is a perfect matching and the s - 1 rounds meet
    every pair once; in the pivot order the first s / 2 rounds pair across the two halves."""
    seen = set()
    for r in range(s - 1):
        used = set()
        for k in range(s // 2):
            p, q = B.shampoo_jacobi_pair(s, halves, r, k)
            assert 0 <= p < q < s
            assert p not in used and q not in used
            used.update((p, q))
            assert (p, q) not in seen
            seen.add((p, q))
            if halves == 1:
                assert (p < s // 2 <= q) == (r < s // 2)
        assert len(used) == s
    assert len(seen) == s * (s - 1) // 2


@pytest.mark.parametrize("s", [4, 12, 32, 256])
def test_block_column_schedule_keeps_two_rounds_inside_four_columns(s):
    """The block-column order of the blocked solver (halves = 2): round 0 pairs the members of
    each super-column (2 S, 2 S + 1); pairs 2 K and 2 K + 1 of rounds 1 + 2 R and 2 + 2 R touch
    the same four block columns, two whole super-columns, in the order the two-round update of
    the eigenvector rows assumes: (a, c), (b, d), then (a, d), (b, c) with a < b < c < d."""
    for k in range(s // 2):
        assert B.shampoo_jacobi_pair(s, 2, 0, k) == (2 * k, 2 * k + 1)
    for R in range(s // 2 - 1):
        for K in range(s // 4):
            first = [B.shampoo_jacobi_pair(s, 2, 1 + 2 * R, 2 * K + i) for i in range(2)]
            second = [B.shampoo_jacobi_pair(s, 2, 2 + 2 * R, 2 * K + i) for i in range(2)]
            a, c = first[0]
            assert a % 2 == 0 and c % 2 == 0 and a < c
            assert first[1] == (a + 1, c + 1)
            assert second == [(a, c + 1), (a + 1, c)]


def test_jacobi_pair_rejects_bad_arguments():
    for args in [(3, 0, 0, 0), (64, 0, 63, 0), (64, 0, 0, 32), (12, 1, 0, 0), (2, 1, 0, 0), (64, 0, -1, 0),
                 (6, 2, 0, 0), (64, 3, 0, 0)]:
        with pytest.raises(B.ShampooError):
            B.shampoo_jacobi_pair(*args)


def test_warm_root_inverse_rejects_bad_arguments_before_any_device_work():
    """Argument errors of shampoo_root_inverse_warm come back before anything touches the GPU:
    the pointers below are never dereferenced."""
    L = B.lib()
    ok_ptr, ws = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x100000)
    big = 1 << 40

    def call(a=ok_ptr, n=256, batch=2, eps=1e-12, r=0.25, x=ok_ptr, qt=ok_ptr, workspace=ws, nbytes=big):
        return L.shampoo_root_inverse_warm(a, n, batch, eps, r, x, None, None, qt, 0, None, workspace, nbytes, None)

    assert call(a=None) == -1 and call(x=None) == -1 and call(qt=None) == -1
    assert call(n=0) == -2 and call(batch=0) == -2
    assert call(n=128) == -7                      # the single-workgroup solver keeps no eigenvectors
    assert call(eps=0.0) == -3 and call(r=-1.0) == -3
    assert call(workspace=None) == -4 and call(workspace=ctypes.c_void_p(0x100004)) == -4
    assert call(nbytes=1024) == -4
    assert call(qt=ctypes.c_void_p(0x10004)) == -4   # the kernels move qt 16 bytes at a time


# ---------------------------------------------------------------------------
# the bound behind the block solver's exit after its float32 sweeps
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n,spread", [(96, 1.0), (96, 0.1), (257, 0.3)])
def test_bound_on_the_root_when_small_off_diagonals_are_dropped(n, spread):
    """The block solver lets a matrix leave after the float32 sweeps when W = D + E has
    min(D) >= 0.1 max(D) and ||E||_F <= 6e-5 sqrt(n) min(D), and then takes D for the spectrum.
    What that costs, for the inverse fourth root (Sec. 3.2.1 with r = 1/4), is at most
    ||E||_F / (4 sqrt(n) min(D)) of the root in the Frobenius norm, up to second order in E.
    Checked with the root inverse by numpy's eigendecomposition on E at the limit."""
    rng = np.random.default_rng(n)
    d = rng.uniform(spread, 1.0, n) * 3.7e-5
    d[0], d[1] = d.max(), spread * d.max()                # both ends of the allowed spread
    E = rng.standard_normal((n, n)); E = E + E.T; np.fill_diagonal(E, 0.0)
    theta = 6.0e-5
    E *= theta * np.sqrt(n) * d.min() / np.linalg.norm(E)
    lam, Q = np.linalg.eigh(np.diag(d) + E)
    exact = (Q * lam ** -0.25) @ Q.T
    taken = np.diag(d ** -0.25)
    err = np.linalg.norm(exact - taken) / np.linalg.norm(exact)
    assert err <= theta / 4 * 1.01
    assert err >= theta / 4 * 0.05        # the bound is not vacuous: the error is of that order
