"""The first-order model of what float32 storage of a factor costs in the Shampoo direction
(tests/test_gpu_parity.py, StorageEffect: it sets the per-block allowance of the end-to-end
GPU comparisons) against the real thing on the CPU: factors rounded to float32 for real, roots
retaken by the oracle in float64."""
import numpy as np

from oracle import shampoo_oracle as so
from test_gpu_parity import StorageEffect


def test_first_order_storage_effect_matches_actual_rounding():
    rng = np.random.default_rng(5)
    n, eps = 96, float(np.float32(1e-12))
    actual2, model2 = [], []
    for trial in range(12):
        G = rng.normal(size=(n, n)) * 1e-3
        L, R = 1e-3 * G @ G.T, 1e-3 * G.T @ G          # single-gradient factors: condition number ~1e6
        Lb, Rb = so.root_inverse(L, eps, 0.25)[0], so.root_inverse(R, eps, 0.25)[0]
        G1 = rng.normal(size=(n, n)) * 1e-3            # a later gradient, seen through the stale roots
        P = so.shampoo_direction(Lb, G1, Rb)
        L32, R32 = L.astype(np.float32).astype(np.float64), R.astype(np.float32).astype(np.float64)
        P32 = so.shampoo_direction(so.root_inverse(L32, eps, 0.25)[0], G1, so.root_inverse(R32, eps, 0.25)[0])
        actual2.append((np.linalg.norm(P32 - P) / np.linalg.norm(P)) ** 2)
        el, er = StorageEffect(L, eps, 2 * trial), StorageEffect(R, eps, 2 * trial + 1)
        d2 = np.mean([np.linalg.norm(el.draw() @ G1 @ Rb + Lb @ G1 @ er.draw()) ** 2 for _ in range(4)])
        model2.append(d2 / np.linalg.norm(P) ** 2)
    ratio = np.sqrt(np.mean(actual2) / np.mean(model2))
    assert 0.5 <= ratio <= 2.0, ratio


def test_storage_effect_of_a_diagonal_factor_is_the_scalar_derivative():
    d = np.array([4.0, 1.0, 0.25])
    e = StorageEffect(d, 0.0, 0)
    dx = np.diag(e.draw())
    # |d x / x| = |d lambda / lambda| / 4 <= 2^-24 / 4 entry by entry
    assert np.all(np.abs(dx) * 4.0 <= 2.0 ** -24 * d ** -0.25 * (1 + 1e-6))
    assert np.any(dx != 0.0)
