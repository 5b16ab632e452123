"""The arithmetic behind the fp16-plane products of the GPU path, checked in numpy on the CPU:
a float32 matrix scaled by a power of two below 2^14 and split into two fp16 terms loses at most
2^-22 of each element (or 2^-25 / scale absolutely, for elements far below the largest), the
three products (h,h) (h,l) (l,h) accumulated in float32 reproduce the float64 product to
float32 accuracy, and undoing the power-of-two scales is exact.  This is a model of the scheme,
not of the kernel: no code is shared with the HIP path."""
import numpy as np
import pytest


def pow2_scale(bound):
    """largest power of two s with s * bound < 2^14 (1 for a zero bound)"""
    if not (bound > 0 and np.isfinite(bound)):
        return 1.0
    _, e = np.frexp(np.float32(bound))      # bound = f 2^e, f in [0.5, 1)
    return float(np.ldexp(1.0, int(np.clip(14 - e, -126, 100))))


def split2h(x, s):
    xs = (x.astype(np.float32) * np.float32(s)).astype(np.float32)
    h = xs.astype(np.float16)
    l = (xs - h.astype(np.float32)).astype(np.float16)
    return h, l


@pytest.mark.parametrize("sigma", [1e-15, 1e-3, 1.0, 1e10])
def test_two_fp16_planes_carry_a_float32(sigma):
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((64, 96)) * sigma).astype(np.float32)
    x[0, :8] *= 1e-7                                   # a few elements far below the largest
    s = pow2_scale(np.abs(x).max())
    assert 2.0 ** 13 <= s * np.abs(x).max() < 2.0 ** 14
    h, l = split2h(x, s)
    assert np.isfinite(h.astype(np.float32)).all()
    back = (h.astype(np.float64) + l.astype(np.float64)) / s
    err = np.abs(back - x.astype(np.float64))
    bound = np.maximum(2.0 ** -22 * np.abs(x.astype(np.float64)), 2.0 ** -24 / s)
    assert (err <= bound).all()


def test_three_plane_products_match_the_float64_product():
    rng = np.random.default_rng(8)
    m, k, n = 96, 256, 80
    a = rng.standard_normal((m, k)).astype(np.float32) * np.float32(3e-2)
    b = (np.eye(k, n) * 40.0 + rng.standard_normal((k, n)) * 0.3).astype(np.float32)   # diagonally dominant, like a root
    sa, sb = pow2_scale(np.abs(a).max()), pow2_scale(np.abs(b).max())
    ah, al = split2h(a, sa)
    bh, bl = split2h(b, sb)
    f32 = lambda v: v.astype(np.float32)
    # products of fp16 values are exact in float32; the sums are float32 like the MFMA accumulators
    acc = f32(ah) @ f32(bh) + (f32(ah) @ f32(bl) + f32(al) @ f32(bh))
    got = acc.astype(np.float64) / (sa * sb)
    want = a.astype(np.float64) @ b.astype(np.float64)
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    assert rel <= 2e-6
    # the plain float32 product is no better
    rel32 = np.linalg.norm((a @ b).astype(np.float64) - want) / np.linalg.norm(want)
    assert rel <= 4 * rel32 + 1e-7
    # without the low planes the error is that of an 11-bit mantissa
    rel_h = np.linalg.norm((f32(ah) @ f32(bh)).astype(np.float64) / (sa * sb) - want) / np.linalg.norm(want)
    assert rel_h > 50 * rel


def test_a_scaled_bf16_gradient_is_one_exact_fp16_plane():
    rng = np.random.default_rng(9)
    g32 = (rng.standard_normal((128, 64)) * 1e-3).astype(np.float32)
    g = (g32.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)        # bf16 values (truncated)
    s = pow2_scale(np.abs(g).max())
    gh = (g * np.float32(s)).astype(np.float16)
    exact = gh.astype(np.float64) / s == g.astype(np.float64)
    # 8 significant bits fit into 11; only elements below 2^-31 of the largest could round
    assert exact[np.abs(g) >= 2.0 ** -31 * np.abs(g).max()].all()
