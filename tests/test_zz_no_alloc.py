"""The entry point that allocates nothing (shampoo_root_inverse_static: the solver's working
arrays in a fixed array inside the library's device image) against shampoo_root_inverse on the
same matrices: two calls in a row, the second one smaller, so that what the first call left in
the shared array is in the way of the second.  Also the n <= 128 path (no scratch at all), the
size limit, and that no device memory is allocated during the calls."""
import sys

import numpy as np
import pytest

from paper_2309_06497_amd import binding as B

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def wishart(batch, n, seed, cols=None):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    cols = cols or 2 * n
    G = torch.randn((batch, n, cols), generator=g, device="cuda", dtype=torch.float32) * 1e-2
    a = torch.bmm(G, G.transpose(1, 2)) / cols
    return (0.5 * (a + a.transpose(1, 2))).contiguous()


def both(a, eps=1e-12, r=0.25):
    """(static entry point, workspace entry point) results for the same input."""
    import torch
    batch, n = a.shape[0], a.shape[1]
    x = torch.full_like(a, float("nan"))
    lam = torch.full((batch, n), float("nan"), dtype=torch.float32, device=a.device)
    failed = torch.full((batch,), 7, dtype=torch.int32, device=a.device)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.shampoo_root_inverse_static(a, eps, r, x, lam, failed)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    x_ref, lam_ref, failed_ref = B.shampoo_root_inverse(a, eps, r, True, True)
    torch.cuda.synchronize()
    return (x, lam, failed), (x_ref, lam_ref, failed_ref)


def compare(got, ref, name):
    import torch
    (x, lam, failed), (x_ref, lam_ref, failed_ref) = got, ref
    assert torch.equal(failed, failed_ref) and int(failed.sum()) == 0, name
    assert torch.isfinite(x).all() and torch.isfinite(lam).all(), name
    # both entry points run the same kernels on the same matrix, each matrix on its own, so the
    # results agree to the last bit; the bar for floating point is 1e-6 all the same
    e_x = float(torch.linalg.norm((x - x_ref).double()) / torch.linalg.norm(x_ref.double()))
    e_l = float((lam - lam_ref).abs().max() / lam_ref.abs().max())
    say(f"    {name}: X rel diff {e_x:.1e}, eigenvalue diff {e_l:.1e}, bitwise equal {torch.equal(x, x_ref)}")
    assert e_x <= 1e-6 and e_l <= 1e-6, name
    for i in range(x.shape[0]):
        assert torch.equal(x[i], x[i].T), name


def test_static_entry_point_two_calls_second_smaller():
    say("case no-alloc root inverse: 7 x 1024, then 3 x 200, then 2 x 2048")
    a1 = wishart(7, 1024, 101)          # five matrices fit the array at a time: two chunks
    compare(*both(a1), "first call, 7 x 1024")
    a2 = wishart(3, 200, 102)           # smaller, padded to 256: reuses the front of the array
    compare(*both(a2), "second call, 3 x 200")
    a3 = wishart(2, 2048, 103, cols=2560)   # the largest size: one matrix fills the array
    compare(*both(a3), "third call, 2 x 2048")


def test_static_entry_point_small_matrices_and_limits():
    import torch
    say("case no-alloc root inverse: LDS path and limits")
    a = wishart(9, 96, 104)
    compare(*both(a), "9 x 96")
    big = torch.zeros((1, 2112, 2112), dtype=torch.float32, device="cuda")
    x = torch.zeros_like(big)
    with pytest.raises(B.ShampooError) as e:
        B.shampoo_root_inverse_static(big, 1e-12, 0.25, x)
    assert e.value.code == -7
    with pytest.raises(B.ShampooError) as e:
        B.shampoo_root_inverse_static(a, 0.0, 0.25, torch.empty_like(a))
    assert e.value.code == -3
