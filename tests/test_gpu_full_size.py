"""Parity at the full sizes of the benchmark workloads, on sampled blocks.

The transformer-shaped set (1152 blocks of 1024 x 1024, bf16 gradients) runs in the
same launch configuration bench.py times; the oracle recomputes a sample of blocks one by
one from the same gradient bits.  The root-inverse stress case uses the 2048 x 2048
rank-64 + 1e-6 I matrices."""
import sys

import numpy as np
import pytest

from oracle import shampoo_oracle as so
from paper_2309_06497_amd import binding as B
from paper_2309_06497_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def rel(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def f32(x):
    return float(np.float32(x))


@pytest.mark.timeout(600)
def test_transformer_full_size_sampled_blocks():
    """Five steps of the 1.2e9-parameter set with the roots refreshed at t = 0 (from a single
    gradient: ill-conditioned) and t = 3 (well conditioned); sampled blocks and two LayerNorm
    vectors against the oracle.  Bars, all plain: factors 1e-5; root inverse against the
    oracle's on the same float32 factor bits 2e-4; directions, momentum and parameter updates
    2e-3 at every step, also while the roots of the single-gradient factors are in use (the
    factor update of those first steps sums in float64; what remains is the float32 storage of
    the factor, measured 3e-4 ... 6e-4 in the direction)."""
    import torch
    shapes = wl.transformer_shapes()
    dev = torch.device("cuda", 0)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    say("case transformer full size: allocating")
    params = [torch.randn(s, generator=gen, device=dev) * 0.02 for s in shapes]
    F = 3
    opt = B.Shampoo(shapes, 1024, 0.999, 1e-12, 0.25, F, 0, 1e-10, 0.9, B.GRAD_BF16)
    table, _ = opt.plan()
    assert len(table) == 1152
    # sampled blocks: (param index, block index inside the parameter)
    two_d = [i for i, s in enumerate(shapes) if len(s) == 2]
    sample = [(two_d[0], 5), (two_d[40], 9), (two_d[-1], 15)]
    vecs = [0, len(shapes) - 1]
    blocks = {}
    for (i, k) in sample:
        r0, c0, m, n = so.block_partition(shapes[i][0], shapes[i][1], 1024)[k]
        blocks[(i, k)] = (slice(r0, r0 + m), slice(c0, c0 + n))
    ora = {key: so.ShampooOracle([(1024, 1024)], 1024, f32(0.999), f32(1e-12), 0.25, F, 0, f32(1e-10), f32(0.9))
           for key in sample}
    w_ora = {key: [params[key[0]][blocks[key]].cpu().numpy().astype(np.float64)] for key in sample}
    w0 = {key: w_ora[key][0].copy() for key in sample}
    ora_v = {i: so.ShampooOracle([shapes[i]], 1024, f32(0.999), f32(1e-12), 0.25, F, 0, f32(1e-10), f32(0.9)) for i in vecs}
    wv_ora = {i: [params[i].cpu().numpy().astype(np.float64)] for i in vecs}
    cond = {key: 0.0 for key in sample}
    for t in range(5):
        say(f"  step {t}")
        grads = [(torch.randn(s, generator=gen, device=dev) * 1e-3).to(torch.bfloat16) for s in shapes]
        opt.step(params, grads, 0.01, t)
        torch.cuda.synchronize()
        for key in sample:
            i, k = key
            g = grads[i][blocks[key]].to(torch.float32).cpu().numpy()
            ora[key].step(w_ora[key], [g], f32(0.01), t)
            L = opt.get(i, k, B.GET_L).cpu().numpy()
            R = opt.get(i, k, B.GET_R).cpu().numpy()
            e_l, e_r = rel(L, ora[key].L[0][0]), rel(R, ora[key].R[0][0])
            P = opt.get(i, k, B.GET_PSH).cpu().numpy()
            e_p = rel(P, ora[key].P_sh[0][0])
            e_m = rel(opt.get(i, k, B.GET_M).cpu().numpy(), ora[key].M[0])
            e_w = rel(params[i][blocks[key]].cpu().numpy().astype(np.float64) - w0[key], w_ora[key][0] - w0[key])
            e_root = -1.0
            if t % F == 0:
                Li = opt.get(i, k, B.GET_LINV).cpu().numpy()
                e_root = rel(Li, so.root_inverse(L, f32(1e-12), 0.25)[0])
                assert e_root <= 2e-4
                # smallest eigenvalue of the factors against the largest: what makes t = 0 hard
                cond[key] = max(np.linalg.eigvalsh(Fm)[-1] / max(np.linalg.eigvalsh(Fm)[0], 1e-300)
                                for Fm in (ora[key].L[0][0], ora[key].R[0][0]))
            say(f"    block {key}: L={e_l:.1e} R={e_r:.1e} root={e_root:.1e} Psh={e_p:.1e} M={e_m:.1e} dW={e_w:.1e}"
                f" (condition number of the factors in use {cond[key]:.1e})")
            assert e_l <= 1e-5 and e_r <= 1e-5
            assert e_p <= 2e-3 and e_m <= 2e-3 and e_w <= 2e-3
            if t >= F:
                assert e_p <= 2e-5
        for i in vecs:
            ora_v[i].step(wv_ora[i], [grads[i].to(torch.float32).cpu().numpy()], f32(0.01), t)
            assert rel(params[i].cpu().numpy(), wv_ora[i][0]) <= 1e-6
        del grads
    st = opt.status()
    assert st == {"refreshes": 2, "failed_roots": 0}


@pytest.mark.timeout(600)
def test_root_inverse_stress_2048():
    """A = sum_{k<64} g_k g_k^T + 1e-6 I at n = 2048, formed in float64 and rounded once to
    float32 (the ridge is below half an ulp of the diagonal, so the float32 matrix is rank 64
    plus rounding noise).  Graded on what float32 input determines: the 64 dominant
    eigenvalues, the action of X on the generators g_k (the range), X^4 (A + eps I) v = v on
    the dominant eigenvectors, symmetry; the full-matrix error against the oracle (which
    depends on the noise eigenvalues of the float32 matrix) is printed and loosely bounded."""
    import torch
    n, rank, batch = 2048, 64, 6
    say("case root stress 2048")
    mats, gens = [], []
    for i in range(batch):
        a, g = wl.psd_stress_matrix(n, rank, 11, i)
        mats.append(a); gens.append(g)
    a = np.stack(mats)
    eps = f32(1e-12)
    x, lam, failed = B.shampoo_root_inverse(torch.from_numpy(a).cuda(), 1e-12, 0.25, True, True)
    x = x.cpu().numpy(); lam = lam.cpu().numpy()
    assert not failed.cpu().numpy().any(), (failed.cpu().numpy(), np.isnan(lam).sum(axis=1))
    for i in range(batch):
        assert np.array_equal(x[i], x[i].T)
        assert np.isfinite(x[i]).all()
    for i in (0, batch - 1):     # oracle on two of them (float64 eigh of a 2048 matrix each)
        xo, lo = so.root_inverse(a[i], eps, 0.25)
        top_gpu = np.sort(lam[i])[-rank:]
        e_top = np.abs(top_gpu - lo[-rank:]).max() / lo[-1]
        g = gens[i]
        xg, xog = x[i].astype(np.float64) @ g, xo @ g
        e_range = np.linalg.norm(xg - xog) / np.linalg.norm(xog)
        w, V = np.linalg.eigh(a[i].astype(np.float64))
        Vd = V[:, -rank:]
        # X^4 (A + eps I) = I restricted to the dominant eigenvectors, without forming X^4
        # (whose null-space part, of size eps^-1 = 1e12, would swamp float32 rounding):
        # X v_i (lambda_i')^(1/4) = v_i
        shift = min(w[0], 0.0)
        lam_new = w[-rank:] - shift + eps
        resid = (x[i].astype(np.float64) @ Vd) * lam_new ** 0.25 - Vd
        e_x4 = np.linalg.norm(resid) / np.sqrt(rank)
        e_full = rel(x[i], xo)
        say(f"    matrix {i}: top-64 eig err {e_top:.1e}, action on range {e_range:.1e}, "
            f"X V lam^(1/4) - V {e_x4:.1e}, full matrix {e_full:.1e}, lambda_min {lo[0]:.2e}")
        assert e_top <= 1e-5
        assert e_range <= 2e-3
        assert e_x4 <= 2e-3
        assert e_full <= 3e-3


@pytest.mark.timeout(900)
def test_resnet50_shapes_every_block():
    """The ResNet-50 parameter set (54 weights -> 1576 blocks in 6 buckets at block 128, 107
    vectors, 25.6e6 parameters), per-tensor sigma log-uniform in [1e-4, 1e-2]: the oracle runs
    the whole set; every block and vector is compared (see Pair.check for the bars)."""
    from test_gpu_parity import Pair
    say("case resnet50 shapes")
    shapes = wl.resnet50_shapes()
    sig = wl.per_tensor_sigmas(shapes, 21)
    p = Pair(shapes, 128, 0.999, 3)
    for t in range(5):
        p.step(wl.gaussian_grads(shapes, 21, t, sig), 0.01, t)
        if t in (0, 1, 3, 4):
            p.check(t)
    assert p.gpu.status() == {"refreshes": 2, "failed_roots": 0}


@pytest.mark.gpu
@pytest.mark.timeout(900)
def test_resnet50_with_convolution_weights_as_tensors():
    """ResNet-50 with its convolution weights given as (out, in, kh, kw): merging (Sec. 4.2.1)
    turns the 1 x 1 ones into matrices and leaves the 3 x 3 ones and the stem as order-3
    tensors (out, in, 9) / (64, 21, 7), blocked at 128; every tensor block's factors, roots,
    direction and momentum and every parameter's update against the oracle."""
    from test_gpu_parity import TensorPair, say
    say("case resnet50, 4-D convolution weights")
    shapes = wl.resnet50_conv4d_shapes()
    sig = wl.per_tensor_sigmas(shapes, 22)
    p = TensorPair(shapes, 128, 0.999, 2, eps=1e-6)
    table, _ = p.gpu.plan()
    n_tensor = sum(1 for r in table if int(r[7]) & 4)
    say(f"    {len(table)} blocks, {n_tensor} of them tensor blocks")
    assert n_tensor == 1 + 3 * 1 + 4 * 1 + 6 * 4 + 3 * 16      # stem; 3 x 3 convolutions of widths 64, 128, 256, 512
    for t in range(3):
        p.step(wl.gaussian_grads(shapes, 22, t, sig), 0.01, t)
        p.check(t)
    assert p.gpu.status() == {"refreshes": 2, "failed_roots": 0}


@pytest.mark.gpu
def test_block_size_2048():
    """Sec. 4.2.1 / Table 5 use preconditioner blocks up to 8192; one 2048 x 2048 block exercises
    16 x 16 tiles per GEMM and the blocked eigensolver at n = 2048 inside the optimizer."""
    from test_gpu_parity import Pair, say
    say("case block 2048")
    shapes = [(2048, 2048), (2048,)]
    p = Pair(shapes, 2048, 0.999, 2, bf16=True)
    for t in range(3):
        p.step(wl.gaussian_grads(shapes, 90, t, 1e-3), 0.01, t)
        p.check(t)
    assert p.gpu.status() == {"refreshes": 2, "failed_roots": 0}


@pytest.mark.gpu
def test_root_inverse_4096():
    """The largest block sizes the paper recommends are 4096 and 8192 (Sec. 4.2.1): one
    well-conditioned 4096 x 4096 factor through the blocked eigensolver (64 pivot pairs per
    round, 127 rounds per sweep) against the oracle."""
    import torch
    from test_gpu_parity import say, rel
    say("case root inverse n=4096")
    n = 4096
    g = torch.Generator(device="cuda")
    g.manual_seed(4096)
    G = torch.randn((n, 2 * n), generator=g, device="cuda", dtype=torch.float32) * 1e-2
    a = (G @ G.T) / (2 * n)
    a = 0.5 * (a + a.T)
    x, lam, failed = B.shampoo_root_inverse(a[None], 1e-12, 0.25, True, True)
    assert int(failed[0]) == 0
    X, lam_o = so.root_inverse(a.cpu().numpy(), float(np.float32(1e-12)), 0.25)
    e_x = rel(x[0].cpu().numpy(), X)
    e_l = np.abs(np.sort(lam[0].cpu().numpy().astype(np.float64)) - lam_o).max() / lam_o.max()
    say(f"    X rel err {e_x:.1e}, eigenvalue err {e_l:.1e} lambda_max")
    assert e_x <= 1e-4 and e_l <= 2e-6
    assert torch.equal(x[0], x[0].T)


@pytest.mark.gpu
@pytest.mark.timeout(600)
def test_root_inverse_8192_by_its_defining_property():
    """The largest block size the library accepts (and the paper's Table 5 uses) is 8192.  A
    LAPACK eigendecomposition of that size takes minutes on the host, so this case is held to
    what defines the result instead of to the oracle: X symmetric, X^4 (A + eps I) = I, and the
    eigenvalues summing to the trace; the product is formed in float64 on the device.  A root
    with relative error d leaves X^4 (A + eps I) - I = 4 d to first order (per eigen-direction),
    so the bar of 1e-4 on the root itself, which the n = 4096 case is held to against the
    oracle, is 4e-4 on this residual (measured 1.5e-4: the error of the accumulated
    eigenvectors grows in proportion to the number of rounds, 1.2e-5 at 4096, 2.3e-5 here)."""
    import torch
    from test_gpu_parity import say
    say("case root inverse n=8192")
    n = 8192
    g = torch.Generator(device="cuda")
    g.manual_seed(8192)
    G = torch.randn((n, 2 * n), generator=g, device="cuda", dtype=torch.float32) * 1e-2
    a = (G @ G.T) / (2 * n)
    del G
    a = 0.5 * (a + a.T)
    x, lam, failed = B.shampoo_root_inverse(a[None], 1e-12, 0.25, True, True)
    torch.cuda.synchronize()
    assert int(failed[0]) == 0
    assert torch.equal(x[0], x[0].T)
    X = x[0].double()
    A = a.double() + float(np.float32(1e-12)) * torch.eye(n, dtype=torch.float64, device="cuda")
    X2 = X @ X
    R = X2 @ X2 @ A
    R -= torch.eye(n, dtype=torch.float64, device="cuda")
    err = float(torch.linalg.norm(R)) / np.sqrt(n)
    tr = float(torch.trace(a.double()))
    e_tr = abs(float(lam[0].double().sum()) - tr) / tr
    say(f"    ||X^4 (A + eps I) - I||_F / sqrt(n) = {err:.1e}, trace error {e_tr:.1e}")
    assert err <= 4e-4 and e_tr <= 1e-6


@pytest.mark.gpu
@pytest.mark.timeout(900)
def test_uniform_config_as_stated_200_steps():
    """The uniform workload as stated: 512 blocks of 128 x 128, float32 gradients N(0, 1e-3^2),
    beta2 = 0.999, roots refreshed every 100 steps, 200 steps (refreshes at t = 0 and t = 100).
    The oracle follows a sample of 32 blocks (blocks are independent) for all 200 steps.
    Factors <= 1e-5 at every checked step up to t = 199 (the drift of a float32 moving average
    over 200 roundings); at t = 100 the root against the oracle's on the same float32 bits
    (2e-4) and the products against float64 from the GPU's roots (2e-5); directions, momentum and
    parameter updates of the sample together <= 2e-3."""
    import torch
    from test_gpu_parity import say, rel
    say("case uniform as stated: 512 blocks, 200 steps, f = 100")
    n_blocks, b, F, steps = 512, 128, 100, 200
    shapes = wl.uniform_shapes(n_blocks, b)
    dev = torch.device("cuda", 0)
    gen = torch.Generator(device=dev)
    gen.manual_seed(2)
    params = [torch.randn(s, generator=gen, device=dev) * 0.02 for s in shapes]
    opt = B.Shampoo(shapes, b, 0.999, 1e-12, 0.25, F, 0, 1e-10, 0.9)
    sample = list(range(0, n_blocks, n_blocks // 32))
    assert len(sample) == 32
    ora = so.ShampooOracle([shapes[i] for i in sample], b, f32(0.999), f32(1e-12), 0.25, F, 0, f32(1e-10), f32(0.9))
    w_ora = [params[i].cpu().numpy().astype(np.float64) for i in sample]
    w0 = [w.copy() for w in w_ora]
    checked = (0, 1, 50, 99, 100, 101, 150, 199)
    for t in range(steps):
        g_all = torch.randn((n_blocks, b, b), generator=gen, device=dev) * 1e-3
        grads = [g_all[i] for i in range(n_blocks)]
        opt.step(params, grads, 0.01, t)
        g_host = g_all[sample].cpu().numpy()
        ora.step(w_ora, [g_host[j] for j in range(32)], f32(0.01), t)
        if t not in checked:
            continue
        worst = {"L": 0.0, "R": 0.0, "root": 0.0, "gemm": 0.0}
        num = {"Psh": 0.0, "M": 0.0, "dW": 0.0}
        den = {"Psh": 0.0, "M": 0.0, "dW": 0.0}
        for j, i in enumerate(sample):
            L = opt.get(i, 0, B.GET_L).cpu().numpy(); R = opt.get(i, 0, B.GET_R).cpu().numpy()
            worst["L"] = max(worst["L"], rel(L, ora.L[j][0])); worst["R"] = max(worst["R"], rel(R, ora.R[j][0]))
            Li = opt.get(i, 0, B.GET_LINV).cpu().numpy(); Ri = opt.get(i, 0, B.GET_RINV).cpu().numpy()
            P = opt.get(i, 0, B.GET_PSH).cpu().numpy()
            if t % F == 0:
                worst["root"] = max(worst["root"], rel(Li, so.root_inverse(L, f32(1e-12), 0.25)[0]),
                                    rel(Ri, so.root_inverse(R, f32(1e-12), 0.25)[0]))
            worst["gemm"] = max(worst["gemm"], rel(P, so.shampoo_direction(Li.astype(np.float64), g_host[j], Ri.astype(np.float64))))
            M = opt.get(i, 0, B.GET_M).cpu().numpy()
            dw_g = params[i].cpu().numpy().astype(np.float64) - w0[j]
            for key, got, want, wgt in (("Psh", P, ora.P_sh[j][0], ora.s_g[j][0]), ("M", M, ora.M[j], None),
                                        ("dW", dw_g, w_ora[j] - w0[j], None)):
                d2, w2 = np.linalg.norm(got - want) ** 2, np.linalg.norm(want) ** 2
                if wgt is not None:       # weight of the block in the grafted search direction
                    d2, w2 = d2 / w2 * wgt, wgt
                num[key] += d2; den[key] += w2
        total = {k: np.sqrt(num[k] / den[k]) for k in num}
        say(f"    t={t} worst of 32 blocks: " + " ".join(f"{k}={v:.1e}" for k, v in worst.items())
            + " | sample together: " + " ".join(f"{k}={v:.1e}" for k, v in total.items()))
        assert worst["L"] <= 1e-5 and worst["R"] <= 1e-5
        assert worst["root"] <= 2e-4 and worst["gemm"] <= 2e-5
        assert all(v <= 2e-3 for v in total.values()), total
        if t >= F:
            assert total["Psh"] <= 2e-5
    assert opt.status() == {"refreshes": 2, "failed_roots": 0}


@pytest.mark.gpu
@pytest.mark.timeout(900)
@pytest.mark.parametrize("bf16", [True, False])
def test_block_size_4096_whole_step(bf16):
    """Block size 4096 (Sec. 4.2.1 names 4096 and 8192 as the ideal sizes; Table 5) through
    the whole step, not only the eigensolver: one 4096 x 4096 block, factor updates over 32 x 32
    tiles, the blocked eigensolver at n = 4096 inside the optimizer, both products, norms,
    momentum and update, at t = 0 (refresh from a single gradient) and t = 1 (the same roots,
    now stale, on a fresh gradient).  The oracle runs the same block: factors 1e-5; the left
    root against the oracle's on the same float32 bits 2e-4; the products against float64 from
    the GPU's roots 2e-5; directions, momentum and parameter updates the plain 2e-3."""
    import torch
    from test_gpu_parity import say, rel, StorageEffect
    n = 4096
    say(f"case block 4096, {'bf16' if bf16 else 'float32'} gradients")
    shapes = [(n, n)]
    dev = torch.device("cuda", 0)
    gen = torch.Generator(device=dev)
    gen.manual_seed(4096 + int(bf16))
    params = [torch.randn(shapes[0], generator=gen, device=dev) * 0.02]
    opt = B.Shampoo(shapes, n, 0.999, 1e-12, 0.25, 2, 0, 1e-10, 0.9, B.GRAD_BF16 if bf16 else B.GRAD_F32)
    ora = so.ShampooOracle(shapes, n, f32(0.999), f32(1e-12), 0.25, 2, 0, f32(1e-10), f32(0.9))
    w_ora = [params[0].cpu().numpy().astype(np.float64)]
    w0 = w_ora[0].copy()
    for t in range(2):
        g = torch.randn(shapes[0], generator=gen, device=dev) * 1e-3
        if bf16:
            g = g.to(torch.bfloat16)
        opt.step(params, [g], 0.01, t)
        torch.cuda.synchronize()
        g_host = g.to(torch.float32).cpu().numpy()
        say(f"  step {t}: oracle")
        ora.step(w_ora, [g_host], f32(0.01), t)
        L = opt.get(0, 0, B.GET_L).cpu().numpy(); R = opt.get(0, 0, B.GET_R).cpu().numpy()
        assert np.array_equal(L, L.T) and np.array_equal(R, R.T)
        e_l, e_r = rel(L, ora.L[0][0]), rel(R, ora.R[0][0])
        Li = opt.get(0, 0, B.GET_LINV).cpu().numpy(); Ri = opt.get(0, 0, B.GET_RINV).cpu().numpy()
        P = opt.get(0, 0, B.GET_PSH).cpu().numpy()
        e_root = -1.0
        if t == 0 and bf16:
            say("  root of the GPU's factor bits: oracle")
            e_root = rel(Li, so.root_inverse(L, f32(1e-12), 0.25)[0])
            assert e_root <= 2e-4
        e_gemm = rel(P, so.shampoo_direction(Li.astype(np.float64), g_host, Ri.astype(np.float64)))
        e_p = rel(P, ora.P_sh[0][0])
        e_m = rel(opt.get(0, 0, B.GET_M).cpu().numpy(), ora.M[0])
        e_w = rel(params[0].cpu().numpy().astype(np.float64) - w0, w_ora[0] - w0)
        norms = opt.get(0, 0, B.GET_NORMS).cpu().numpy()
        say(f"    t={t}: L={e_l:.1e} R={e_r:.1e} root={e_root:.1e} gemm={e_gemm:.1e} Psh={e_p:.1e} M={e_m:.1e} dW={e_w:.1e}")
        assert e_l <= 1e-5 and e_r <= 1e-5
        assert e_gemm <= 2e-5
        allow = 0.0
        if t == 1:
            # The roots in use are those of a single 4096 x 4096 gradient (condition number of the
            # factor 1e8 and up) and meet a fresh gradient: float32 storage of the factor alone
            # costs s (test_gpu_parity.StorageEffect, from the oracle's factors; two draws),
            # and the block is allowed 8 s on top of the bar, at most ten bars, as everywhere.
            say("  storage effect of the t = 0 factors: oracle")
            s_blk = np.sqrt(np.mean([np.linalg.norm(effects[0].draw() @ g_host @ ora.Rbar[0][0]
                                                    + ora.Lbar[0][0] @ g_host @ effects[1].draw()) ** 2
                                     for _ in range(2)])) / np.linalg.norm(ora.P_sh[0][0])
            allow = min(8.0 * s_blk, 2e-2)
            say(f"    s = {s_blk:.1e}")
            assert 2.0 * s_blk <= 2e-3, "the block is expected to be resolved by float32"
        else:
            effects = (StorageEffect(ora.L[0][0], f32(1e-12), 1), StorageEffect(ora.R[0][0], f32(1e-12), 2))
        assert e_p <= 2e-3 + allow and e_m <= 2e-3 + allow and e_w <= 2e-3 + allow
        assert abs(norms[0] - ora.s_g[0][0]) <= 2e-4 * ora.s_g[0][0]
        assert abs(norms[1] - ora.s_sh[0][0]) <= 5e-3 * ora.s_sh[0][0]
    assert opt.status() == {"refreshes": 1, "failed_roots": 0}


@pytest.mark.gpu
@pytest.mark.timeout(900)
def test_block_size_8192_whole_step_by_defining_properties():
    """The largest block size (8192, Table 5) through the whole step.  A float64
    eigendecomposition of that size takes minutes on the host, so the oracle is not run here
    ("parity unpinned" against the oracle at this size); every stage is held to what defines it,
    evaluated in float64 on the device: factors against G G^T / G^T G of the same bf16 bits;
    roots by X^4 (L + eps I) = I (four gradients are summed before the refresh, so that the
    factors are well conditioned and the identity is a sharp test); Lbar G Rbar against the
    float64 product of the GPU's roots; the grafted update by its norm, ||dW|| = lr ||P_graft||
    at the first Shampoo step with zero momentum."""
    import torch
    from test_gpu_parity import say
    n = 8192
    say("case block 8192")
    shapes = [(n, n)]
    dev = torch.device("cuda", 0)
    gen = torch.Generator(device=dev)
    gen.manual_seed(8192)
    params = [torch.randn(shapes[0], generator=gen, device=dev) * 0.02]
    start = 3
    opt = B.Shampoo(shapes, n, 1.0, 1e-12, 0.25, start, start, 1e-10, 0.0, B.GRAD_BF16)
    Lref = torch.zeros((n, n), dtype=torch.float64, device=dev)
    Rref = torch.zeros((n, n), dtype=torch.float64, device=dev)
    Aref = torch.zeros((n, n), dtype=torch.float64, device=dev)
    eye = torch.eye(n, dtype=torch.float64, device=dev)
    frob = lambda a, b_: float(torch.linalg.norm(a - b_) / torch.linalg.norm(b_))
    for t in range(start + 1):
        g = (torch.randn(shapes[0], generator=gen, device=dev) * 1e-3).to(torch.bfloat16)
        w_before = params[0].clone()
        opt.step(params, [g], 0.01, t)
        torch.cuda.synchronize()
        say(f"  step {t} done")
        gd = g.double()
        Lref += gd @ gd.T; Rref += gd.T @ gd; Aref += gd * gd
    L = opt.get(0, 0, B.GET_L); R = opt.get(0, 0, B.GET_R)
    assert torch.equal(L, L.T) and torch.equal(R, R.T)
    e_l, e_r = frob(L.double(), Lref), frob(R.double(), Rref)
    Li = opt.get(0, 0, B.GET_LINV).double(); Ri = opt.get(0, 0, B.GET_RINV).double()
    eps = float(np.float32(1e-12))
    e_roots = []
    for X, F in ((Li, L.double()), (Ri, R.double())):
        X2 = X @ X
        e_roots.append(float(torch.linalg.norm(X2 @ X2 @ (F + eps * eye) - eye)) / np.sqrt(n))
    P = opt.get(0, 0, B.GET_PSH).double()
    e_gemm = frob(P, Li @ gd @ Ri)
    # grafting: the update has the length of the AdaGrad direction (momentum 0, first Shampoo step)
    pg = gd / (Aref.sqrt() + float(np.float32(1e-10)))
    dw = (params[0] - w_before).double()
    e_norm = abs(float(torch.linalg.norm(dw)) - float(np.float32(0.01)) * float(torch.linalg.norm(pg))) / float(torch.linalg.norm(dw))
    e_dir = frob(dw, -float(np.float32(0.01)) * torch.linalg.norm(pg) * P / torch.linalg.norm(P))
    say(f"    L={e_l:.1e} R={e_r:.1e} X^4(F+eps)-I: {e_roots[0]:.1e} {e_roots[1]:.1e} gemm={e_gemm:.1e} "
        f"|dW| vs lr|P_graft| {e_norm:.1e} dW direction {e_dir:.1e}")
    assert e_l <= 1e-5 and e_r <= 1e-5
    assert max(e_roots) <= 4e-4      # 4 x the 1e-4 bar on the root itself: the residual is four times the root's relative error
    assert e_gemm <= 2e-5
    assert e_norm <= 1e-4 and e_dir <= 1e-4
    assert opt.status() == {"refreshes": 1, "failed_roots": 0}
