"""Seeded synthetic workloads: parameter shape lists and gradient generators.

This module holds no optimizer arithmetic.  It only describes parameter sets
(shapes) and draws seeded random inputs, so that the tests can hand identical
bits to the HIP library and to the CPU oracle.  It depends on numpy only.

Workloads (the shapes stand in for the models the paper trains; the paper's
own experiment is ImageNet ResNet-50 training, Sec. 5, which needs a dataset
that is not used here):
  tiny          one 256x128 weight (block 64) + one bias of 128
  uniform       512 weights of 128x128
  resnet50      ResNet-50 layer list, conv weights viewed as (out, in*kh*kw),
                fc as 2048x1000, BatchNorm / bias vectors 1-D
  transformer   24 layers at d=2048: QKV 2048x6144, out 2048x2048,
                MLP up 2048x8192, MLP down 8192x2048, LayerNorm vectors 1-D
  root stress   rank-64 + 1e-6 I PSD matrices of 2048x2048
"""
import numpy as np


# ----------------------------------------------------------------------------
# bf16 <-> f32 bit helpers (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits):
    """Exact widening of bfloat16 bits (uint16) to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# Shape lists
# ----------------------------------------------------------------------------
def tiny_shapes():
    return [(256, 128), (128,)]


def uniform_shapes(count=512, n=128):
    return [(n, n)] * count


def resnet50_shapes():
    """ResNet-50: 7x7 stem, bottleneck stages [3, 4, 6, 3] with widths
    64/128/256/512 and 4x expansion, 1x1 projection on the first block of each
    stage, fc 2048 -> 1000.  Every conv is followed by a BatchNorm (weight and
    bias vectors).  Conv weights are (out, in*kh*kw); fc is stored 2048x1000."""
    shapes = []

    def conv_bn(cout, cin, k):
        shapes.append((cout, cin * k * k))
        shapes.append((cout,))
        shapes.append((cout,))

    conv_bn(64, 3, 7)
    cin = 64
    for width, depth in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(depth):
            conv_bn(width, cin, 1)
            conv_bn(width, width, 3)
            conv_bn(width * 4, width, 1)
            if blk == 0:
                conv_bn(width * 4, cin, 1)
            cin = width * 4
    shapes.append((2048, 1000))
    shapes.append((1000,))
    return shapes


def resnet50_conv4d_shapes():
    """The same network with its convolution weights left as (out, in, kh, kw) tensors, the
    form the paper's merging of small dimensions (Sec. 4.2.1) starts from: with block size
    128 a 1 x 1 convolution merges to the matrix (out, in), a 3 x 3 one to the order-3 tensor
    (out, in, 9) and the 7 x 7 stem to (64, 21, 7)."""
    shapes = []
    for s in resnet50_shapes():
        shapes.append(s)
    out, i = [], 0
    # walk the 2-D list again, restoring (cin, k) from the construction order
    def conv_bn(cout, cin, k):
        out.append((cout, cin, k, k))
        out.append((cout,))
        out.append((cout,))
    conv_bn(64, 3, 7)
    cin = 64
    for width, depth in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(depth):
            conv_bn(width, cin, 1)
            conv_bn(width, width, 3)
            conv_bn(width * 4, width, 1)
            if blk == 0:
                conv_bn(width * 4, cin, 1)
            cin = width * 4
    out.append((2048, 1000))
    out.append((1000,))
    assert [numel(a) for a in out] == [numel(b) for b in shapes]
    return out


def transformer_shapes(layers=24, d=2048):
    """Per layer: LayerNorm (w, b), QKV d x 3d, attention out d x d, LayerNorm
    (w, b), MLP up d x 4d, MLP down 4d x d; one final LayerNorm pair."""
    shapes = []
    for _ in range(layers):
        shapes += [(d,), (d,), (d, 3 * d), (d, d), (d,), (d,), (d, 4 * d), (4 * d, d)]
    shapes += [(d,), (d,)]
    return shapes


def numel(shape):
    n = 1
    for s in shape:
        n *= int(s)
    return n


# ----------------------------------------------------------------------------
# Seeded inputs (host side, numpy).  One independent stream per (seed, step,
# parameter index) so any subset can be regenerated on its own.
# ----------------------------------------------------------------------------
def _rng(seed, *keys):
    return np.random.default_rng([int(seed)] + [int(k) for k in keys])


def init_params(shapes, seed, sigma=0.02):
    """W_0 ~ N(0, sigma^2) float32 for every parameter."""
    return [(_rng(seed, 0x57, i).standard_normal(s) * sigma).astype(np.float32)
            for i, s in enumerate(shapes)]


def per_tensor_sigmas(shapes, seed, lo=1e-4, hi=1e-2):
    """One sigma per tensor, log-uniform in [lo, hi]."""
    u = _rng(seed, 0x51).random(len(shapes))
    return np.exp(np.log(lo) + u * (np.log(hi) - np.log(lo)))


def gaussian_grads(shapes, seed, step, sigma):
    """G_t ~ N(0, sigma^2) float32; sigma is a scalar or one value per tensor."""
    sig = np.broadcast_to(np.asarray(sigma, dtype=np.float64), (len(shapes),))
    return [(_rng(seed, 0x47, step, i).standard_normal(s) * sig[i]).astype(np.float32)
            for i, s in enumerate(shapes)]


def psd_stress_matrix(n, rank, seed, index, ridge=1e-6):
    """A = sum_{k<rank} g_k g_k^T + ridge*I with g_k ~ N(0, I_n), formed in
    float64 and rounded once to float32.  Returns (A float32, g float64 n x rank)."""
    g = _rng(seed, 0x53, index).standard_normal((n, rank))
    A = g @ g.T + ridge * np.eye(n)
    return A.astype(np.float32), g


def persistent_subspace_grads(shapes, seed, step, sigma, noise=0.05, decay=1.0):
    """Gradients whose singular vectors persist over the steps, as those of a network in
    training do (the eigenvectors of its Kronecker factors move slowly, which is what a warm
    start of the root-inverse refresh can use): for a matrix parameter
        G_t = sigma (U diag(s_k c_tk) V^T sqrt(min(m, n)) + noise Z_t),
    U, V fixed orthonormal bases drawn once per (seed, parameter), s_k = (k + 1)^(-decay) a fixed
    spectrum, c_tk = 1 + 0.3 N(0, 1) a fresh jitter of every singular value, Z_t fresh N(0, 1)
    noise.  Vectors get plain Gaussian gradients.  float32, one stream per (seed, step, index)."""
    out = []
    for i, s in enumerate(shapes):
        r = _rng(seed, 0x50, step, i)
        if len(s) != 2:
            out.append((r.standard_normal(s) * sigma).astype(np.float32))
            continue
        m, n = s
        k = min(m, n)
        rb = _rng(seed, 0x42, i)                     # the bases do not depend on the step
        U = np.linalg.qr(rb.standard_normal((m, k)))[0]
        V = np.linalg.qr(rb.standard_normal((n, k)))[0]
        sv = (np.arange(k) + 1.0) ** (-decay) * (1.0 + 0.3 * r.standard_normal(k))
        G = (U * sv) @ V.T * np.sqrt(k) + noise * r.standard_normal((m, n))
        out.append((G * sigma).astype(np.float32))
    return out
