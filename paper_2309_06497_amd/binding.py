"""ctypes binding of libshampoo.so: the same entry points as include/shampoo.h.

Argument marshalling only -- every step of the optimizer runs in the HIP
kernels of the library.  PyTorch is used for device memory and streams.
The library is loaded on first use and a missing library is an error: there
is no fallback path.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libshampoo.so")

GRAD_F32, GRAD_BF16 = 0, 1
GET_L, GET_R, GET_LINV, GET_RINV, GET_A, GET_M, GET_PSH, GET_NORMS, GET_GF, GET_L2, GET_L2INV, GET_L3, GET_L3INV = range(13)
MAX_NDIM = 4
GRAFT_ADAGRAD, GRAFT_SGD, GRAFT_RMSPROP, GRAFT_ADAM = 0, 1, 2, 3
ROOT_EIGH, ROOT_NEWTON = 0, 1
LARGE_DIM_BLOCKING, LARGE_DIM_ADAGRAD, LARGE_DIM_DIAGONAL = 0, 1, 2
MATRIX_CORES_AUTO, MATRIX_CORES_FP32 = 0, 1
STAGE_FACTOR, STAGE_GRAFT, STAGE_ROOT, STAGE_PRECOND, STAGE_UPDATE, STAGE_DIAG, STAGE_FUSED, STAGE_PRECOND2 = range(8)
STAGE_NAMES = ("factor", "graft", "root", "precond", "update", "diag", "fused", "precond2")

EXPORTS = (
    "shampoo_plan", "shampoo_workspace_bytes", "shampoo_create", "shampoo_step", "shampoo_get",
    "shampoo_status", "shampoo_set_timing", "shampoo_get_timing", "shampoo_destroy",
    "shampoo_root_inverse_workspace_bytes", "shampoo_root_inverse", "shampoo_root_inverse_static",
    "shampoo_root_inverse_warm_workspace_bytes", "shampoo_root_inverse_warm",
    "shampoo_root_inverse_newton_workspace_bytes", "shampoo_root_inverse_newton", "shampoo_jacobi_pair",
    "shampoo_strerror",
)


class ShampooConfig(ctypes.Structure):
    _fields_ = [
        ("n_params", ctypes.c_int32),
        ("ndim", ctypes.POINTER(ctypes.c_int32)),
        ("shape", ctypes.POINTER(ctypes.c_int64)),
        ("block_size", ctypes.c_int32),
        ("beta2", ctypes.c_float),
        ("epsilon", ctypes.c_float),
        ("root_exponent", ctypes.c_float),
        ("precondition_frequency", ctypes.c_int32),
        ("start_preconditioning_step", ctypes.c_int32),
        ("graft_epsilon", ctypes.c_float),
        ("momentum", ctypes.c_float),
        ("beta1", ctypes.c_float),
        ("weight_decay", ctypes.c_float),
        ("use_decoupled_weight_decay", ctypes.c_int32),
        ("use_nesterov", ctypes.c_int32),
        ("grafting_type", ctypes.c_int32),
        ("grafting_beta2", ctypes.c_float),
        ("use_bias_correction", ctypes.c_int32),
        ("large_dim_method", ctypes.c_int32),
        ("root_method", ctypes.c_int32),
        ("newton_tolerance", ctypes.c_float),
        ("newton_max_iterations", ctypes.c_int32),
        ("precond_matrix_cores", ctypes.c_int32),
        ("warm_start_roots", ctypes.c_int32),
        ("grad_dtype", ctypes.c_int32),
        ("device", ctypes.c_int32),
    ]


_lib = None


def lib():
    """The loaded library (raises OSError if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise OSError(f"{LIB_PATH} not found: build it with `python -m paper_2309_06497_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    cfgp = ctypes.POINTER(ShampooConfig)
    L.shampoo_plan.argtypes = [cfgp, ctypes.POINTER(i64), i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.shampoo_plan.restype = ctypes.c_int
    L.shampoo_workspace_bytes.argtypes = [cfgp]
    L.shampoo_workspace_bytes.restype = sz
    L.shampoo_create.argtypes = [cfgp, vp, sz, vp, ctypes.POINTER(vp)]
    L.shampoo_create.restype = ctypes.c_int
    L.shampoo_step.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), f32, i64, vp]
    L.shampoo_step.restype = ctypes.c_int
    L.shampoo_get.argtypes = [vp, i32, i32, i32, vp, sz, vp]
    L.shampoo_get.restype = ctypes.c_int
    L.shampoo_status.argtypes = [vp, vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.shampoo_status.restype = ctypes.c_int
    L.shampoo_set_timing.argtypes = [vp, i32]
    L.shampoo_set_timing.restype = ctypes.c_int
    L.shampoo_get_timing.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    L.shampoo_get_timing.restype = ctypes.c_int
    L.shampoo_destroy.argtypes = [vp]
    L.shampoo_destroy.restype = ctypes.c_int
    L.shampoo_root_inverse_workspace_bytes.argtypes = [i32, i32]
    L.shampoo_root_inverse_workspace_bytes.restype = sz
    L.shampoo_root_inverse.argtypes = [vp, i32, i32, f32, f32, vp, vp, vp, vp, sz, vp]
    L.shampoo_root_inverse.restype = ctypes.c_int
    L.shampoo_root_inverse_warm_workspace_bytes.argtypes = [i32, i32]
    L.shampoo_root_inverse_warm_workspace_bytes.restype = sz
    L.shampoo_root_inverse_warm.argtypes = [vp, i32, i32, f32, f32, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.shampoo_root_inverse_warm.restype = ctypes.c_int
    L.shampoo_root_inverse_static.argtypes = [vp, i32, i32, f32, f32, vp, vp, vp, vp]
    L.shampoo_root_inverse_static.restype = ctypes.c_int
    L.shampoo_root_inverse_newton_workspace_bytes.argtypes = [i32, i32]
    L.shampoo_root_inverse_newton_workspace_bytes.restype = sz
    L.shampoo_root_inverse_newton.argtypes = [vp, i32, i32, f32, i32, f32, i32, vp, vp, vp, vp, sz, vp]
    L.shampoo_root_inverse_newton.restype = ctypes.c_int
    L.shampoo_jacobi_pair.argtypes = [ctypes.c_int32] * 4 + [ctypes.POINTER(ctypes.c_int32)] * 2
    L.shampoo_jacobi_pair.restype = ctypes.c_int
    L.shampoo_strerror.argtypes = [ctypes.c_int]
    L.shampoo_strerror.restype = ctypes.c_char_p
    _lib = L
    return L


class ShampooError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"libshampoo error {code}: {lib().shampoo_strerror(code).decode()}")


def _check(code):
    if code != 0:
        raise ShampooError(code)


def make_config(shapes, block_size, beta2, epsilon, root_exponent, precondition_frequency,
                start_preconditioning_step=0, graft_epsilon=1e-10, momentum=0.0,
                grad_dtype=GRAD_F32, device=0, beta1=0.0, weight_decay=0.0,
                use_decoupled_weight_decay=True, use_nesterov=False, grafting_type=GRAFT_ADAGRAD,
                use_bias_correction=False, root_method=ROOT_EIGH,
                newton_tolerance=1e-6, newton_max_iterations=100, grafting_beta2=0.999,
                large_dim_method=LARGE_DIM_BLOCKING, precond_matrix_cores=MATRIX_CORES_AUTO,
                warm_start_roots=False):
    """Builds a ShampooConfig; keeps the shape arrays alive on the returned object."""
    n = len(shapes)
    ndim = (ctypes.c_int32 * max(n, 1))(*[len(s) for s in shapes])
    flat = []
    for s in shapes:
        dims = [int(d) for d in s][:MAX_NDIM]
        flat += dims + [1] * (MAX_NDIM - len(dims))
    shape = (ctypes.c_int64 * max(MAX_NDIM * n, 1))(*flat)
    cfg = ShampooConfig(n, ndim, shape, block_size, beta2, epsilon, root_exponent,
                        precondition_frequency, start_preconditioning_step, graft_epsilon,
                        momentum, beta1, weight_decay, 1 if use_decoupled_weight_decay else 0,
                        1 if use_nesterov else 0, grafting_type, grafting_beta2, 1 if use_bias_correction else 0,
                        large_dim_method, root_method, newton_tolerance, newton_max_iterations,
                        precond_matrix_cores, 1 if warm_start_roots else 0, grad_dtype, device)
    cfg._keep = (ndim, shape)
    return cfg


def shampoo_plan(cfg):
    """Returns (table int64 [n_blocks, 12], n_buckets); rows are
    {param, row0, col0, m, n, bucket, slot, flags, s3, d3, s4, d4}.  Host only."""
    nb, nk = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().shampoo_plan(ctypes.byref(cfg), None, 0, ctypes.byref(nb), ctypes.byref(nk)))
    table = np.zeros((max(nb.value, 1), 12), dtype=np.int64)
    _check(lib().shampoo_plan(ctypes.byref(cfg), table.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                              nb.value, ctypes.byref(nb), ctypes.byref(nk)))
    return table[:nb.value], nk.value


def shampoo_workspace_bytes(cfg):
    return lib().shampoo_workspace_bytes(ctypes.byref(cfg))


def _stream_ptr(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


class Shampoo:
    """Owns the workspace tensor and the library handle for one parameter list."""

    def __init__(self, shapes, block_size, beta2, epsilon, root_exponent, precondition_frequency,
                 start_preconditioning_step=0, graft_epsilon=1e-10, momentum=0.0,
                 grad_dtype=GRAD_F32, device=0, beta1=0.0, weight_decay=0.0,
                 use_decoupled_weight_decay=True, use_nesterov=False, grafting_type=GRAFT_ADAGRAD,
                use_bias_correction=False, root_method=ROOT_EIGH,
                newton_tolerance=1e-6, newton_max_iterations=100, grafting_beta2=0.999,
                large_dim_method=LARGE_DIM_BLOCKING, precond_matrix_cores=MATRIX_CORES_AUTO,
                warm_start_roots=False):
        import torch
        self.shapes = [tuple(s) for s in shapes]
        self.cfg = make_config(self.shapes, block_size, beta2, epsilon, root_exponent,
                               precondition_frequency, start_preconditioning_step, graft_epsilon,
                               momentum, grad_dtype, device, beta1, weight_decay,
                               use_decoupled_weight_decay, use_nesterov, grafting_type,
                               use_bias_correction, root_method, newton_tolerance, newton_max_iterations,
                               grafting_beta2, large_dim_method, precond_matrix_cores, warm_start_roots)
        self.device = torch.device("cuda", device)
        self.grad_dtype = grad_dtype
        nbytes = shampoo_workspace_bytes(self.cfg)
        if nbytes == 0:
            raise ShampooError(lib().shampoo_plan(ctypes.byref(self.cfg), None, 0, None, None) or -2)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.handle = ctypes.c_void_p()
        with torch.cuda.device(self.device):
            _check(lib().shampoo_create(ctypes.byref(self.cfg), ctypes.c_void_p(self.workspace.data_ptr()),
                                        nbytes, _stream_ptr(), ctypes.byref(self.handle)))
        self._n = len(self.shapes)
        self._pw = (ctypes.c_void_p * self._n)()
        self._pg = (ctypes.c_void_p * self._n)()

    def step(self, params, grads, lr, step):
        """params / grads: lists of contiguous CUDA tensors (float32 / float32-or-bfloat16)."""
        import torch
        gdt = torch.bfloat16 if self.grad_dtype == GRAD_BF16 else torch.float32
        if len(params) != self._n or len(grads) != self._n:
            raise ValueError("one parameter and one gradient tensor per declared parameter")
        for i in range(self._n):
            w, g = params[i], grads[i]
            if not (w.is_cuda and g.is_cuda and w.device == self.device and g.device == self.device):
                raise ValueError(f"parameter {i}: tensors must live on {self.device}")
            if w.dtype != torch.float32 or g.dtype != gdt:
                raise ValueError(f"parameter {i}: parameters are float32, gradients {gdt}")
            if not (w.is_contiguous() and g.is_contiguous()):
                raise ValueError(f"parameter {i}: tensors must be contiguous")
            if tuple(w.shape) != tuple(self.shapes[i]) or tuple(g.shape) != tuple(self.shapes[i]):
                raise ValueError(f"parameter {i}: shape differs from the one given at creation")
            self._pw[i] = w.data_ptr()
            self._pg[i] = g.data_ptr()
        _check(lib().shampoo_step(self.handle, self._pw, self._pg, lr, step, _stream_ptr()))

    def get(self, param, block, which):
        import torch
        s = self.shapes[param]
        table = self.plan()[0]
        rows = table[table[:, 0] == param] if len(table) else table
        if len(rows) == 0:      # 1-D, or a matrix on the diagonal-method path
            shape = tuple(s)
        else:
            if not 0 <= block < len(rows):
                raise ShampooError(-2)
            m, n, flags, d3, d4 = (int(rows[block, k]) for k in (3, 4, 7, 9, 11))
            if flags & 4:        # a block of a tensor parameter: m x n x d3 (x d4), one factor per dimension
                blk = (m, n, d3, d4) if (flags >> 4) == 4 else (m, n, d3)
                dl = blk[-1]     # R / RINV belong to the last dimension
                shape = {GET_L: (m, m), GET_LINV: (m, m), GET_L2: (n, n), GET_L2INV: (n, n),
                         GET_L3: (d3, d3), GET_L3INV: (d3, d3),
                         GET_R: (dl, dl), GET_RINV: (dl, dl), GET_A: blk, GET_M: blk, GET_PSH: blk,
                         GET_NORMS: (2,), GET_GF: blk}[which]
            else:
                lshape = (m,) if flags & 1 else (m, m)
                rshape = (n,) if flags & 2 else (n, n)
                shape = {GET_L: lshape, GET_LINV: lshape, GET_R: rshape, GET_RINV: rshape,
                         GET_A: (m, n), GET_M: (m, n), GET_PSH: (m, n), GET_NORMS: (2,), GET_GF: (m, n)}[which]
        out = torch.empty(shape, dtype=torch.float32, device=self.device)
        _check(lib().shampoo_get(self.handle, param, block, which, ctypes.c_void_p(out.data_ptr()),
                                 out.numel() * 4, _stream_ptr()))
        return out

    def plan(self):
        if not hasattr(self, "_plan"):
            self._plan = shampoo_plan(self.cfg)
        return self._plan

    def status(self):
        a, b = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(lib().shampoo_status(self.handle, _stream_ptr(), ctypes.byref(a), ctypes.byref(b)))
        return {"refreshes": a.value, "failed_roots": b.value}

    def set_timing(self, enable):
        _check(lib().shampoo_set_timing(self.handle, 1 if enable else 0))

    def get_timing(self):
        """{stage name: (total ms, intervals)} since the last call."""
        out = {}
        for st, name in enumerate(STAGE_NAMES):
            ms, cnt = ctypes.c_double(0), ctypes.c_int64(0)
            _check(lib().shampoo_get_timing(self.handle, st, ctypes.byref(ms), ctypes.byref(cnt)))
            out[name] = (ms.value, cnt.value)
        return out

    def destroy(self):
        if self.handle:
            lib().shampoo_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def shampoo_root_inverse(a, epsilon, r, want_lambda=False, want_failed=False):
    """a: CUDA float32 tensor [batch, n, n] (symmetric).  Returns X [batch, n, n]
    (and eigenvalues [batch, n], failure flags [batch] on request)."""
    import torch
    assert a.is_cuda and a.dtype == torch.float32 and a.dim() == 3 and a.shape[1] == a.shape[2]
    a = a.contiguous()
    batch, n = a.shape[0], a.shape[1]
    x = torch.empty_like(a)
    lam = torch.empty((batch, n), dtype=torch.float32, device=a.device) if want_lambda else None
    failed = torch.zeros((batch,), dtype=torch.int32, device=a.device) if want_failed else None
    nbytes = lib().shampoo_root_inverse_workspace_bytes(n, batch)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=a.device)
    with torch.cuda.device(a.device):
        _check(lib().shampoo_root_inverse(
            ctypes.c_void_p(a.data_ptr()), n, batch, epsilon, r, ctypes.c_void_p(x.data_ptr()),
            ctypes.c_void_p(lam.data_ptr()) if lam is not None else None,
            ctypes.c_void_p(failed.data_ptr()) if failed is not None else None,
            ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream_ptr()))
        torch.cuda.current_stream().synchronize()   # ws is released on return
    res = [x]
    if want_lambda:
        res.append(lam)
    if want_failed:
        res.append(failed)
    return res[0] if len(res) == 1 else tuple(res)


def shampoo_root_inverse_warm(a, epsilon, r, qt, start):
    """shampoo_root_inverse with the eigenvectors kept in qt ([batch, np, np] float32 CUDA tensor,
    np = n rounded up to 64) between calls; start: begin from them.  Returns
    (X, eigenvalues, failed, sweeps)."""
    import torch
    assert a.is_cuda and a.dtype == torch.float32 and a.dim() == 3 and a.shape[1] == a.shape[2]
    a = a.contiguous()
    batch, n = a.shape[0], a.shape[1]
    npad = (n + 63) // 64 * 64
    assert qt.is_cuda and qt.dtype == torch.float32 and tuple(qt.shape) == (batch, npad, npad) and qt.is_contiguous()
    x = torch.empty_like(a)
    lam = torch.empty((batch, n), dtype=torch.float32, device=a.device)
    failed = torch.zeros((batch,), dtype=torch.int32, device=a.device)
    sweeps = torch.zeros((batch,), dtype=torch.int32, device=a.device)
    nbytes = lib().shampoo_root_inverse_warm_workspace_bytes(n, batch)
    if nbytes == 0:
        raise ShampooError(-7)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=a.device)
    with torch.cuda.device(a.device):
        _check(lib().shampoo_root_inverse_warm(
            ctypes.c_void_p(a.data_ptr()), n, batch, epsilon, r, ctypes.c_void_p(x.data_ptr()),
            ctypes.c_void_p(lam.data_ptr()), ctypes.c_void_p(failed.data_ptr()), ctypes.c_void_p(qt.data_ptr()),
            1 if start else 0, ctypes.c_void_p(sweeps.data_ptr()), ctypes.c_void_p(ws.data_ptr()), ws.numel(),
            _stream_ptr()))
        torch.cuda.current_stream().synchronize()   # ws is released on return
    return x, lam, failed, sweeps


def shampoo_root_inverse_static(a, epsilon, r, x, lam=None, failed=None):
    """shampoo_root_inverse without a workspace (the library's fixed scratch array is used):
    a, x: CUDA float32 tensors [batch, n, n]; lam [batch, n] float32 and failed [batch] int32
    optional.  Outputs are written into the tensors given: nothing is allocated here either.
    Asynchronous on the current stream."""
    import torch
    assert a.is_cuda and a.dtype == torch.float32 and a.dim() == 3 and a.shape[1] == a.shape[2] and a.is_contiguous()
    assert x.is_cuda and x.dtype == torch.float32 and x.shape == a.shape and x.is_contiguous()
    batch, n = a.shape[0], a.shape[1]
    assert lam is None or (lam.dtype == torch.float32 and lam.shape == (batch, n) and lam.is_contiguous())
    assert failed is None or (failed.dtype == torch.int32 and failed.shape == (batch,) and failed.is_contiguous())
    with torch.cuda.device(a.device):
        _check(lib().shampoo_root_inverse_static(
            ctypes.c_void_p(a.data_ptr()), n, batch, epsilon, r, ctypes.c_void_p(x.data_ptr()),
            ctypes.c_void_p(lam.data_ptr()) if lam is not None else None,
            ctypes.c_void_p(failed.data_ptr()) if failed is not None else None, _stream_ptr()))


def shampoo_jacobi_pair(s, halves, rnd, k):
    """(p, q), p < q: pair k of round rnd of the eigensolver's sweep over s indices (host only)."""
    p, q = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().shampoo_jacobi_pair(s, int(halves), rnd, k, ctypes.byref(p), ctypes.byref(q)))
    return p.value, q.value


def shampoo_root_inverse_newton(a, epsilon, p, tolerance=1e-6, max_iterations=100, want_iterations=False,
                                want_failed=False):
    """a: CUDA float32 tensor [batch, n, n] (symmetric).  Returns X [batch, n, n], the coupled
    inverse Newton approximation of (a + epsilon I)^(-1/p) (and the iteration counts [batch],
    failure flags [batch] on request)."""
    import torch
    assert a.is_cuda and a.dtype == torch.float32 and a.dim() == 3 and a.shape[1] == a.shape[2]
    a = a.contiguous()
    batch, n = a.shape[0], a.shape[1]
    x = torch.empty_like(a)
    iters = torch.zeros((batch,), dtype=torch.int32, device=a.device) if want_iterations else None
    failed = torch.zeros((batch,), dtype=torch.int32, device=a.device) if want_failed else None
    nbytes = lib().shampoo_root_inverse_newton_workspace_bytes(n, batch)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=a.device)
    with torch.cuda.device(a.device):
        _check(lib().shampoo_root_inverse_newton(
            ctypes.c_void_p(a.data_ptr()), n, batch, epsilon, p, tolerance, max_iterations,
            ctypes.c_void_p(x.data_ptr()),
            ctypes.c_void_p(iters.data_ptr()) if iters is not None else None,
            ctypes.c_void_p(failed.data_ptr()) if failed is not None else None,
            ctypes.c_void_p(ws.data_ptr()), ws.numel(), _stream_ptr()))
        torch.cuda.current_stream().synchronize()   # ws is released on return
    res = [x]
    if want_iterations:
        res.append(iters)
    if want_failed:
        res.append(failed)
    return res[0] if len(res) == 1 else tuple(res)
