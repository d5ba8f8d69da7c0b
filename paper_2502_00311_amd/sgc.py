"""Thin binding over the C ABI of libsgc.so (include/sgc.h): argument marshalling only.

Function names and argument order mirror the C entry points. Tensors are torch tensors on the
GPU (torch is used for device memory and streams, nothing else); every step of the path runs in
the HIP kernels. There is no fallback: a missing library or a failing call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libsgc.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_ALIGN, ERR_WORKSPACE, ERR_STEP, ERR_DEVICE = -1, -2, -3, -4, -5, -6, -7
GRAD_F32, GRAD_BF16 = 0, 1
MATRIX_STORED, MATRIX_PHILOX = 0, 1
MATRIX_FLAG_SCREEN_BF16 = 1
MATRIX_FLAG_MATERIALIZE = 2
MATRIX_FLAG_MULTI_LAUNCH = 4

EXPORTS = [
    "sgc_status_string", "sgc_matrix_fill", "sgc_matrix_colnorms", "sgc_matrix_gram", "sgc_sparsify_project",
    "sgc_adam_compressed", "sgc_omp_workspace_bytes", "sgc_omp_workspace_bytes_for", "sgc_recover_omp",
    "sgc_omp_static_workspace_bytes", "sgc_recover_omp_static", "sgc_recover_omp_shared", "sgc_reproject",
    "sgc_reproject_moment",
    "sgc_omp_recurrence_workspace_bytes", "sgc_recover_omp_recurrence",
    "sgc_apply", "sgc_outer_workspace_bytes", "sgc_outer_project", "sgc_outer_apply",
    "sgc_outer_refresh_workspace_bytes", "sgc_outer_refresh",
    "sgc_profile_enable", "sgc_profile_read", "sgc_probe",
]
PROBE_VALU, PROBE_MFMA, PROBE_READ, PROBE_RW44, PROBE_COPY, PROBE_MFMA_VALU4, PROBE_MFMA_VALU8 = 0, 1, 2, 3, 4, 5, 6
PROBE_SPLIT_BOTH, PROBE_SPLIT_MFMA, PROBE_SPLIT_VALU = 7, 8, 9
PROFILE_CLASSES = ["topk", "project", "adam", "omp_corr", "omp_select_update", "apply", "other", "omp_matrix_fill",
                   "outer_project", "outer_apply", "outer_refresh"]


class sgc_matrix(ctypes.Structure):
    _fields_ = [
        ("mode", ctypes.c_int32), ("d", ctypes.c_int32), ("r", ctypes.c_int32), ("flags", ctypes.c_int32),
        ("seed", ctypes.c_uint64), ("At", ctypes.c_void_p), ("inv_colnorm", ctypes.c_void_p),
        ("gram", ctypes.c_void_p),
    ]


class sgc_hyper(ctypes.Structure):
    _fields_ = [("beta1", ctypes.c_double), ("beta2", ctypes.c_double), ("eps", ctypes.c_double),
                ("lr", ctypes.c_double), ("alpha", ctypes.c_double)]


class sgc_profile(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double * len(PROFILE_CLASSES)), ("launches", ctypes.c_int64 * len(PROFILE_CLASSES))]


class SgcError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, status_string(status)))


_lib = None


def lib():
    """Load libsgc.so (built in-tree by csrc/build.py). Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libsgc.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_size_t
        L.sgc_status_string.restype = ctypes.c_char_p
        L.sgc_status_string.argtypes = [i32]
        L.sgc_matrix_fill.restype = i32
        L.sgc_matrix_fill.argtypes = [u64, i32, i64, i64, vp, vp]
        L.sgc_matrix_colnorms.restype = i32
        L.sgc_matrix_colnorms.argtypes = [ctypes.POINTER(sgc_matrix), vp, vp]
        L.sgc_matrix_gram.restype = i32
        L.sgc_matrix_gram.argtypes = [ctypes.POINTER(sgc_matrix), vp, vp]
        L.sgc_sparsify_project.restype = i32
        L.sgc_sparsify_project.argtypes = [vp, i32, i64, i32, i32, ctypes.POINTER(sgc_matrix), vp, vp, vp, vp, vp]
        L.sgc_adam_compressed.restype = i32
        L.sgc_adam_compressed.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, ctypes.POINTER(sgc_hyper), vp]
        L.sgc_omp_workspace_bytes.restype = sz
        L.sgc_omp_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.sgc_omp_workspace_bytes_for.restype = sz
        L.sgc_omp_workspace_bytes_for.argtypes = [i32, i32, ctypes.POINTER(sgc_matrix)]
        L.sgc_recover_omp.restype = i32
        L.sgc_recover_omp.argtypes = [vp, i32, ctypes.POINTER(sgc_matrix), i32, vp, vp, vp, sz, vp]
        L.sgc_omp_static_workspace_bytes.restype = sz
        L.sgc_omp_static_workspace_bytes.argtypes = []
        L.sgc_recover_omp_static.restype = i32
        L.sgc_recover_omp_static.argtypes = [vp, i32, ctypes.POINTER(sgc_matrix), i32, vp, vp, vp]
        L.sgc_reproject_moment.restype = i32
        L.sgc_reproject_moment.argtypes = [vp, vp, i64, i32, ctypes.POINTER(sgc_matrix), ctypes.c_double, i32, vp, vp]
        L.sgc_omp_recurrence_workspace_bytes.restype = sz
        L.sgc_omp_recurrence_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.sgc_recover_omp_recurrence.restype = i32
        L.sgc_recover_omp_recurrence.argtypes = [vp, i32, ctypes.POINTER(sgc_matrix), i32, i32, vp, vp, vp, sz, vp]
        L.sgc_recover_omp_shared.restype = i32
        L.sgc_recover_omp_shared.argtypes = [vp, vp, i32, ctypes.POINTER(sgc_matrix), i32, vp, vp, vp, vp, sz, vp]
        L.sgc_reproject.restype = i32
        L.sgc_reproject.argtypes = [vp, vp, i64, i32, ctypes.POINTER(sgc_matrix), ctypes.c_double, vp, vp]
        L.sgc_apply.restype = i32
        L.sgc_apply.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, ctypes.POINTER(sgc_hyper), vp]
        L.sgc_outer_workspace_bytes.restype = sz
        L.sgc_outer_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.sgc_outer_project.restype = i32
        L.sgc_outer_project.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
        L.sgc_outer_refresh_workspace_bytes.restype = sz
        L.sgc_outer_refresh_workspace_bytes.argtypes = [i32, i32, i32, i32, i32]
        L.sgc_outer_refresh.restype = i32
        L.sgc_outer_refresh.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, sz, vp]
        L.sgc_outer_apply.restype = i32
        L.sgc_outer_apply.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, ctypes.POINTER(sgc_hyper), vp, sz, vp]
        L.sgc_probe.restype = i32
        L.sgc_probe.argtypes = [i32, vp, vp, i64, i32, i32, vp]
        L.sgc_profile_enable.restype = i32
        L.sgc_profile_enable.argtypes = [i32]
        L.sgc_profile_read.restype = i32
        L.sgc_profile_read.argtypes = [ctypes.POINTER(sgc_profile)]
        _lib = L
    return _lib


def status_string(status):
    return lib().sgc_status_string(int(status)).decode()


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


_GRAD_DTYPES = (torch.float32, torch.bfloat16, torch.int16, torch.uint16)


def _expect(t, dtypes, what):
    """The C ABI takes untyped pointers: a tensor of another element type would be read as garbage."""
    if t is not None and t.dtype not in dtypes:
        raise TypeError("%s must be %s, got %s" % (what, " or ".join(str(x) for x in dtypes), t.dtype))


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status, where):
    if status != OK:
        raise SgcError(status, where)


def hyper(beta1=0.9, beta2=0.999, eps=1e-8, lr=1e-3, alpha=1.0):
    return sgc_hyper(beta1, beta2, eps, lr, alpha)


class Matrix:
    """Host-side descriptor of the measurement matrix plus the device buffers it points to."""

    def __init__(self, d, r, At=None, seed=0, inv_colnorm=None, gram=None):
        self.d, self.r, self.seed = int(d), int(r), int(seed)
        self.At = At                    # torch [d, r] float32 on the GPU, or None (generated)
        self.inv_colnorm = inv_colnorm  # torch [d] float32 on the GPU, or None
        self.gram = gram                # torch [d, d] float64 on the GPU, or None
        self.flags = 0                  # MATRIX_FLAG_*
        self.mode = MATRIX_STORED if At is not None else MATRIX_PHILOX

    def c(self):
        return sgc_matrix(self.mode, self.d, self.r, self.flags, self.seed,
                          self.At.data_ptr() if self.At is not None else None,
                          self.inv_colnorm.data_ptr() if self.inv_colnorm is not None else None,
                          self.gram.data_ptr() if self.gram is not None else None)


def sgc_matrix_fill(seed, r, row0, rows, At_out, stream=None):
    _check(lib().sgc_matrix_fill(seed, r, row0, rows, _ptr(At_out), _stream(stream)), "sgc_matrix_fill")


def sgc_matrix_colnorms(A, inv_colnorm_out, stream=None):
    _check(lib().sgc_matrix_colnorms(ctypes.byref(A.c()), _ptr(inv_colnorm_out), _stream(stream)), "sgc_matrix_colnorms")


def sgc_matrix_gram(A, gram_out, stream=None):
    _check(lib().sgc_matrix_gram(ctypes.byref(A.c()), _ptr(gram_out), _stream(stream)), "sgc_matrix_gram")


def sgc_sparsify_project(grad, n, d, k, A, idx, val, p, q, stream=None):
    _expect(grad, _GRAD_DTYPES, "grad")
    _expect(idx, (torch.int32,), "idx")
    for t, nm in ((val, "val"), (p, "p"), (q, "q")):
        _expect(t, (torch.float32,), nm)
    gt = GRAD_BF16 if grad.dtype in (torch.bfloat16, torch.int16, torch.uint16) else GRAD_F32
    _check(lib().sgc_sparsify_project(_ptr(grad), gt, n, d, k, ctypes.byref(A.c()), _ptr(idx), _ptr(val), _ptr(p), _ptr(q), _stream(stream)), "sgc_sparsify_project")


def sgc_adam_compressed(p, q, m, v, mhat, vhat, count, step, h, stream=None):
    _check(lib().sgc_adam_compressed(_ptr(p), _ptr(q), _ptr(m), _ptr(v), _ptr(mhat), _ptr(vhat), count, step, ctypes.byref(h), _stream(stream)), "sgc_adam_compressed")


def sgc_omp_workspace_bytes(N, d, r, k):
    return int(lib().sgc_omp_workspace_bytes(N, d, r, k))


def sgc_recover_omp(y, N, A, k, sel, x, ws, stream=None):
    _expect(y, (torch.float32,), "y")
    _expect(sel, (torch.int32,), "sel")
    _expect(x, (torch.float32,), "x")
    _check(lib().sgc_recover_omp(_ptr(y), N, ctypes.byref(A.c()), k, _ptr(sel), _ptr(x), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "sgc_recover_omp")


def sgc_omp_workspace_bytes_for(N, k, A):
    return int(lib().sgc_omp_workspace_bytes_for(N, k, ctypes.byref(A.c())))


def sgc_omp_static_workspace_bytes():
    return int(lib().sgc_omp_static_workspace_bytes())


def sgc_recover_omp_static(y, N, A, k, sel, x, stream=None):
    _expect(y, (torch.float32,), "y")
    _expect(sel, (torch.int32,), "sel")
    _expect(x, (torch.float32,), "x")
    _check(lib().sgc_recover_omp_static(_ptr(y), N, ctypes.byref(A.c()), k, _ptr(sel), _ptr(x), _stream(stream)), "sgc_recover_omp_static")


def sgc_omp_recurrence_workspace_bytes(N, d, r, k, head=None):
    return int(lib().sgc_omp_recurrence_workspace_bytes(N, d, r, k, k if head is None else head))


def sgc_recover_omp_recurrence(y, N, A, k, sel, x, ws, stream=None, head=None):
    """head: iterations served by the recurrence (default: all k)."""
    _expect(y, (torch.float32,), "y")
    _expect(sel, (torch.int32,), "sel")
    _expect(x, (torch.float32,), "x")
    _expect(A.gram, (torch.float64,), "A.gram")
    _check(lib().sgc_recover_omp_recurrence(_ptr(y), N, ctypes.byref(A.c()), k, k if head is None else head, _ptr(sel), _ptr(x), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "sgc_recover_omp_recurrence")


def sgc_recover_omp_shared(y_m, y_v, C, A, k, sel, x, z, ws, stream=None):
    _check(lib().sgc_recover_omp_shared(_ptr(y_m), _ptr(y_v), C, ctypes.byref(A.c()), k, _ptr(sel), _ptr(x), _ptr(z), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "sgc_recover_omp_shared")


def sgc_reproject(sel, x, N, k, A_new, scale, out, stream=None):
    _check(lib().sgc_reproject(_ptr(sel), _ptr(x), N, k, ctypes.byref(A_new.c()), scale, _ptr(out), _stream(stream)), "sgc_reproject")


def sgc_reproject_moment(sel, x, N, k, A_new, beta, step, out, stream=None):
    _check(lib().sgc_reproject_moment(_ptr(sel), _ptr(x), N, k, ctypes.byref(A_new.c()), beta, step, _ptr(out), _stream(stream)), "sgc_reproject_moment")


def sgc_apply(W, C, d, k, sel_m, x_m, sel_v, x_v, h, stream=None):
    _check(lib().sgc_apply(_ptr(W), C, d, k, _ptr(sel_m), _ptr(x_m), _ptr(sel_v), _ptr(x_v), ctypes.byref(h), _stream(stream)), "sgc_apply")


def sgc_outer_workspace_bytes(count, rho, m, n):
    return int(lib().sgc_outer_workspace_bytes(count, rho, m, n))


def sgc_outer_project(B, G, count, rho, m, n, Gc, ws, stream=None):
    _expect(G, _GRAD_DTYPES, "G")
    _expect(B, (torch.float32,), "B")
    _expect(Gc, (torch.float32,), "Gc")
    gt = GRAD_BF16 if G.dtype in (torch.bfloat16, torch.int16, torch.uint16) else GRAD_F32
    _check(lib().sgc_outer_project(_ptr(B), _ptr(G), gt, count, rho, m, n, _ptr(Gc), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "sgc_outer_project")


def sgc_outer_apply(W, B, count, rho, m, n, d, k, sel_m, x_m, sel_v, x_v, h, ws, stream=None):
    _expect(W, (torch.float32,), "W")
    _expect(B, (torch.float32,), "B")
    _check(lib().sgc_outer_apply(_ptr(W), _ptr(B), count, rho, m, n, d, k, _ptr(sel_m), _ptr(x_m), _ptr(sel_v), _ptr(x_v), ctypes.byref(h), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "sgc_outer_apply")


def sgc_outer_refresh_workspace_bytes(count, rho, m, n, grad_type=GRAD_F32):
    return int(lib().sgc_outer_refresh_workspace_bytes(count, rho, m, n, grad_type))


def sgc_outer_refresh(B, G, count, rho, m, n, iters, sigma, ws, stream=None):
    _expect(G, _GRAD_DTYPES, "G")
    _expect(B, (torch.float32,), "B")
    _expect(sigma, (torch.float32,), "sigma")
    gt = GRAD_BF16 if G.dtype in (torch.bfloat16, torch.int16, torch.uint16) else GRAD_F32
    _check(lib().sgc_outer_refresh(_ptr(B), _ptr(G), gt, count, rho, m, n, iters, _ptr(sigma) if sigma is not None else None,
                                   _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "sgc_outer_refresh")


def sgc_probe(kind, a, b, nbytes, blocks, iters, stream=None):
    _check(lib().sgc_probe(kind, _ptr(a), _ptr(b), nbytes, blocks, iters, _stream(stream)), "sgc_probe")


def sgc_profile_enable(on):
    _check(lib().sgc_profile_enable(1 if on else 0), "sgc_profile_enable")


def sgc_profile_read():
    """{class name: (total ms, launches)} of the kernels launched since sgc_profile_enable(True)."""
    out = sgc_profile()
    _check(lib().sgc_profile_read(ctypes.byref(out)), "sgc_profile_read")
    return {n: (out.ms[i], out.launches[i]) for i, n in enumerate(PROFILE_CLASSES)}


class StepBuffers:
    """Device buffers of one SGC step on C chunks (allocation only; no arithmetic)."""

    def __init__(self, C, d, r, k, device="cuda", recurrence=False, screen=False, flags=0):
        f32, i32 = torch.float32, torch.int32
        self.C, self.d, self.r, self.k = C, d, r, k
        # recurrence: False, True (all k iterations) or the number of iterations the recurrence serves; the
        # workspace is then sized for sgc_recover_omp_recurrence, which step() calls
        self.recurrence = (k if recurrence is True else int(recurrence)) if recurrence else 0
        self.idx = torch.empty((C, k), dtype=i32, device=device)
        self.val = torch.empty((C, k), dtype=f32, device=device)
        self.p = torch.empty((C, r), dtype=f32, device=device)
        self.q = torch.empty((C, r), dtype=f32, device=device)
        self.m = torch.zeros((C, r), dtype=f32, device=device)
        self.v = torch.zeros((C, r), dtype=f32, device=device)
        self.hat = torch.empty((2 * C, r), dtype=f32, device=device)  # [mhat; vhat]
        self.sel = torch.empty((2 * C, k), dtype=i32, device=device)
        self.x = torch.empty((2 * C, k), dtype=f32, device=device)
        # screen: the matrix will carry MATRIX_FLAG_SCREEN_BF16, whose bfloat16 planes take 4 d r bytes more
        if self.recurrence:
            nbytes = sgc_omp_recurrence_workspace_bytes(2 * C, d, r, k, self.recurrence)
        elif screen or flags:
            probe = Matrix(d, r, seed=0)
            probe.flags = flags | (MATRIX_FLAG_SCREEN_BF16 if screen else 0)
            nbytes = sgc_omp_workspace_bytes_for(2 * C, k, probe)
        else:
            nbytes = sgc_omp_workspace_bytes(2 * C, d, r, k)
        if nbytes == 0:
            raise SgcError(ERR_SHAPE, "sgc_omp_workspace_bytes")
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)


def step(grad, W, buf, A, t, h, stream=None, shared_support=False, A_new=None):
    """The four calls of one step, in order (Alg. 2 then the weight update). shared_support: one
    support per chunk from mhat with vhat fitted on it; then buf.sel[:C], buf.x[:C] hold the support
    and x, buf.x[C:] holds z, and buf.sel[C:] is not written. A_new: SGCA (App. C): after the update
    the state buf.m, buf.v is re-aligned with A_new from the vectors just recovered; the caller passes
    A_new as A from the next step on."""
    C, d, r, k = buf.C, buf.d, buf.r, buf.k
    sgc_sparsify_project(grad, C * d, d, k, A, buf.idx, buf.val, buf.p, buf.q, stream)
    sgc_adam_compressed(buf.p, buf.q, buf.m, buf.v, buf.hat[:C], buf.hat[C:], C * r, t, h, stream)
    if shared_support:
        sgc_recover_omp_shared(buf.hat[:C], buf.hat[C:], C, A, k, buf.sel[:C], buf.x[:C], buf.x[C:], buf.ws, stream)
        sgc_apply(W, C, d, k, buf.sel[:C], buf.x[:C], buf.sel[:C], buf.x[C:], h, stream)
        if A_new is not None:
            sgc_reproject_moment(buf.sel[:C], buf.x[:C], C, k, A_new, h.beta1, t, buf.m, stream)
            sgc_reproject_moment(buf.sel[:C], buf.x[C:], C, k, A_new, h.beta2, t, buf.v, stream)
        return
    if buf.recurrence:
        sgc_recover_omp_recurrence(buf.hat, 2 * C, A, k, buf.sel, buf.x, buf.ws, stream, head=buf.recurrence)
    else:
        sgc_recover_omp(buf.hat, 2 * C, A, k, buf.sel, buf.x, buf.ws, stream)
    sgc_apply(W, C, d, k, buf.sel[:C], buf.x[:C], buf.sel[C:], buf.x[C:], h, stream)
    if A_new is not None:
        sgc_reproject_moment(buf.sel[:C], buf.x[:C], C, k, A_new, h.beta1, t, buf.m, stream)
        sgc_reproject_moment(buf.sel[C:], buf.x[C:], C, k, A_new, h.beta2, t, buf.v, stream)


class OuterBuffers:
    """Device buffers of the outer projection of CESGC for a batch of `count` m x n weight matrices
    (allocation only)."""

    def __init__(self, rho, m, n, count=1, device="cuda"):
        self.rho, self.m, self.n, self.count = rho, m, n, count
        self.Gc = torch.empty((count, rho, n) if count > 1 else (rho, n), dtype=torch.float32, device=device)
        nbytes = sgc_outer_workspace_bytes(count, rho, m, n)
        if nbytes == 0:
            raise SgcError(ERR_SHAPE, "sgc_outer_workspace_bytes")
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=device)


def step_cesgc(G, W, B, obuf, buf, A, t, h, stream=None):
    """One CESGC step (Sec. 4.4) on a batch of equal weight matrices ([count, m, n], or [m, n] for one):
    Gc = B G, Alg. 2 on the chunks of Gc, then W <- W - lr B^T N. buf: StepBuffers for count*rho*n/d
    chunks."""
    rho, m, n, count = obuf.rho, obuf.m, obuf.n, obuf.count
    C, d, r, k = buf.C, buf.d, buf.r, buf.k
    sgc_outer_project(B, G, count, rho, m, n, obuf.Gc, obuf.ws, stream)
    sgc_sparsify_project(obuf.Gc, C * d, d, k, A, buf.idx, buf.val, buf.p, buf.q, stream)
    sgc_adam_compressed(buf.p, buf.q, buf.m, buf.v, buf.hat[:C], buf.hat[C:], C * r, t, h, stream)
    sgc_recover_omp(buf.hat, 2 * C, A, k, buf.sel, buf.x, buf.ws, stream)
    sgc_outer_apply(W, B, count, rho, m, n, d, k, buf.sel[:C], buf.x[:C], buf.sel[C:], buf.x[C:], h, obuf.ws, stream)
