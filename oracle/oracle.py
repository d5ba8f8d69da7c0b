"""ctypes front end of the CPU oracle (oracle/sgc_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of the benchmark. Nothing here touches the HIP library, and the
HIP library never calls into this module.

Every function takes and returns numpy arrays on the host. `step` strings the
pieces together in the order of Alg. 2 of the paper for a batch of independent
chunks (MESGC, Sec. 4.4).

`outer_refresh` (the projection matrix of CESGC, Sec. 4.4) lives here rather than in the C file: it
is the definition itself, a singular value decomposition, through numpy's LAPACK routine in double.
Its pins: matrices built from known orthonormal factors and singular values (which must come back
row by row), Eckart-Young optimality against random orthonormal competitors with the singular
values cross-checked through an eigenvalue routine, and a diagonal matrix worked by hand.
The OMP functions follow the plain definition; that App. B's recurrences (which the GPU engines
use) reach the same selections, values and residual is pinned by writing them out in the tests.
Nothing here is "parity unpinned".
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sgc_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (plain -O2, no contraction of a*b+c)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def build_sanitized():
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (any finding aborts), as a separate
    library; a process that wants it sets SGC_ORACLE_LIB to its path and preloads the sanitizer runtime."""
    out = os.path.join(_HERE, "liboracle_san.so")
    if not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-fPIC", "-shared", "-o", out, _SRC, "-lm"]
        )
    return out


def lib():
    global _lib
    if _lib is None:
        override = os.environ.get("SGC_ORACLE_LIB")
        if override:
            _lib = ctypes.CDLL(override)
        else:
            build()
            _lib = ctypes.CDLL(_LIB)
    return _lib


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def topk(g, k):
    """Sparsify_k per chunk (Sec. 4.2, Def. 1). g: [C, d] float32 or uint16 (bf16 bits)."""
    g = np.ascontiguousarray(g)
    C, d = g.shape
    idx = np.empty((C, k), np.int32)
    val = np.empty((C, k), np.float32)
    if g.dtype == np.float32:
        rc = lib().oracle_topk_f32(_p(g, ctypes.c_float), ctypes.c_int64(C), d, k, _p(idx, ctypes.c_int32), _p(val, ctypes.c_float))
    elif g.dtype == np.uint16:
        rc = lib().oracle_topk_bf16(_p(g, ctypes.c_uint16), ctypes.c_int64(C), d, k, _p(idx, ctypes.c_int32), _p(val, ctypes.c_float))
    else:
        raise TypeError(g.dtype)
    if rc:
        raise ValueError("oracle_topk rc=%d" % rc)
    return idx, val


def project(idx, val, At):
    """p = A Sparsify(G), q = A Sparsify(G^2) (eq. 5-6). At: [d, r] float32."""
    idx = _c(idx, np.int32)
    val = _c(val, np.float32)
    At = _c(At, np.float32)
    C, k = idx.shape
    d, r = At.shape
    p = np.empty((C, r), np.float32)
    q = np.empty((C, r), np.float32)
    rc = lib().oracle_project(_p(idx, ctypes.c_int32), _p(val, ctypes.c_float), ctypes.c_int64(C), k, _p(At, ctypes.c_float), d, r, _p(p, ctypes.c_float), _p(q, ctypes.c_float))
    if rc:
        raise ValueError("oracle_project rc=%d" % rc)
    return p, q


def philox4x32_10(ctr, key):
    ctr = _c(ctr, np.uint32)
    key = _c(key, np.uint32)
    out = np.empty(4, np.uint32)
    lib().oracle_philox4x32_10(_p(ctr, ctypes.c_uint32), _p(key, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


def normal_pair(w0, w1, scale=1.0):
    out = np.empty(2, np.float32)
    lib().oracle_normal_pair(ctypes.c_uint32(int(w0)), ctypes.c_uint32(int(w1)), ctypes.c_float(scale), _p(out, ctypes.c_float))
    return out


def philox_matrix(seed, d, r, i0=0, rows=None):
    """Rows [i0, i0+rows) of At for the counter-based matrix (Sec. 4.3 distribution)."""
    rows = d - i0 if rows is None else rows
    out = np.empty((rows, r), np.float32)
    rc = lib().oracle_philox_matrix(ctypes.c_uint64(seed), r, ctypes.c_int64(i0), ctypes.c_int64(rows), _p(out, ctypes.c_float))
    if rc:
        raise ValueError("oracle_philox_matrix rc=%d" % rc)
    return out


def adam(p, q, m, v, step, beta1=0.9, beta2=0.999):
    """Alg. 2 lines 2-5. Returns (m_new, v_new, mhat, vhat); inputs are not modified."""
    p = _c(p, np.float32)
    q = _c(q, np.float32)
    m = np.array(m, np.float32, copy=True, order="C")
    v = np.array(v, np.float32, copy=True, order="C")
    mh = np.empty_like(m)
    vh = np.empty_like(v)
    rc = lib().oracle_adam(_p(p, ctypes.c_float), _p(q, ctypes.c_float), _p(m, ctypes.c_float), _p(v, ctypes.c_float), _p(mh, ctypes.c_float), _p(vh, ctypes.c_float), ctypes.c_int64(m.size), int(step), ctypes.c_double(beta1), ctypes.c_double(beta2))
    if rc:
        raise ValueError("oracle_adam rc=%d" % rc)
    return m, v, mh, vh


def colnorms(At):
    At = _c(At, np.float32)
    d, r = At.shape
    out = np.empty(d, np.float64)
    lib().oracle_colnorms(_p(At, ctypes.c_float), d, r, _p(out, ctypes.c_double))
    return out


def omp(y, At, k, norm=None, forced=None, want_top2=False):
    """OMP_A(y) for one right-hand side (Sec. 4.3 eq. 9).

    Returns dict(sel, x, x64, res, top2). `forced` dictates the first selections.
    """
    y = _c(y, np.float32)
    At = _c(At, np.float32)
    d, r = At.shape
    assert y.shape == (r,)
    sel = np.empty(k, np.int32)
    x = np.empty(k, np.float32)
    x64 = np.empty(k, np.float64)
    res = np.empty(r, np.float64)
    top2 = np.empty(2 * k, np.float64) if want_top2 else None
    norm = _c(norm, np.float64) if norm is not None else None
    forced = _c(forced, np.int32) if forced is not None else None
    nf = 0 if forced is None else forced.size
    rc = lib().oracle_omp(_p(y, ctypes.c_float), _p(At, ctypes.c_float), d, r, k, _p(norm, ctypes.c_double), _p(forced, ctypes.c_int32), nf, _p(sel, ctypes.c_int32), _p(x, ctypes.c_float), _p(x64, ctypes.c_double), _p(res, ctypes.c_double), _p(top2, ctypes.c_double))
    if rc:
        raise ValueError("oracle_omp rc=%d" % rc)
    return dict(sel=sel, x=x, x64=x64, res=res, top2=None if top2 is None else top2.reshape(k, 2))


def omp_batch(Y, At, k):
    Y = _c(Y, np.float32)
    At = _c(At, np.float32)
    N, r = Y.shape
    d = At.shape[0]
    sel = np.empty((N, k), np.int32)
    x = np.empty((N, k), np.float32)
    rc = lib().oracle_omp_batch(_p(Y, ctypes.c_float), N, _p(At, ctypes.c_float), d, r, k, _p(sel, ctypes.c_int32), _p(x, ctypes.c_float))
    if rc:
        raise ValueError("oracle_omp_batch rc=%d" % rc)
    return sel, x


def lstsq_support(y, At, sel):
    """argmin_x || y - A_sel x ||_2 in double (normal equations, Cholesky) on a given support."""
    y = _c(y, np.float32)
    At = _c(At, np.float32)
    sel = _c(sel, np.int32)
    d, r = At.shape
    x64 = np.zeros(sel.size, np.float64)
    rc = lib().oracle_lstsq_support(_p(y, ctypes.c_float), _p(At, ctypes.c_float), d, r, _p(sel, ctypes.c_int32), sel.size, _p(x64, ctypes.c_double))
    if rc:
        raise ValueError("oracle_lstsq_support rc=%d" % rc)
    return x64


def omp_pick(y, At, prefix, norm=None):
    """One iteration of OMP's definition after the selections `prefix`: least squares on the prefix, residual,
    normalised argmax over the unselected positions. Returns dict(lam, top2, res)."""
    y = _c(y, np.float32)
    At = _c(At, np.float32)
    prefix = _c(prefix, np.int32)
    d, r = At.shape
    norm = _c(norm if norm is not None else colnorms(At), np.float64)
    lam = ctypes.c_int32(-1)
    top2 = np.empty(2, np.float64)
    res = np.empty(r, np.float64)
    rc = lib().oracle_omp_pick(_p(y, ctypes.c_float), _p(At, ctypes.c_float), d, r, _p(norm, ctypes.c_double), _p(prefix, ctypes.c_int32), prefix.size, ctypes.byref(lam), _p(top2, ctypes.c_double), _p(res, ctypes.c_double))
    if rc:
        raise ValueError("oracle_omp_pick rc=%d" % rc)
    return dict(lam=int(lam.value), top2=top2, res=res)


def philox_matrix_threads(seed, d, r, workers=8):
    """philox_matrix for a large matrix: row ranges filled by several host threads (the generator is
    counter-based, so the result is the same whatever the split)."""
    from concurrent.futures import ThreadPoolExecutor
    out = np.empty((d, r), np.float32)
    edges = np.linspace(0, d, 4 * workers + 1).astype(np.int64)

    def fill(i):
        a, b = int(edges[i]), int(edges[i + 1])
        if b > a:
            rc = lib().oracle_philox_matrix(ctypes.c_uint64(seed), r, ctypes.c_int64(a), ctypes.c_int64(b - a), _p(out[a:b], ctypes.c_float))
            if rc:
                raise ValueError("oracle_philox_matrix rc=%d" % rc)

    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(fill, range(4 * workers)))
    return out


def omp_shared(Ym, Yv, At, k, norm=None):
    """Shared-support recovery of C chunks: support and x from OMP on Ym[c], z = least-squares fit
    of Yv[c] on that support (Sec. 4.3, the remark after eq. 11). Returns sel, x, z, each [C, k]."""
    Ym = _c(Ym, np.float32)
    Yv = _c(Yv, np.float32)
    At = _c(At, np.float32)
    C, r = Ym.shape
    d = At.shape[0]
    assert Yv.shape == (C, r) and At.shape[1] == r
    norm = _c(norm if norm is not None else colnorms(At), np.float64)
    sel = np.empty((C, k), np.int32)
    x = np.empty((C, k), np.float32)
    z = np.empty((C, k), np.float32)
    for c in range(C):
        rc = lib().oracle_omp_shared(_p(Ym[c], ctypes.c_float), _p(Yv[c], ctypes.c_float), _p(At, ctypes.c_float), d, r, k, _p(norm, ctypes.c_double), _p(sel[c], ctypes.c_int32), _p(x[c], ctypes.c_float), _p(z[c], ctypes.c_float))
        if rc:
            raise ValueError("oracle_omp_shared rc=%d" % rc)
    return sel, x, z


def reproject(sel, x, At_new, scale=1.0):
    """out = scale * A' x for sparse vectors given as (positions, values) (App. C, Alg. 4 l.10-11)."""
    sel = _c(sel, np.int32)
    x = _c(x, np.float32)
    At_new = _c(At_new, np.float32)
    N, k = sel.shape
    d, r = At_new.shape
    out = np.empty((N, r), np.float32)
    rc = lib().oracle_reproject(_p(sel, ctypes.c_int32), _p(x, ctypes.c_float), ctypes.c_int64(N), k, _p(At_new, ctypes.c_float), d, r, ctypes.c_double(scale), _p(out, ctypes.c_float))
    if rc:
        raise ValueError("oracle_reproject rc=%d" % rc)
    return out


def apply(W, d, sel_m, x_m, sel_v, x_v, alpha=1.0, eps=1e-8, lr=1e-3):
    """W <- W - lr * alpha * x / (sqrt(z) + eps) on the recovered supports (eq. 11, eq. 3)."""
    W = np.array(W, np.float32, copy=True, order="C")
    sel_m = _c(sel_m, np.int32)
    sel_v = _c(sel_v, np.int32)
    x_m = _c(x_m, np.float32)
    x_v = _c(x_v, np.float32)
    C, k = sel_m.shape
    assert W.size == C * d
    rc = lib().oracle_apply(_p(W, ctypes.c_float), ctypes.c_int64(C), d, k, _p(sel_m, ctypes.c_int32), _p(x_m, ctypes.c_float), _p(sel_v, ctypes.c_int32), _p(x_v, ctypes.c_float), ctypes.c_double(alpha), ctypes.c_double(eps), ctypes.c_double(lr))
    if rc:
        raise ValueError("oracle_apply rc=%d" % rc)
    return W


def outer_project(B, G):
    """Gc = B G (CESGC, Sec. 4.4). B: [rho, m], G: [m, n] -> [rho, n]."""
    B = _c(B, np.float32)
    G = _c(G, np.float32)
    rho, m = B.shape
    assert G.shape[0] == m
    n = G.shape[1]
    out = np.empty((rho, n), np.float32)
    rc = lib().oracle_outer_project(_p(B, ctypes.c_float), _p(G, ctypes.c_float), rho, m, n, _p(out, ctypes.c_float))
    if rc:
        raise ValueError("oracle_outer_project rc=%d" % rc)
    return out


def outer_apply(W, B, d, sel_m, x_m, sel_v, x_v, alpha=1.0, eps=1e-8, lr=1e-3):
    """W <- W - lr * B^T N with N the update of SGC in the compressed space (CESGC, Sec. 4.4).
    W: [m, n]; the chunks are the row-major rho x n compressed gradient cut in pieces of d."""
    W = np.array(W, np.float32, copy=True, order="C")
    B = _c(B, np.float32)
    sel_m = _c(sel_m, np.int32)
    sel_v = _c(sel_v, np.int32)
    x_m = _c(x_m, np.float32)
    x_v = _c(x_v, np.float32)
    rho, m = B.shape
    n = W.shape[1]
    C, k = sel_m.shape
    assert W.shape[0] == m and C * d == rho * n
    rc = lib().oracle_outer_apply(_p(W, ctypes.c_float), _p(B, ctypes.c_float), rho, m, n, d, k, _p(sel_m, ctypes.c_int32), _p(x_m, ctypes.c_float), _p(sel_v, ctypes.c_int32), _p(x_v, ctypes.c_float), ctypes.c_double(alpha), ctypes.c_double(eps), ctypes.c_double(lr))
    if rc:
        raise ValueError("oracle_outer_apply rc=%d" % rc)
    return W


def outer_refresh(G, rho):
    """The projection matrix of CESGC (Sec. 4.4): the singular value decomposition of the gradient
    matrix G [m, n]; the rho leading left singular vectors are the ROWS of B [rho, m]. Returns (B, sigma)
    with sigma the rho leading singular values, in double. A singular vector's sign is not defined; the
    rows come back with their largest-magnitude entry positive."""
    G = np.asarray(G, np.float64)
    U, s, _ = np.linalg.svd(G, full_matrices=False)
    B = U[:, :rho].T.copy()
    for i in range(B.shape[0]):
        if B[i, np.argmax(np.abs(B[i]))] < 0:
            B[i] = -B[i]
    return B, s[:rho].copy()


def step_cesgc(G, W, B, m, v, t, At, d, k, beta1=0.9, beta2=0.999, eps=1e-8, lr=1e-3, alpha=1.0):
    """One CESGC step (Sec. 4.4) on one weight matrix: compress with B, run Alg. 2 on the chunks of
    the compressed gradient, take the update back with B^T. m, v: [C, r] with C = rho*n/d."""
    Gc = outer_project(B, G)
    C = Gc.size // d
    idx, val = topk(Gc.reshape(C, d), k)
    p, q = project(idx, val, At)
    m2, v2, mh, vh = adam(p, q, m, v, t, beta1, beta2)
    Y = np.concatenate([mh.reshape(C, -1), vh.reshape(C, -1)], axis=0)
    sel, x = omp_batch(Y, At, k)
    W2 = outer_apply(W, B, d, sel[:C], x[:C], sel[C:], x[C:], alpha, eps, lr)
    return dict(Gc=Gc, idx=idx, val=val, p=p, q=q, m=m2, v=v2, mhat=mh, vhat=vh, sel_m=sel[:C], x_m=x[:C], sel_v=sel[C:], x_v=x[C:], W=W2)


def step(g, W, m, v, t, At, k, beta1=0.9, beta2=0.999, eps=1e-8, lr=1e-3, alpha=1.0, shared_support=False,
         At_new=None):
    """One full SGC step (Alg. 2 + the weight update) on C chunks. g: [C, d].
    shared_support: recover the support from mhat only and fit vhat on it.
    At_new: SGCA (App. C): after the update the returned state m, v is re-aligned with the new matrix,
    m = (1 - beta1^t) A' OMP_A(mhat), v = (1 - beta2^t) A' OMP_A(vhat); the caller continues with At_new."""
    C, d = g.shape
    idx, val = topk(g, k)
    p, q = project(idx, val, At)
    m2, v2, mh, vh = adam(p, q, m, v, t, beta1, beta2)
    if shared_support:
        sel_s, x_s, z_s = omp_shared(mh.reshape(C, -1), vh.reshape(C, -1), At, k)
        W2 = apply(W, d, sel_s, x_s, sel_s, z_s, alpha, eps, lr)
        if At_new is not None:
            m2 = reproject(sel_s, x_s, At_new, 1.0 - beta1 ** t)
            v2 = reproject(sel_s, z_s, At_new, 1.0 - beta2 ** t)
        return dict(idx=idx, val=val, p=p, q=q, m=m2, v=v2, mhat=mh, vhat=vh, sel_m=sel_s, x_m=x_s, sel_v=sel_s, x_v=z_s, W=W2)
    Y = np.concatenate([mh.reshape(C, -1), vh.reshape(C, -1)], axis=0)
    sel, x = omp_batch(Y, At, k)
    W2 = apply(W, d, sel[:C], x[:C], sel[C:], x[C:], alpha, eps, lr)
    if At_new is not None:
        m2 = reproject(sel[:C], x[:C], At_new, 1.0 - beta1 ** t)
        v2 = reproject(sel[C:], x[C:], At_new, 1.0 - beta2 ** t)
    return dict(idx=idx, val=val, p=p, q=q, m=m2, v=v2, mhat=mh, vhat=vh, sel_m=sel[:C], x_m=x[:C], sel_v=sel[C:], x_v=x[C:], W=W2)
