"""Host-side checks of the C ABI: the library loads, exports every function the header declares,
and rejects bad arguments before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2502_00311_amd import sgc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sgc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sgc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    L = sgc.lib()
    names = declared_functions()
    assert set(names) == set(sgc.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert sgc.status_string(0) == "ok"
    for s in range(-7, 0):
        assert sgc.status_string(s) not in ("ok", "unknown status")
    assert sgc.status_string(-99) == "unknown status"


FAKE = ctypes.c_void_p(0x1000)      # aligned, never dereferenced: validation fails first
ODD = ctypes.c_void_p(0x1004)


def mat(mode=0, d=64, r=16, At=0x1000, inv=0x1000, seed=1, gram=None):
    return sgc.sgc_matrix(mode, d, r, 0, seed, At, inv, gram)


def test_sparsify_project_rejects_bad_arguments():
    L = sgc.lib()
    f = L.sgc_sparsify_project
    A = mat()
    ok_args = dict(grad=FAKE, gt=0, n=128, d=64, k=4, A=ctypes.byref(A), idx=FAKE, val=FAKE, p=FAKE, q=FAKE)

    def call(**kw):
        a = dict(ok_args, **kw)
        return f(a["grad"], a["gt"], a["n"], a["d"], a["k"], a["A"], a["idx"], a["val"], a["p"], a["q"], None)

    assert call(grad=None) == sgc.ERR_NULL
    assert call(idx=None) == sgc.ERR_NULL
    assert call(p=None) == sgc.ERR_NULL
    assert call(A=None) == sgc.ERR_NULL
    assert call(gt=7) == sgc.ERR_DTYPE
    assert call(k=0) == sgc.ERR_SHAPE
    assert call(k=65) == sgc.ERR_SHAPE          # k > d
    assert call(k=17) == sgc.ERR_SHAPE          # k > r
    assert call(n=100) == sgc.ERR_SHAPE         # n % d
    assert call(d=32) == sgc.ERR_SHAPE          # d != A.d
    assert call(grad=ODD) == sgc.ERR_ALIGN
    assert call(p=ODD) == sgc.ERR_ALIGN
    bad = mat(r=18)
    assert call(A=ctypes.byref(bad)) == sgc.ERR_SHAPE
    bad = mat(mode=5)
    assert call(A=ctypes.byref(bad)) == sgc.ERR_DTYPE
    bad = mat(At=None)
    assert call(A=ctypes.byref(bad)) == sgc.ERR_NULL
    bad = mat(At=0x1004)
    assert call(A=ctypes.byref(bad)) == sgc.ERR_ALIGN


def test_adam_rejects_bad_arguments():
    L = sgc.lib()
    h = sgc.hyper()

    def call(p=FAKE, q=FAKE, m=FAKE, v=FAKE, mh=FAKE, vh=FAKE, count=16, step=1, hh=h):
        return L.sgc_adam_compressed(p, q, m, v, mh, vh, count, step, ctypes.byref(hh) if hh is not None else None, None)

    assert call(m=None) == sgc.ERR_NULL
    assert call(hh=None) == sgc.ERR_NULL
    assert call(count=-1) == sgc.ERR_SHAPE
    assert call(step=0) == sgc.ERR_STEP
    assert call(hh=sgc.hyper(beta1=1.0)) == sgc.ERR_STEP
    assert call(hh=sgc.hyper(beta2=-0.1)) == sgc.ERR_STEP
    assert call(v=ODD) == sgc.ERR_ALIGN


def test_omp_rejects_bad_arguments_and_sizes_workspace():
    L = sgc.lib()
    A = mat(d=4096, r=256)
    need = sgc.sgc_omp_workspace_bytes(2, 4096, 256, 32)
    assert need > 2 * 32 * 256 * 4
    assert sgc.sgc_omp_workspace_bytes(0, 4096, 256, 32) == 0
    assert sgc.sgc_omp_workspace_bytes(2, 4096, 250, 32) == 0     # r % 4
    assert sgc.sgc_omp_workspace_bytes(2, 4096, 256, 300) == 0    # k > r
    # workspace grows with every dimension
    assert sgc.sgc_omp_workspace_bytes(4, 4096, 256, 32) > need
    assert sgc.sgc_omp_workspace_bytes(2, 8192, 256, 32) > need
    assert sgc.sgc_omp_workspace_bytes(2, 4096, 512, 32) > need
    assert sgc.sgc_omp_workspace_bytes(2, 4096, 256, 64) > need

    def call(y=FAKE, N=2, AA=A, k=32, sel=FAKE, x=FAKE, ws=FAKE, nbytes=need):
        return L.sgc_recover_omp(y, N, ctypes.byref(AA) if AA is not None else None, k, sel, x, ws, nbytes, None)

    assert call(y=None) == sgc.ERR_NULL
    assert call(ws=None) == sgc.ERR_NULL
    assert call(AA=None) == sgc.ERR_NULL
    assert call(AA=mat(d=4096, r=256, inv=None)) == sgc.ERR_NULL
    assert call(N=0) == sgc.ERR_SHAPE
    assert call(k=0) == sgc.ERR_SHAPE
    assert call(k=257) == sgc.ERR_SHAPE
    # the exact need depends on the matrix: a stored one is read in place (no column copies, no panel), the
    # bfloat16 planes of the screening contraction are counted only for a matrix that asks for them
    exact = L.sgc_omp_workspace_bytes_for(2, 32, ctypes.byref(A))
    gen = mat(mode=1, d=4096, r=256)
    assert 0 < exact < L.sgc_omp_workspace_bytes_for(2, 32, ctypes.byref(gen)) == need
    scr = sgc.sgc_matrix(0, 4096, 256, sgc.MATRIX_FLAG_SCREEN_BF16, 1, 0x1000, 0x1000, None)
    assert L.sgc_omp_workspace_bytes_for(2, 32, ctypes.byref(scr)) >= exact + 4096 * 256 * 4
    assert L.sgc_omp_workspace_bytes_for(2, 300, ctypes.byref(A)) == 0 and L.sgc_omp_workspace_bytes_for(2, 32, None) == 0
    assert call(nbytes=exact - 1) == sgc.ERR_WORKSPACE
    assert call(AA=gen, nbytes=need - 1) == sgc.ERR_WORKSPACE
    assert call(AA=scr, nbytes=exact) == sgc.ERR_WORKSPACE         # sized without the planes
    assert call(ws=ctypes.c_void_p(0x1010)) == sgc.ERR_ALIGN

    # the variant with the workspace in a static device array: same checks, and sizes beyond the array are refused
    cap = L.sgc_omp_static_workspace_bytes()
    assert cap == 32 << 20

    def stat(y=FAKE, N=2, AA=A, k=32, sel=FAKE, x=FAKE):
        return L.sgc_recover_omp_static(y, N, ctypes.byref(AA) if AA is not None else None, k, sel, x, None)

    assert stat(y=None) == sgc.ERR_NULL and stat(sel=None) == sgc.ERR_NULL and stat(AA=None) == sgc.ERR_NULL
    assert stat(AA=mat(d=4096, r=256, inv=None)) == sgc.ERR_NULL
    assert stat(N=0) == sgc.ERR_SHAPE and stat(k=257) == sgc.ERR_SHAPE
    assert stat(y=ODD) == sgc.ERR_ALIGN
    big = mat(d=65536, r=2048)
    assert L.sgc_omp_workspace_bytes_for(128, 256, ctypes.byref(big)) > cap
    assert stat(N=128, AA=big, k=256) == sgc.ERR_WORKSPACE

    # the engine with App. B's recurrence: the same checks, a larger workspace, and the Gram table is required
    more = sgc.sgc_omp_recurrence_workspace_bytes(2, 4096, 256, 32)
    assert more >= need + 2 * 33 * 4096 * 4
    assert need + 2 * 9 * 4096 * 4 <= sgc.sgc_omp_recurrence_workspace_bytes(2, 4096, 256, 32, 8) < more
    assert sgc.sgc_omp_recurrence_workspace_bytes(2, 4098, 256, 32) == 0   # d % 4
    assert sgc.sgc_omp_recurrence_workspace_bytes(2, 4096, 256, 300) == 0
    assert sgc.sgc_omp_recurrence_workspace_bytes(2, 4096, 256, 32, 0) == 0 and sgc.sgc_omp_recurrence_workspace_bytes(2, 4096, 256, 32, 33) == 0

    def rec(y=FAKE, N=2, AA=None, k=32, head=32, ws=FAKE, nbytes=more):
        AA = AA if AA is not None else mat(d=4096, r=256, gram=0x1000)
        return L.sgc_recover_omp_recurrence(y, N, ctypes.byref(AA), k, head, FAKE, FAKE, ws, nbytes, None)

    assert rec(y=None) == sgc.ERR_NULL
    assert rec(AA=mat(d=4096, r=256)) == sgc.ERR_NULL              # no table
    assert rec(k=0) == sgc.ERR_SHAPE and rec(N=0) == sgc.ERR_SHAPE
    assert rec(head=0) == sgc.ERR_SHAPE and rec(head=33) == sgc.ERR_SHAPE
    assert rec(AA=mat(d=4098, r=256, gram=0x1000)) == sgc.ERR_SHAPE  # d % 4
    assert rec(nbytes=need) == sgc.ERR_WORKSPACE                   # sized for the plain recovery
    # a generated matrix that does not fit the workspace's panel whole (256 MB of rows, few right-hand sides)
    big_ws = sgc.sgc_omp_recurrence_workspace_bytes(2, 1 << 20, 64, 4)
    assert big_ws > 0
    assert L.sgc_recover_omp_recurrence(FAKE, 2, ctypes.byref(mat(mode=1, d=1 << 20, r=64, gram=0x1000)), 4, 4, FAKE, FAKE,
                                        FAKE, big_ws, None) == sgc.ERR_SHAPE
    assert rec(ws=ctypes.c_void_p(0x1010)) == sgc.ERR_ALIGN


def test_apply_and_matrix_helpers_reject_bad_arguments():
    L = sgc.lib()
    h = sgc.hyper()
    assert L.sgc_apply(None, 1, 64, 4, FAKE, FAKE, FAKE, FAKE, ctypes.byref(h), None) == sgc.ERR_NULL
    assert L.sgc_apply(FAKE, 1, 64, 0, FAKE, FAKE, FAKE, FAKE, ctypes.byref(h), None) == sgc.ERR_SHAPE
    assert L.sgc_apply(FAKE, 1, 64, 65, FAKE, FAKE, FAKE, FAKE, ctypes.byref(h), None) == sgc.ERR_SHAPE
    assert L.sgc_apply(FAKE, -1, 64, 4, FAKE, FAKE, FAKE, FAKE, ctypes.byref(h), None) == sgc.ERR_SHAPE
    assert L.sgc_matrix_fill(1, 16, 0, 4, None, None) == sgc.ERR_NULL
    assert L.sgc_matrix_fill(1, 18, 0, 4, FAKE, None) == sgc.ERR_SHAPE
    assert L.sgc_matrix_fill(1, 16, 0, -4, FAKE, None) == sgc.ERR_SHAPE
    A = mat()
    assert L.sgc_matrix_colnorms(ctypes.byref(A), None, None) == sgc.ERR_NULL
    assert L.sgc_matrix_colnorms(None, FAKE, None) == sgc.ERR_NULL


def test_shared_recovery_and_reprojection_reject_bad_arguments():
    L = sgc.lib()
    A = mat(d=4096, r=256)
    need = sgc.sgc_omp_workspace_bytes(2, 4096, 256, 32)

    def shared(ym=FAKE, yv=FAKE, C=2, AA=A, k=32, sel=FAKE, x=FAKE, z=FAKE, ws=FAKE, nbytes=need):
        return L.sgc_recover_omp_shared(ym, yv, C, ctypes.byref(AA) if AA is not None else None, k, sel, x, z, ws, nbytes, None)

    assert shared(yv=None) == sgc.ERR_NULL
    assert shared(z=None) == sgc.ERR_NULL
    assert shared(AA=mat(d=4096, r=256, inv=None)) == sgc.ERR_NULL
    assert shared(C=0) == sgc.ERR_SHAPE
    assert shared(k=1025) == sgc.ERR_SHAPE
    assert shared(yv=ODD) == sgc.ERR_ALIGN
    assert shared(nbytes=L.sgc_omp_workspace_bytes_for(2, 32, ctypes.byref(A)) - 1) == sgc.ERR_WORKSPACE

    def reproject(sel=FAKE, x=FAKE, N=2, k=8, AA=A, scale=0.5, out=FAKE):
        return L.sgc_reproject(sel, x, N, k, ctypes.byref(AA) if AA is not None else None, scale, out, None)

    assert reproject(sel=None) == sgc.ERR_NULL
    assert reproject(out=None) == sgc.ERR_NULL
    assert reproject(AA=None) == sgc.ERR_NULL
    assert reproject(N=-1) == sgc.ERR_SHAPE
    assert reproject(k=0) == sgc.ERR_SHAPE
    assert reproject(k=4097) == sgc.ERR_SHAPE
    assert reproject(out=ODD) == sgc.ERR_ALIGN
    assert reproject(AA=mat(mode=9)) == sgc.ERR_DTYPE

    def moment(beta=0.9, step=3, out=FAKE, sel=FAKE):
        return L.sgc_reproject_moment(sel, FAKE, 2, 8, ctypes.byref(A), beta, step, out, None)

    assert moment(step=0) == sgc.ERR_STEP and moment(beta=1.0) == sgc.ERR_STEP and moment(beta=-0.5) == sgc.ERR_STEP
    assert moment(sel=None) == sgc.ERR_NULL and moment(out=ODD) == sgc.ERR_ALIGN

    # the machine probes validate like everything else
    assert L.sgc_probe(99, FAKE, FAKE, 1024, 1, 1, None) == sgc.ERR_DTYPE
    assert L.sgc_probe(sgc.PROBE_READ, None, FAKE, 1024, 1, 1, None) == sgc.ERR_NULL
    assert L.sgc_probe(sgc.PROBE_VALU, None, None, 0, 1, 1, None) == sgc.ERR_NULL
    assert L.sgc_probe(sgc.PROBE_VALU, None, FAKE, 0, 0, 1, None) == sgc.ERR_SHAPE
    assert L.sgc_probe(sgc.PROBE_COPY, ODD, FAKE, 1024, 1, 1, None) == sgc.ERR_ALIGN


def test_gram_rejects_bad_arguments():
    L = sgc.lib()
    A = mat()
    assert L.sgc_matrix_gram(ctypes.byref(A), None, None) == sgc.ERR_NULL
    assert L.sgc_matrix_gram(None, FAKE, None) == sgc.ERR_NULL
    assert L.sgc_matrix_gram(ctypes.byref(A), ODD, None) == sgc.ERR_ALIGN
    big = mat(mode=1, d=65537, r=16, At=None)
    assert L.sgc_matrix_gram(ctypes.byref(big), FAKE, None) == sgc.ERR_SHAPE
    bad = mat(r=18)
    assert L.sgc_matrix_gram(ctypes.byref(bad), FAKE, None) == sgc.ERR_SHAPE


def test_outer_projection_rejects_bad_arguments_and_sizes_workspace():
    L = sgc.lib()
    nbytes = sgc.sgc_outer_workspace_bytes(1, 32, 4096, 4096)
    assert nbytes >= 32 * 4096 * 4 and nbytes % 256 == 0
    assert sgc.sgc_outer_workspace_bytes(16, 32, 4096, 4096) >= 16 * 32 * 4096 * 4
    assert sgc.sgc_outer_workspace_bytes(1, 0, 8, 8) == 0
    assert sgc.sgc_outer_workspace_bytes(0, 4, 8, 8) == 0
    assert sgc.sgc_outer_workspace_bytes(1, 4, 8, 6) == 0          # n % 4
    assert sgc.sgc_outer_workspace_bytes(1, 4, 8, 1 << 23) == 0
    assert sgc.sgc_outer_workspace_bytes(70000, 4, 8, 8) == 0      # batch beyond the grid limit
    small = sgc.sgc_outer_workspace_bytes(1, 4, 8, 8)
    p = L.sgc_outer_project
    assert p(None, FAKE, 0, 1, 4, 8, 8, FAKE, FAKE, small, None) == sgc.ERR_NULL
    assert p(FAKE, FAKE, 0, 1, 4, 8, 8, FAKE, None, small, None) == sgc.ERR_NULL
    assert p(FAKE, FAKE, 0, 1, 4, 8, 6, FAKE, FAKE, small, None) == sgc.ERR_SHAPE
    assert p(FAKE, FAKE, 5, 1, 4, 8, 8, FAKE, FAKE, small, None) == sgc.ERR_DTYPE
    assert p(FAKE, FAKE, 0, 1, 0, 8, 8, FAKE, FAKE, small, None) == sgc.ERR_SHAPE
    assert p(FAKE, FAKE, 1, 0, 4, 8, 8, FAKE, FAKE, small, None) == sgc.ERR_SHAPE
    assert p(FAKE, ODD, 0, 1, 4, 8, 8, FAKE, FAKE, small, None) == sgc.ERR_ALIGN
    assert p(FAKE, FAKE, 0, 1, 4, 8, 8, FAKE, ODD, small, None) == sgc.ERR_ALIGN
    assert p(FAKE, FAKE, 1, 1, 4, 8, 8, FAKE, FAKE, small - 1, None) == sgc.ERR_WORKSPACE
    one = sgc.sgc_outer_workspace_bytes(1, 4, 8, 256)
    assert p(FAKE, FAKE, 0, 2, 4, 8, 256, FAKE, FAKE, one, None) == sgc.ERR_WORKSPACE  # sized for one matrix
    a = L.sgc_outer_apply
    h = sgc.hyper()

    def call(W=FAKE, B=FAKE, count=1, rho=4, m=8, n=8, d=16, k=2, sel=FAKE, hh=ctypes.byref(h), ws=FAKE, nb=small):
        return a(W, B, count, rho, m, n, d, k, sel, FAKE, FAKE, FAKE, hh, ws, nb, None)

    assert call(W=None) == sgc.ERR_NULL
    assert call(sel=None) == sgc.ERR_NULL
    assert call(hh=None) == sgc.ERR_NULL
    assert call(count=0) == sgc.ERR_SHAPE
    assert call(d=5) == sgc.ERR_SHAPE           # rho * n not a multiple of d
    assert call(k=0) == sgc.ERR_SHAPE
    assert call(k=17) == sgc.ERR_SHAPE          # k > d
    assert call(W=ODD) == sgc.ERR_ALIGN
    assert call(nb=small - 1) == sgc.ERR_WORKSPACE
    # the renewal of B: sizes are validated before anything touches the device
    f = L.sgc_outer_refresh
    need = sgc.sgc_outer_refresh_workspace_bytes(1, 4, 64, 128)
    assert need > 64 * 128 * 4 + 4 * 128 * 4                      # a transposed copy of G and a rho x n matrix
    assert sgc.sgc_outer_refresh_workspace_bytes(1, 4, 64, 128, sgc.GRAD_BF16) == need - 64 * 128 * 2
    assert sgc.sgc_outer_refresh_workspace_bytes(3, 4, 64, 128) > 2 * need
    for bad in ((1, 65, 64, 128), (1, 0, 64, 128), (1, 4, 62, 128), (1, 4, 64, 126), (1, 8, 4, 128), (1, 8, 128, 4),
                (1, 4, 64, 1 << 23), (0, 4, 64, 128), (70000, 4, 64, 128)):
        assert sgc.sgc_outer_refresh_workspace_bytes(*bad) == 0, bad
    assert sgc.sgc_outer_refresh_workspace_bytes(1, 4, 64, 128, 7) == 0

    def fresh(B=FAKE, G=FAKE, gt=0, count=1, rho=4, m=64, n=128, iters=2, ws=FAKE, nb=need):
        return f(B, G, gt, count, rho, m, n, iters, None, ws, nb, None)

    assert fresh(B=None) == sgc.ERR_NULL and fresh(G=None) == sgc.ERR_NULL and fresh(ws=None) == sgc.ERR_NULL
    assert fresh(gt=3) == sgc.ERR_DTYPE
    assert fresh(rho=65) == sgc.ERR_SHAPE and fresh(m=62) == sgc.ERR_SHAPE and fresh(n=126) == sgc.ERR_SHAPE
    assert fresh(iters=-1) == sgc.ERR_SHAPE and fresh(iters=1001) == sgc.ERR_SHAPE
    assert fresh(B=ODD) == sgc.ERR_ALIGN and fresh(G=ODD) == sgc.ERR_ALIGN and fresh(ws=ODD) == sgc.ERR_ALIGN
    assert fresh(nb=need - 1) == sgc.ERR_WORKSPACE and fresh(count=2) == sgc.ERR_WORKSPACE and fresh(count=0) == sgc.ERR_SHAPE


def test_binding_rejects_tensors_of_the_wrong_element_type():
    """The C ABI takes untyped pointers; the binding refuses what would be read as garbage (no GPU needed:
    the check comes before the library is called)."""
    import torch
    g64 = torch.zeros((4, 8), dtype=torch.float64)
    f32 = torch.zeros((4, 8), dtype=torch.float32)
    with pytest.raises(TypeError):
        sgc.sgc_outer_project(f32, g64, 1, 4, 4, 8, f32, f32)
    with pytest.raises(TypeError):
        sgc.sgc_outer_refresh(f32, g64, 1, 4, 4, 8, 1, None, f32)
    with pytest.raises(TypeError):
        sgc.sgc_recover_omp(g64, 4, None, 1, f32, f32, f32)
    with pytest.raises(TypeError):
        sgc.sgc_sparsify_project(g64, 32, 8, 1, None, f32, f32, f32, f32)
