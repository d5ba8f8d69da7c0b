"""sgc_recover_omp_static (the recovery for callers that cannot allocate: workspace in a static device
array) against sgc_recover_omp with a caller workspace, through the raw C ABI: two calls in a row on the
same GPU, the second with a smaller input, plus a third that reuses the array after a generated matrix
has left its column copies there. Same kernels, same inputs: supports and values must be identical; the
first call is also checked against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2502_00311_amd import sgc, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(*a):
    print(*a, flush=True)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def matrix(mode, seed, d, r):
    if mode == "stored":
        At = synth.gaussian_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=dev(At))
    else:
        At = orc.philox_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=None, seed=seed)
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    return A, At


def both(Y, A, k):
    """(sel, x) of the static-workspace entry point and of the caller-workspace one, raw C ABI."""
    L = sgc.lib()
    N, r = Y.shape
    y = dev(Y)
    cA = A.c()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    sel_s = torch.full((N, k), -1, dtype=torch.int32, device=DEV)
    x_s = torch.full((N, k), float("nan"), dtype=torch.float32, device=DEV)
    st = L.sgc_recover_omp_static(ctypes.c_void_p(y.data_ptr()), N, ctypes.byref(cA), k, ctypes.c_void_p(sel_s.data_ptr()),
                                  ctypes.c_void_p(x_s.data_ptr()), stream)
    assert st == sgc.OK, sgc.status_string(st)
    torch.cuda.synchronize()
    nbytes = L.sgc_omp_workspace_bytes_for(N, k, ctypes.byref(cA))
    assert 0 < nbytes <= L.sgc_omp_static_workspace_bytes()
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    sel = torch.empty((N, k), dtype=torch.int32, device=DEV)
    x = torch.empty((N, k), dtype=torch.float32, device=DEV)
    st = L.sgc_recover_omp(ctypes.c_void_p(y.data_ptr()), N, ctypes.byref(cA), k, ctypes.c_void_p(sel.data_ptr()),
                           ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(ws.data_ptr()), nbytes, stream)
    assert st == sgc.OK, sgc.status_string(st)
    torch.cuda.synchronize()
    return sel_s.cpu().numpy(), x_s.cpu().numpy(), sel.cpu().numpy(), x.cpu().numpy()


def test_static_workspace_recovery_two_calls_in_a_row_then_a_third():
    rng = np.random.default_rng(2024)
    # first call: cfg1's shape with a few right-hand sides, stored matrix
    say("static workspace, call 1: N=6 d=4096 r=256 k=32 stored")
    A1, At1 = matrix("stored", 1, 4096, 256)
    Y1 = rng.standard_normal((6, 256)).astype(np.float32)
    sel_s, x_s, sel, x = both(Y1, A1, 32)
    assert np.array_equal(sel_s, sel) and np.array_equal(x_s, x)
    norm = orc.colnorms(At1)
    for n in range(6):
        ref = orc.omp(Y1[n], At1, 32, norm=norm)
        assert np.array_equal(sel_s[n], ref["sel"])
        assert np.abs(x_s[n] - ref["x"]).max() <= 1e-4 * np.abs(ref["x"]).max()
    # second call, smaller input, generated matrix (its column copies and panel land in the array too)
    say("static workspace, call 2: N=3 d=1000 r=64 k=8 generated")
    A2, At2 = matrix("philox", 9, 1000, 64)
    Y2 = rng.standard_normal((3, 64)).astype(np.float32)
    sel_s, x_s, sel, x = both(Y2, A2, 8)
    assert np.array_equal(sel_s, sel) and np.array_equal(x_s, x)
    norm = orc.colnorms(At2)
    for n in range(3):
        ref = orc.omp(Y2[n], At2, 8, norm=norm)
        assert np.array_equal(sel_s[n], ref["sel"])
        assert np.abs(x_s[n] - ref["x"]).max() <= 1e-4 * np.abs(ref["x"]).max()
    # third call: the first input again, over whatever the second call left in the array
    say("static workspace, call 3: the first input again")
    sel_s3, x_s3, _, _ = both(Y1, A1, 32)
    sel_s1, x_s1, _, _ = both(Y1[:2], A1, 32)
    for n in range(6):
        assert np.array_equal(sel_s3[n], orc.omp(Y1[n], At1, 32, norm=orc.colnorms(At1))["sel"])
    assert np.array_equal(sel_s1, sel_s3[:2]) and np.array_equal(x_s1, x_s3[:2])


def test_static_workspace_refuses_what_does_not_fit():
    L = sgc.lib()
    A, _ = matrix("philox", 3, 16384, 1024)     # generated: column copies of 64 x 1024 floats per right-hand side
    N, k = 256, 64
    assert L.sgc_omp_workspace_bytes_for(N, k, ctypes.byref(A.c())) > L.sgc_omp_static_workspace_bytes()
    y = torch.zeros((N, 1024), dtype=torch.float32, device=DEV)
    sel = torch.full((N, k), -7, dtype=torch.int32, device=DEV)
    x = torch.zeros((N, k), dtype=torch.float32, device=DEV)
    with pytest.raises(sgc.SgcError) as e:
        sgc.sgc_recover_omp_static(y, N, A, k, sel, x)
    assert e.value.status == sgc.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((sel == -7).all())              # nothing was launched
