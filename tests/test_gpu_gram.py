"""The optional Gram table (App. B precomputes A^H A): the table itself against a float64 product,
and the recovery with the table against the CPU oracle and against the recovery without it."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2502_00311_amd import sgc, synth

pytestmark = pytest.mark.gpu
TOL = 1e-4
DEV = "cuda"


def say(*a):
    print(*a, flush=True)


def relerr(a, ref):
    a = np.asarray(a, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    return 0.0 if a.size == 0 else float(np.abs(a - ref).max() / (den if den > 0 else 1.0))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def make_matrix(mode, seed, d, r, gram=True):
    if mode == "stored":
        At = synth.gaussian_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=dev(At))
    else:
        At = orc.philox_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=None, seed=seed)
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    if gram:
        G = torch.empty((d, d), dtype=torch.float64, device=DEV)
        sgc.sgc_matrix_gram(A, G)
        A.gram = G
    return A, At


def run_omp(Y, A, k):
    N, r = Y.shape
    sel = torch.empty((N, k), dtype=torch.int32, device=DEV)
    x = torch.empty((N, k), dtype=torch.float32, device=DEV)
    ws = torch.empty(sgc.sgc_omp_workspace_bytes_for(N, k, A), dtype=torch.uint8, device=DEV)
    sgc.sgc_recover_omp(dev(Y), N, A, k, sel, x, ws)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), x.cpu().numpy()


@pytest.mark.parametrize("d,r,mode", [(1, 4, "stored"), (100, 8, "stored"), (300, 40, "philox"), (1000, 132, "stored"),
                                      (257, 1024, "philox")])
def test_gram_table_equals_float64_product(d, r, mode):
    say("gram", d, r, mode)
    A, At = make_matrix(mode, 51, d, r)
    torch.cuda.synchronize()
    A64 = At.astype(np.float64)
    ref = A64 @ A64.T
    got = A.gram.cpu().numpy()
    assert np.abs(got - ref).max() <= 1e-13 * np.abs(ref).max()
    assert np.array_equal(got, got.T)


@pytest.mark.parametrize("N,d,r,k,mode", [
    (1, 100, 16, 4, "stored"),
    (5, 1000, 96, 12, "philox"),
    (2, 4096, 256, 32, "stored"),
    (130, 768, 64, 8, "stored"),     # full position tiles, ragged tile of right-hand sides
    (2, 2048, 512, 320, "stored"),
])
def test_omp_with_gram_table_matches_oracle(N, d, r, k, mode):
    say("omp+gram", N, d, r, k, mode)
    rng = np.random.default_rng(N * 5 + d)
    A, At = make_matrix(mode, 22, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    if N > 2:
        Y[1] = 0.0
    sel, x = run_omp(Y, A, k)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    for n in range(N):
        assert relerr(x[n], rx[n]) < TOL, n
    # and the same supports as without the table
    A.gram = None
    sel2, x2 = run_omp(Y, A, k)
    assert np.array_equal(sel, sel2)
    for n in range(N):
        assert relerr(x[n], x2[n]) < 1e-6, n


def test_full_steps_with_gram_table_and_shared_support():
    w = synth.shrink(synth.CFG2, C=3, d=4096, r=256, k=32)
    A, At = make_matrix(w.matrix, w.a_seed, w.d, w.r)
    buf = sgc.StepBuffers(w.C, w.d, w.r, w.k)
    W = dev(synth.weights(w))
    h = sgc.hyper()
    C = w.C
    for t in range(1, 4):
        g = synth.gradients(w, t)
        shared = t == 3
        sgc.step(dev(g), W, buf, A, t, h, shared_support=shared)
        torch.cuda.synchronize()
        mh, vh = buf.hat[:C].cpu().numpy(), buf.hat[C:].cpu().numpy()
        sel, x = buf.sel.cpu().numpy(), buf.x.cpu().numpy()
        if shared:
            rsel, rx, rz = orc.omp_shared(mh, vh, At, w.k)
            assert np.array_equal(sel[:C], rsel)
            for c in range(C):
                assert relerr(x[c], rx[c]) < TOL and relerr(x[C + c], rz[c]) < TOL
        else:
            rsel, rx = orc.omp_batch(np.concatenate([mh, vh]), At, w.k)
            assert np.array_equal(sel, rsel)
            for n in range(2 * C):
                assert relerr(x[n], rx[n]) < TOL
