"""The recovery with App. B's correlation recurrence (Alg. 3: Gram table, p <- p - b a, no contraction inside
the iterations) against the CPU oracle and against the recovery with the contraction: the same supports bit
for bit, the same values (the least squares is the same code once the selections agree)."""
import ctypes

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


def make_matrix(mode, seed, d, r):
    if mode == "stored":
        At = synth.gaussian_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=dev(At))
    else:
        At = orc.philox_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=None, seed=seed)
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    G = torch.empty((d, d), dtype=torch.float64, device=DEV)
    sgc.sgc_matrix_gram(A, G)
    A.gram = G
    return A, At


def run(Y, A, k, recurrence, head=None):
    N, r = Y.shape
    sel = torch.empty((N, k), dtype=torch.int32, device=DEV)
    x = torch.empty((N, k), dtype=torch.float32, device=DEV)
    if recurrence:
        ws = torch.empty(sgc.sgc_omp_recurrence_workspace_bytes(N, A.d, r, k, head), dtype=torch.uint8, device=DEV)
        sgc.sgc_recover_omp_recurrence(dev(Y), N, A, k, sel, x, ws, head=head)
    else:
        ws = torch.empty(sgc.sgc_omp_workspace_bytes_for(N, k, A), dtype=torch.uint8, device=DEV)
        sgc.sgc_recover_omp(dev(Y), N, A, k, sel, x, ws)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), x.cpu().numpy()


@pytest.mark.parametrize("N,d,r,k,mode", [
    (1, 100, 16, 4, "stored"),         # one ragged tile
    (5, 1000, 96, 12, "philox"),       # generated matrix (written to the workspace panel), ragged tiles
    (2, 4096, 256, 32, "stored"),      # cfg1 shape
    (130, 768, 64, 8, "stored"),       # more than one tile of right-hand sides of the first contraction
    (3, 5004, 128, 16, "philox"),      # several workgroups per right-hand side, the last one ragged
    (2, 2048, 512, 320, "stored"),     # 320 updates of the float vector in a row
    (70, 16384, 64, 6, "stored"),      # 16 workgroups per right-hand side
])
def test_recurrence_matches_oracle_and_contraction(N, d, r, k, mode):
    say("recurrence", N, d, r, k, mode)
    rng = np.random.default_rng(N * 7 + d)
    A, At = make_matrix(mode, 23, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    if N > 2:
        Y[1] = 0.0                                   # exact ties: lowest positions, values 0
        Y[2] *= 1e-20                                # tiny scale
    sel, x = run(Y, A, k, True)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    for n in range(N):
        assert relerr(x[n], rx[n]) < TOL, n
    sel2, x2 = run(Y, A, k, False)
    assert np.array_equal(sel, sel2)
    assert np.array_equal(x.view(np.uint32), x2.view(np.uint32))
    # the recurrence for the first iterations only, the contraction after: the same again
    for head in sorted({1, max(1, k // 3), k - 1} - {0, k}):
        sel3, x3 = run(Y, A, k, True, head=head)
        assert np.array_equal(sel, sel3), head
        assert np.array_equal(x.view(np.uint32), x3.view(np.uint32)), head


@pytest.mark.parametrize("flags", [0, sgc.MATRIX_FLAG_SCREEN_BF16], ids=["float", "screen_bf16"])
def test_recurrence_head_then_pipelined_contraction(flags):
    # full tiles and enough of them for the hand-scheduled contraction kernels to take over after the head
    rng = np.random.default_rng(29)
    N, d, r, k, head = 130, 32768, 64, 6, 3
    A, At = make_matrix("stored", 31, d, r)
    A.flags = flags
    Y = rng.standard_normal((N, r)).astype(np.float32)
    sel, x = run(Y, A, k, True, head=head)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    for n in range(N):
        assert relerr(x[n], rx[n]) < TOL, n


def test_recurrence_at_benchmark_shape_agrees_with_the_contraction_engine():
    # configuration 3's shape (d = 16384, r = 1024, k = 64, generated matrix) on 192 right-hand sides with the
    # heavy tails of the benchmark's moments: 64 updates of p per right-hand side, every selection identical.
    # (The contraction engine is checked against the oracle at this size in test_gpu_full_size.py.)
    rng = np.random.default_rng(17)
    N, d, r, k = 192, 16384, 1024, 64
    A, _ = make_matrix("philox", 9, d, r)
    Y = (rng.standard_t(3.0, size=(N, r)) * 1e-3).astype(np.float32)
    Y[N // 2:] = np.abs(Y[N // 2:]) * 1e-3               # like second moments: non-negative, much smaller
    sel, x = run(Y, A, k, True)
    sel2, x2 = run(Y, A, k, False)
    assert np.array_equal(sel, sel2)
    assert np.array_equal(x.view(np.uint32), x2.view(np.uint32))
    # sampled right-hand sides against the oracle itself
    At = orc.philox_matrix(9, d, r)
    for n in (0, 77, 100, 191):
        rsel, rx = orc.omp_batch(Y[n:n + 1], At, k)
        assert np.array_equal(sel[n], rsel[0]), n
        assert relerr(x[n], rx[0]) < TOL, n


def test_recurrence_exact_recovery():
    # k-sparse vectors measured without noise, k iterations: every pick is made on a residual far above rounding
    rng = np.random.default_rng(3)
    N, d, r, k = 6, 2048, 256, 8
    A, At = make_matrix("stored", 4, d, r)
    X = np.zeros((N, d), np.float32)
    supp = [np.sort(rng.permutation(d)[:k]) for _ in range(N)]
    for n in range(N):
        X[n, supp[n]] = rng.standard_normal(k).astype(np.float32) + np.sign(rng.standard_normal(k)).astype(np.float32)
    Y = (X.astype(np.float64) @ At.astype(np.float64)).astype(np.float32)
    sel, x = run(Y, A, k, True)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    for n in range(N):
        assert np.array_equal(np.sort(sel[n]), supp[n])
        assert relerr(x[n], X[n, sel[n]]) < 1e-5


def test_recurrence_with_iterations_to_spare_stays_valid():
    # a 5-sparse vector recovered with k = 12: after the fifth pick the residual is rounding noise and the
    # float correlation vector no longer decides the same picks as the oracle (the limit App. B's recurrence
    # has by construction); what must still hold: the meaningful picks and values, and a valid support
    rng = np.random.default_rng(5)
    N, d, r, k, sp = 4, 1024, 128, 12, 5
    A, At = make_matrix("stored", 6, d, r)
    X = np.zeros((N, d), np.float32)
    supp = [np.sort(rng.permutation(d)[:sp]) for _ in range(N)]
    for n in range(N):
        X[n, supp[n]] = (1.0 + rng.random(sp)).astype(np.float32) * np.sign(rng.standard_normal(sp)).astype(np.float32)
    Y = (X.astype(np.float64) @ At.astype(np.float64)).astype(np.float32)
    sel, x = run(Y, A, k, True)
    for n in range(N):
        assert sorted(sel[n][:sp].tolist()) == supp[n].tolist()
        assert relerr(x[n][:sp], X[n, sel[n][:sp]]) < 1e-5
        assert len(set(sel[n].tolist())) == k and sel[n].min() >= 0 and sel[n].max() < d
        assert np.abs(x[n][sp:]).max() < 1e-4 and np.isfinite(x[n]).all()


def test_recurrence_validation():
    L = sgc.lib()
    A, _ = make_matrix("stored", 4, 256, 32)
    Y = torch.zeros((2, 32), device=DEV)
    sel = torch.empty((2, 4), dtype=torch.int32, device=DEV)
    x = torch.empty((2, 4), device=DEV)
    need = sgc.sgc_omp_recurrence_workspace_bytes(2, 256, 32, 4)
    assert need >= sgc.sgc_omp_workspace_bytes(2, 256, 32, 4) + 2 * 5 * 256 * 4
    assert sgc.sgc_omp_recurrence_workspace_bytes(2, 254, 32, 4) == 0          # d % 4
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    f = L.sgc_recover_omp_recurrence
    p = lambda t: t.data_ptr()
    assert f(p(Y), 2, ctypes.byref(A.c()), 4, 4, p(sel), p(x), p(ws), need, None) == 0
    assert f(p(Y), 2, ctypes.byref(A.c()), 4, 2, p(sel), p(x), p(ws), need, None) == 0
    assert f(p(Y), 2, ctypes.byref(A.c()), 4, 5, p(sel), p(x), p(ws), need, None) == sgc.ERR_SHAPE
    assert f(p(Y), 2, ctypes.byref(A.c()), 4, 4, p(sel), p(x), p(ws), need - 1, None) == sgc.ERR_WORKSPACE
    assert f(None, 2, ctypes.byref(A.c()), 4, 4, p(sel), p(x), p(ws), need, None) == sgc.ERR_NULL
    A.gram = None
    assert f(p(Y), 2, ctypes.byref(A.c()), 4, 4, p(sel), p(x), p(ws), need, None) == sgc.ERR_NULL   # no table
    torch.cuda.synchronize()
