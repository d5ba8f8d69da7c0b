"""Seeded random shapes of the other entry points against the oracle: sparsify + project (sizes on both
sides of every kernel choice, ties, zeros, heavy tails, bfloat16 gradients, both matrix modes; top-k
bit-exact), the two outer products of CESGC (ragged and full tiles, batches) and the renewal of its projection
matrix (random sizes, ranks and batches; spectra that converge in the rounds given)."""
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


def relerr(a, ref):
    a = np.asarray(a, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    return 0.0 if a.size == 0 else float(np.abs(a - ref).max() / (den if den > 0 else 1.0))


@pytest.mark.parametrize("seed", range(32))
def test_sparsify_project_random_shape(seed):
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([int(rng.integers(4, 300)), int(rng.integers(300, 9000)), 4096, 16384, 65536,
                        int(rng.integers(65537, 200000))]))
    r = 4 * int(rng.integers(1, 80))
    k = int(rng.integers(1, min(d, r, 600) + 1))
    C = int(rng.integers(1, max(2, min(40, 3_000_000 // d))))
    bf16 = rng.random() < 0.3
    mode = "philox" if rng.random() < 0.5 else "stored"
    kind = int(rng.integers(0, 4))
    say("sparsify_project", seed, dict(C=C, d=d, r=r, k=k, bf16=bf16, mode=mode, kind=kind))
    g = rng.standard_normal((C, d)).astype(np.float32)
    if kind == 1:
        g = np.round(g * 2) / 2                                  # many ties
    elif kind == 2:
        g[:, rng.integers(0, d, size=max(1, d // 3))] = 0        # many zeros
    elif kind == 3:
        g = (rng.standard_t(2.0, size=(C, d)) * 1e-3).astype(np.float32)
    if bf16:
        gref = synth.f32_to_bf16_bits(g)
        gin = dev(gref.view(np.int16))
    else:
        gref = g
        gin = dev(g)
    if mode == "stored":
        At = synth.gaussian_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=dev(At))
    else:
        At = orc.philox_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=None, seed=seed)
    idx = torch.empty((C, k), dtype=torch.int32, device=DEV)
    val = torch.empty((C, k), device=DEV)
    p = torch.empty((C, r), device=DEV)
    q = torch.empty((C, r), device=DEV)
    sgc.sgc_sparsify_project(gin, C * d, d, k, A, idx, val, p, q)
    torch.cuda.synchronize()
    ridx, rval = orc.topk(gref, k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.array_equal(val.cpu().numpy().view(np.uint32), rval.view(np.uint32))
    rp, rq = orc.project(ridx, rval, At)
    pn, qn = p.cpu().numpy(), q.cpu().numpy()
    for c in range(C):
        assert relerr(pn[c], rp[c]) < 1e-5 and relerr(qn[c], rq[c]) < 1e-5, c


@pytest.mark.parametrize("seed", range(20))
def test_outer_products_random_shape(seed):
    rng = np.random.default_rng(9000 + seed)
    count = int(rng.integers(1, 4))
    rho = int(rng.integers(1, 100))
    m = int(rng.integers(1, 700))
    n = 4 * int(rng.integers(1, 200))
    if rng.random() < 0.4:                                       # full tiles: the branch-free paths
        m = 32 * int(rng.integers(1, 20))
        n = 128 * int(rng.integers(1, 6))
        rho = int(rng.choice([16, 32, 64, 96]))
    total = rho * n
    d = int(rng.choice([x for x in range(2, min(total, 4096) + 1) if total % x == 0]))
    k = int(rng.integers(1, min(d, 40) + 1))
    say("outer", seed, dict(count=count, rho=rho, m=m, n=n, d=d, k=k))
    B = rng.standard_normal((count, rho, m)).astype(np.float32)
    G = rng.standard_normal((count, m, n)).astype(np.float32)
    W = rng.standard_normal((count, m, n)).astype(np.float32)
    Cm = total // d
    sel = np.stack([rng.permutation(d)[:k] for _ in range(count * Cm)]).astype(np.int32)
    x = rng.standard_normal((count * Cm, k)).astype(np.float32)
    z = (rng.standard_normal((count * Cm, k)) ** 2).astype(np.float32)
    ob = sgc.OuterBuffers(rho, m, n, count=count)
    h = sgc.hyper(alpha=2.0, lr=0.01, eps=1e-3)
    Bd, Wd = dev(B), dev(W)
    sgc.sgc_outer_project(Bd, dev(G), count, rho, m, n, ob.Gc, ob.ws)
    sgc.sgc_outer_apply(Wd, Bd, count, rho, m, n, d, k, dev(sel), dev(x), dev(sel), dev(z), h, ob.ws)
    torch.cuda.synchronize()
    Gc = ob.Gc.cpu().numpy().reshape(count, rho, n)
    Wn = Wd.cpu().numpy()
    for c in range(count):
        assert relerr(Gc[c], orc.outer_project(B[c], G[c])) < 1e-5, c
        lo, hi = c * Cm, (c + 1) * Cm
        ref = orc.outer_apply(W[c], B[c], d, sel[lo:hi], x[lo:hi], sel[lo:hi], z[lo:hi], alpha=2.0, eps=1e-3, lr=0.01)
        assert relerr(Wn[c] - W[c], ref.astype(np.float64) - W[c]) < 1e-4, c


@pytest.mark.parametrize("seed", range(16))
def test_outer_refresh_random_shape(seed):
    rng = np.random.default_rng(7000 + seed)
    rho = int(rng.integers(1, 65))
    m = 4 * int(rng.integers((rho + 3) // 4, 160))
    n = 4 * int(rng.integers((rho + 3) // 4, 160))
    count = int(rng.integers(1, 4))
    q = min(m, n, rho + 3)
    ratio = 0.5 if rho <= 12 else (0.75 if rho <= 24 else 0.88)   # keeps the spectrum within float's reach
    iters = {0.5: 14, 0.75: 30, 0.88: 70}[ratio]
    say("outer_refresh", seed, dict(count=count, rho=rho, m=m, n=n, ratio=ratio))
    Gs = []
    for _ in range(count):
        U, _r = np.linalg.qr(rng.standard_normal((m, q)))
        V, _r = np.linalg.qr(rng.standard_normal((n, q)))
        Gs.append(((U * (2.0 * ratio ** np.arange(q))) @ V.T).astype(np.float32))
    Gs = np.stack(Gs)
    B = dev(rng.standard_normal((count, rho, m)).astype(np.float32))
    ws = torch.empty(sgc.sgc_outer_refresh_workspace_bytes(count, rho, m, n), dtype=torch.uint8, device=DEV)
    sig = torch.empty((count, rho), device=DEV)
    sgc.sgc_outer_refresh(B, dev(Gs), count, rho, m, n, iters, sig, ws)
    torch.cuda.synchronize()
    Bn, sn = B.cpu().numpy().astype(np.float64), sig.cpu().numpy().astype(np.float64)
    for j in range(count):
        Bref, sref = orc.outer_refresh(Gs[j], rho)
        lead = max(1, int(np.sum(sref / sref[0] > 3e-2)))         # rows far enough above the float rounding of the passes
        assert np.abs(Bn[j] @ Bn[j].T - np.eye(rho)).max() < 1e-5, j
        assert np.abs(sn[j] / sref - 1).max() < 2e-3, j
        assert np.abs(Bn[j][:lead] - Bref[:lead]).max() < 2e-4, j
        assert np.abs(Bn[j].T @ Bn[j] - Bref.T @ Bref).max() < 5e-3, j


@pytest.mark.parametrize("seed", range(12))
def test_recovery_with_very_few_measurements_random_shape(seed):
    """r <= 16 and at least 128 right-hand sides: the contraction on the vector ALUs (supports bit-exact)."""
    rng = np.random.default_rng(11000 + seed)
    N = int(rng.integers(128, 700))
    r = 4 * int(rng.integers(1, 5))
    d = int(rng.integers(r, 6000))
    k = int(rng.integers(1, min(r, d) + 1))
    mode = "stored" if rng.random() < 0.5 else "philox"
    say("narrow", seed, dict(N=N, d=d, r=r, k=k, mode=mode))
    if mode == "stored":
        At = synth.gaussian_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=dev(At))
    else:
        At = orc.philox_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=None, seed=seed)
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    Y[0] = 0.0
    Y[5] = np.round(Y[5])
    sel = torch.empty((N, k), dtype=torch.int32, device=DEV)
    x = torch.empty((N, k), device=DEV)
    ws = torch.empty(sgc.sgc_omp_workspace_bytes(N, d, r, k), dtype=torch.uint8, device=DEV)
    sgc.sgc_recover_omp(dev(Y), N, A, k, sel, x, ws)
    torch.cuda.synchronize()
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel.cpu().numpy(), rsel)
    xn = x.cpu().numpy()
    for n in range(N):
        assert relerr(xn[n], rx[n]) < 1e-4, n
