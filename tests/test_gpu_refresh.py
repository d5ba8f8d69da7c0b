"""The renewal of CESGC's projection matrix (Sec. 4.4) against the CPU oracle (a singular value
decomposition in double). What is unique is compared: singular values, the projector B^T B of the
subspace, and - where the singular values are well separated - the rows themselves, whose sign both
sides fix the same way. Tolerances: the passes over G accumulate in float (2^-24 per product, summed
over up to 4096 terms with random signs: ~1e-6 relative), and a singular vector moves by that error
divided by the relative gap to its neighbours (>= 0.2 in the cases that compare rows): 1e-4 covers it."""
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


def spectrum_matrix(rng, m, n, sigma):
    q = len(sigma)
    U, _ = np.linalg.qr(rng.standard_normal((m, q)))
    V, _ = np.linalg.qr(rng.standard_normal((n, q)))
    return ((U * sigma) @ V.T).astype(np.float32)


def refresh(G, rho, iters, start=None, seed=0):
    m, n = G.shape[-2:]
    if start is None:
        start = np.random.default_rng(1000 + seed).standard_normal((rho, m)).astype(np.float32)
    B = dev(start.astype(np.float32))
    Gd = G if isinstance(G, torch.Tensor) else dev(G)
    gt = sgc.GRAD_BF16 if Gd.dtype in (torch.int16, torch.bfloat16) else sgc.GRAD_F32
    ws = torch.empty(sgc.sgc_outer_refresh_workspace_bytes(1, rho, m, n, gt), dtype=torch.uint8, device=DEV)
    sigma = torch.empty(rho, dtype=torch.float32, device=DEV)
    sgc.sgc_outer_refresh(B, Gd, 1, rho, m, n, iters, sigma, ws)
    torch.cuda.synchronize()
    return B.cpu().numpy().astype(np.float64), sigma.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("m,n,rho,ratio,iters,lead,ptol", [
    (256, 384, 8, 0.5, 12, 8, 1e-4),       # several tiles either way
    (100, 52, 5, 0.5, 12, 5, 1e-4),        # ragged tiles, odd rho (the Jacobi pairing pads it)
    (64, 64, 1, 0.5, 12, 1, 1e-4),         # a single vector: power iteration
    (512, 1024, 64, 0.9, 70, 24, 2e-3),    # the largest rho; singular values over three decades
    (36, 2048, 32, 0.85, 45, 16, 1e-3),    # m barely above rho
    (2048, 40, 32, 0.85, 45, 16, 1e-3),    # n barely above rho
])
def test_refresh_matches_the_decomposition(m, n, rho, ratio, iters, lead, ptol):
    """`lead` rows are compared one by one; the float passes over G leave an error of ~1e-7 sigma_1 in
    every direction, which the last rows of a spectrum spanning decades feel in proportion to
    sigma_1 / sigma_i - they are covered by the projector of the whole subspace at `ptol`."""
    say("refresh", m, n, rho, ratio, iters)
    rng = np.random.default_rng(m + n + rho)
    q = min(m, n, rho + 4)
    sigma = 3.0 * ratio ** np.arange(q)
    G = spectrum_matrix(rng, m, n, sigma)
    B, s = refresh(G, rho, iters, seed=rho)
    Bref, sref = orc.outer_refresh(G, rho)
    assert np.abs(B @ B.T - np.eye(rho)).max() < 1e-5
    assert np.abs(s - sref).max() < 1e-4 * sref[0]
    assert np.abs(s / sref - 1).max() < 1e-3                      # the small ones too
    assert np.abs(B.T @ B - Bref.T @ Bref).max() < ptol
    assert np.abs(B[:lead] - Bref[:lead]).max() < 1e-4            # rows, signs included


def test_refresh_bfloat16_gradient():
    rng = np.random.default_rng(7)
    m, n, rho = 192, 320, 8
    # rounding to bfloat16 adds a flat tail of singular values near 5e-4; the 8 wanted ones stay far above it
    G = spectrum_matrix(rng, m, n, 2.0 * 0.6 ** np.arange(12))
    bits = synth.f32_to_bf16_bits(G)
    Gw = (bits.astype(np.uint32) << 16).view(np.float32)          # what the bit patterns mean
    B, s = refresh(dev(bits.view(np.int16)), rho, 20)
    Bref, sref = orc.outer_refresh(Gw, rho)
    assert np.abs(s / sref - 1).max() < 1e-3
    assert np.abs(B.T @ B - Bref.T @ Bref).max() < 1e-4
    assert np.abs(B - Bref).max() < 1e-4


def test_refresh_batch_of_matrices():
    # three different matrices in one call: every kernel covers the batch, results per matrix as alone
    rng = np.random.default_rng(12)
    count, m, n, rho = 3, 160, 288, 7
    Gs = np.stack([spectrum_matrix(rng, m, n, (2.0 + j) * 0.55 ** np.arange(10)) for j in range(count)])
    start = rng.standard_normal((count, rho, m)).astype(np.float32)
    B = dev(start)
    ws = torch.empty(sgc.sgc_outer_refresh_workspace_bytes(count, rho, m, n), dtype=torch.uint8, device=DEV)
    sigma = torch.empty((count, rho), dtype=torch.float32, device=DEV)
    sgc.sgc_outer_refresh(B, dev(Gs), count, rho, m, n, 14, sigma, ws)
    torch.cuda.synchronize()
    Bn, sn = B.cpu().numpy().astype(np.float64), sigma.cpu().numpy().astype(np.float64)
    for j in range(count):
        Bref, sref = orc.outer_refresh(Gs[j], rho)
        assert np.abs(sn[j] / sref - 1).max() < 1e-3, j
        assert np.abs(Bn[j] - Bref).max() < 1e-4, j
        alone, s_alone = refresh(Gs[j], rho, 14, start=start[j])
        assert np.array_equal(alone, Bn[j]) and np.array_equal(s_alone, sn[j]), j   # fixed summation orders


def test_refresh_equal_singular_values_give_the_same_subspace():
    rng = np.random.default_rng(8)
    m, n, rho = 128, 256, 6
    G = spectrum_matrix(rng, m, n, np.array([4.0, 4.0, 4.0, 2.0, 2.0, 1.0, 0.01, 0.005]))
    B, s = refresh(G, rho, 10)
    Bref, sref = orc.outer_refresh(G, rho)
    assert np.abs(s - sref).max() < 1e-4 * sref[0]
    assert np.abs(B @ B.T - np.eye(rho)).max() < 1e-5
    assert np.abs(B.T @ B - Bref.T @ Bref).max() < 1e-4           # the vectors inside a cluster are free
    assert np.abs(B[5] - Bref[5]).max() < 1e-4                    # the simple one is not


def test_refresh_rank_below_rho_gives_zero_rows():
    rng = np.random.default_rng(9)
    m, n, rho = 64, 96, 5
    G = spectrum_matrix(rng, m, n, np.array([3.0, 2.0, 1.0]))
    B, s = refresh(G, rho, 8)
    Bref, sref = orc.outer_refresh(G, 3)
    assert np.abs(s[:3] - sref).max() < 1e-4 * sref[0]
    assert np.abs(B[:3] - Bref).max() < 1e-4
    assert np.abs(s[3:]).max() < 1e-5 and np.isfinite(B).all()
    # what is left spans nothing of G: rows that are zero, or orthogonal to G's range
    assert np.abs(B[3:] @ G.astype(np.float64)).max() < 1e-5
    Gz = np.zeros((m, n), np.float32)
    Bz, sz = refresh(Gz, rho, 3)
    assert np.array_equal(Bz, np.zeros((rho, m))) and np.array_equal(sz, np.zeros(rho))


def test_refresh_fills_zero_rows_of_the_start_matrix_again():
    # the sequence a periodic caller sees: a gradient of rank 3 leaves two zero rows in B; the next renewal,
    # started from that B on a gradient of full rank, must return all five singular vectors
    rng = np.random.default_rng(13)
    m, n, rho = 96, 160, 5
    G_low = spectrum_matrix(rng, m, n, np.array([3.0, 2.0, 1.0]))
    B_low, s_low = refresh(G_low, rho, 8)
    assert np.array_equal(B_low[3:], np.zeros((2, m)))
    G_full = spectrum_matrix(rng, m, n, 2.0 * 0.5 ** np.arange(8))
    B, s = refresh(G_full, rho, 14, start=B_low)
    Bref, sref = orc.outer_refresh(G_full, rho)
    assert np.abs(s / sref - 1).max() < 1e-3
    assert np.abs(B - Bref).max() < 1e-4


def test_refresh_without_rounds_leaves_zero_rows_alone():
    rng = np.random.default_rng(14)
    m, n, rho = 64, 96, 4
    G = rng.standard_normal((m, n)).astype(np.float32)
    Q, _ = np.linalg.qr(rng.standard_normal((m, rho)))
    start = Q.T.copy()
    start[2] = 0.0
    B, s = refresh(G, rho, 0, start=start)
    live = np.delete(start, 2, axis=0)
    assert np.abs(B.T @ B - live.T @ live).max() < 1e-5          # the three directions given, rotated; nothing invented
    assert np.abs(B[3]).max() == 0.0 and s[3] == 0.0


def test_refresh_from_the_previous_matrix_needs_few_rounds():
    # the periodic use: the gradient's subspace has drifted a little since the last decomposition
    rng = np.random.default_rng(10)
    m, n, rho = 256, 512, 16
    sigma = 2.0 * 0.75 ** np.arange(16)
    U, _ = np.linalg.qr(rng.standard_normal((m, 16)))
    V, _ = np.linalg.qr(rng.standard_normal((n, 16)))
    U2, _ = np.linalg.qr(U + 0.02 * rng.standard_normal((m, 16)))
    G_old = ((U * sigma) @ V.T).astype(np.float32)
    G_new = ((U2 * sigma) @ V.T).astype(np.float32)
    B_old, _ = orc.outer_refresh(G_old, rho)
    Bref, sref = orc.outer_refresh(G_new, rho)
    B, s = refresh(G_new, rho, 2, start=B_old)
    assert np.abs(B.T @ B - Bref.T @ Bref).max() < 1e-4           # rank 16 exactly: one round finds the subspace
    assert np.abs(s / sref - 1).max() < 1e-3


def test_refresh_without_rounds_rotates_inside_the_subspace():
    rng = np.random.default_rng(11)
    m, n, rho = 128, 200, 8
    G = rng.standard_normal((m, n)).astype(np.float32)
    Q, _ = np.linalg.qr(rng.standard_normal((m, rho)))
    B, s = refresh(G, rho, 0, start=Q.T)
    assert np.abs(B.T @ B - Q @ Q.T).max() < 1e-5                 # same subspace
    sref = np.linalg.svd(Q.T @ G.astype(np.float64), compute_uv=False)
    assert np.abs(s - sref).max() < 1e-4 * sref[0]                # ordered by what each direction captures
    assert (np.diff(s) <= 0).all()


def test_refresh_full_size_properties():
    # 4096 x 4096, rank 32 (the benchmark's matrices): a decomposition on the CPU would take minutes, so
    # properties are checked in double. The recipe's gradient has a few directions above a flat noise
    # floor (as real gradients do): the leading rows must satisfy the eigen-equation of G G^T; inside
    # the floor no direction is distinguished, and what holds is that the rows are orthonormal, that
    # B G has orthogonal rows of norms sigma (the Rayleigh-Ritz step), and that B captures at least what
    # the recipe's own directions capture.
    m = n = 4096
    rho = 32
    basis = synth.orthonormal_rows(5, 2 * rho, m)
    G = synth.matrix_gradient(5, 0, m, n, basis)
    B, s = refresh(G, rho, 25, seed=3)
    assert np.abs(B @ B.T - np.eye(rho)).max() < 1e-5
    assert (np.diff(s) <= 0).all()
    G64 = G.astype(np.float64)
    Z = B @ G64
    assert np.abs(Z @ Z.T - np.diag(s ** 2)).max() < 1e-4 * s[0] ** 2
    lead = 5
    R = Z[:lead] @ G64.T - (s[:lead] ** 2)[:, None] * B[:lead]
    assert np.abs(R).max() < 2e-4 * s[0] ** 2
    inside = np.linalg.norm(B[:lead] @ basis[:16].astype(np.float64).T, axis=1)
    assert inside.min() > 0.98                                     # they lie in the planted directions
    assert np.linalg.norm(Z) >= np.linalg.norm(basis[:rho].astype(np.float64) @ G64)


def test_refresh_validation():
    L = sgc.lib()
    B = torch.zeros((4, 64), device=DEV)
    G = torch.zeros((64, 64), device=DEV)
    ws = torch.empty(sgc.sgc_outer_refresh_workspace_bytes(1, 4, 64, 64), dtype=torch.uint8, device=DEV)
    p = lambda t: t.data_ptr()
    ok = lambda **kw: L.sgc_outer_refresh(*[kw.get(k, d) for k, d in [
        ("B", p(B)), ("G", p(G)), ("gt", 0), ("count", 1), ("rho", 4), ("m", 64), ("n", 64), ("iters", 1), ("sigma", None),
        ("ws", p(ws)), ("wsb", ws.numel()), ("stream", None)]])
    assert ok() == 0
    assert ok(B=None) == sgc.ERR_NULL and ok(G=None) == sgc.ERR_NULL and ok(ws=None) == sgc.ERR_NULL
    assert ok(gt=5) == sgc.ERR_DTYPE
    assert ok(count=2) == sgc.ERR_WORKSPACE                        # sized for one matrix
    for bad in (dict(count=0), dict(rho=0), dict(rho=65), dict(m=62), dict(n=30), dict(iters=-1), dict(iters=1001), dict(rho=4, m=2)):
        assert ok(**bad) == sgc.ERR_SHAPE, bad
    assert ok(B=p(B) + 4) == sgc.ERR_ALIGN and ok(ws=p(ws) + 16) == sgc.ERR_ALIGN
    assert ok(wsb=ws.numel() - 1) == sgc.ERR_WORKSPACE
    assert sgc.sgc_outer_refresh_workspace_bytes(1, 65, 64, 64) == 0
    torch.cuda.synchronize()
