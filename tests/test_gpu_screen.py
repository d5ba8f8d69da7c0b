"""The bfloat16 screening contraction (an option of the matrix): the recovery must select the same
support as the CPU oracle, bit for bit, and return the same values as with the float contraction."""
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
    A.flags = sgc.MATRIX_FLAG_SCREEN_BF16
    return A, At


def run_omp(Y, A, k):
    N, r = Y.shape
    sel = torch.empty((N, k), dtype=torch.int32, device=DEV)
    x = torch.empty((N, k), dtype=torch.float32, device=DEV)
    ws = torch.empty(sgc.sgc_omp_workspace_bytes_for(N, k, A), dtype=torch.uint8, device=DEV)
    sgc.sgc_recover_omp(dev(Y), N, A, k, sel, x, ws)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), x.cpu().numpy()


@pytest.mark.parametrize("N,d,r,k", [
    (1, 100, 32, 4),         # one ragged tile, one stage
    (5, 1000, 96, 12),       # ragged positions, three stages (odd count)
    (2, 4096, 256, 32),      # cfg1 shape
    (130, 700, 64, 8),       # two tiles of right-hand sides, ragged
    (3, 2000, 100, 10),      # depth not a multiple of 32: the float contraction is used instead
    (128, 32768, 64, 4),     # full tiles, 128 of them: the pipelined form of the screening contraction
    (200, 16384, 128, 4),    # the same with a ragged second tile of right-hand sides
    (65, 32768, 64, 3),      # ... one right-hand side in the second tile; the shortest depth loop (two stages)
    (1040, 16384, 64, 3),    # 256 right-hand sides per workgroup, a ragged fifth tile of them, two stages
    (1024, 16384, 128, 2),   # ... full tiles, four stages
])
def test_screened_recovery_matches_oracle(N, d, r, k):
    say("screen", N, d, r, k)
    rng = np.random.default_rng(N * 3 + d)
    A, At = make_matrix("stored", 24, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    if N > 2:
        Y[1] = 0.0                                   # exact ties: lowest positions, values 0
        Y[2] *= 1e-20                                # tiny scale
    sel, x = run_omp(Y, A, k)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    for n in range(N):
        assert relerr(x[n], rx[n]) < TOL, n
    A.flags = 0
    sel2, x2 = run_omp(Y, A, k)
    assert np.array_equal(sel, sel2)
    assert np.array_equal(x.view(np.uint32), x2.view(np.uint32))   # the least squares never sees the contraction


@pytest.mark.parametrize("d", [3000, 8192], ids=["ragged", "full_tiles"])
def test_screened_recovery_generated_matrix_many_right_hand_sides(d):
    N, r, k = 600, 64, 6
    rng = np.random.default_rng(N + d)
    A, At = make_matrix("philox", 33, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    sel, x = run_omp(Y, A, k)
    norm = orc.colnorms(At)
    for n in [0, 1, 127, 128, 300, N - 1]:
        ref = orc.omp(Y[n], At, k, norm=norm)
        assert np.array_equal(sel[n], ref["sel"]), n
        assert relerr(x[n], ref["x"]) < TOL


def test_screened_exact_recovery_and_sparser_right_hand_sides():
    d, r, k = 1024, 256, 8
    A, At = make_matrix("stored", 20, d, r)
    A64 = At.astype(np.float64).T
    Y = np.zeros((3, r), np.float32)
    x0, pos0 = synth.sparse_signal(0, d, k)
    x1, pos1 = synth.sparse_signal(1, d, 5)
    Y[0] = (A64 @ x0).astype(np.float32)
    Y[1] = (A64 @ x1).astype(np.float32)
    sel, x = run_omp(Y, A, k)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel[0], rsel[0]) and sorted(sel[0].tolist()) == pos0.tolist()
    assert np.array_equal(sel[1][:5], rsel[1][:5]) and len(set(sel[1].tolist())) == k
    assert sel[2].tolist() == list(range(k)) and not x[2].any()


def test_cfg2_full_size_screened_two_steps_sampled():
    w = synth.CFG2
    C, d, r, k = w.C, w.d, w.r, w.k
    At = synth.gaussian_matrix(w.a_seed, d, r)
    A = sgc.Matrix(d, r, At=dev(At))
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    norm = orc.colnorms(At)
    buf = sgc.StepBuffers(C, d, r, k, screen=True)
    buf2 = sgc.StepBuffers(C, d, r, k)
    W = dev(synth.weights(w))
    W2 = W.clone()
    h = sgc.hyper()
    for t in (1, 2):
        g = dev(synth.gradients(w, t))
        A.flags = sgc.MATRIX_FLAG_SCREEN_BF16
        sgc.step(g, W, buf, A, t, h)
        A.flags = 0
        sgc.step(g, W2, buf2, A, t, h)
        torch.cuda.synchronize()
        # the whole run equals the float-contraction run bit for bit
        assert torch.equal(buf.sel, buf2.sel) and torch.equal(buf.x, buf2.x) and torch.equal(W, W2)
    hat, sel = buf.hat.cpu().numpy(), buf.sel.cpu().numpy()
    for n, j in [(0, 0), (64, 17), (31, 255)]:
        rep = orc.omp(hat[n], At, j + 1, norm=norm, forced=sel[n, :j])
        assert rep["sel"][j] == sel[n, j]


def test_all_options_together_screen_gram_shared_support():
    """Screening contraction + Gram table + shared support over consecutive steps, stage-wise
    against the oracle on the GPU's own moments."""
    w = synth.shrink(synth.CFG2, C=3, d=4096, r=256, k=32)
    A, At = make_matrix(w.matrix, w.a_seed, w.d, w.r)
    A.gram = torch.empty((w.d, w.d), dtype=torch.float64, device=DEV)
    sgc.sgc_matrix_gram(A, A.gram)
    buf = sgc.StepBuffers(w.C, w.d, w.r, w.k, screen=True)
    W = dev(synth.weights(w))
    h = sgc.hyper()
    C = w.C
    for t in range(1, 4):
        sgc.step(dev(synth.gradients(w, t)), W, buf, A, t, h, shared_support=True)
        torch.cuda.synchronize()
        mh, vh = buf.hat[:C].cpu().numpy(), buf.hat[C:].cpu().numpy()
        rsel, rx, rz = orc.omp_shared(mh, vh, At, w.k)
        assert np.array_equal(buf.sel[:C].cpu().numpy(), rsel)
        x, z = buf.x[:C].cpu().numpy(), buf.x[C:].cpu().numpy()
        for c in range(C):
            assert relerr(x[c], rx[c]) < TOL and relerr(z[c], rz[c]) < TOL
