"""Parity of the outer projection of CESGC (Sec. 4.4: Gc = B G before SGC, W <- W - lr B^T N after it)
against the CPU oracle, through the C ABI. Bar: Gc and the weight change within 1e-4 of the per-matrix
maximum; the steps in between are checked stage-wise on the compressed gradient the GPU produced
(support bit-exact, values within 1e-4), as in the plain step."""
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


SHAPES = [
    (1, 2, 4),            # one row of B, one pair of rows of G, one quad of columns
    (5, 37, 24),          # everything ragged
    (32, 300, 132),       # one full block of B, several slices, a second ragged column strip
    (33, 70, 256),        # the two-block kernel with one row in the second block
    (64, 1000, 512),      # the two-block kernel, ragged rows
    (64, 1024, 512),      # the two-block kernel on full tiles (the branch-free paths)
    (96, 512, 384),       # three rows of blocks of 32: two launches' worth of 64, the last half empty
    (130, 64, 128),       # three blocks of 64 rows of B, the last ragged
    (32, 1024, 1024),     # the paper's rank on a square matrix: 8 strips x 16 slices
]


@pytest.mark.parametrize("rho,m,n", SHAPES)
def test_outer_project_matches_oracle(rho, m, n):
    say("outer_project", rho, m, n)
    rng = np.random.default_rng(rho + m + n)
    B = rng.standard_normal((rho, m)).astype(np.float32)
    G = rng.standard_normal((m, n)).astype(np.float32)
    ob = sgc.OuterBuffers(rho, m, n)
    ob.Gc.fill_(7.0)
    sgc.sgc_outer_project(dev(B), dev(G), 1, rho, m, n, ob.Gc, ob.ws)
    torch.cuda.synchronize()
    ref = orc.outer_project(B, G)
    assert relerr(ob.Gc.cpu().numpy(), ref) < 1e-5
    # reproducible: a second run gives the same bits
    first = ob.Gc.clone()
    sgc.sgc_outer_project(dev(B), dev(G), 1, rho, m, n, ob.Gc, ob.ws)
    torch.cuda.synchronize()
    assert torch.equal(first, ob.Gc)


@pytest.mark.parametrize("count,rho,m,n", [(1, 5, 37, 24), (1, 32, 300, 132), (2, 64, 1000, 512), (3, 32, 256, 256),
                                           (1, 32, 1024, 1024)])
def test_outer_project_of_bf16_gradients(count, rho, m, n):
    """G as bfloat16 bit patterns: the result is the projection of the widened values."""
    say("outer_project bf16", count, rho, m, n)
    rng = np.random.default_rng(rho + m + n + 1)
    B = rng.standard_normal((count, rho, m)).astype(np.float32)
    bits = synth.f32_to_bf16_bits(rng.standard_t(3.0, size=(count, m, n)).astype(np.float32))
    G = synth.bf16_bits_to_f32(bits)
    ob = sgc.OuterBuffers(rho, m, n, count=count)
    sgc.sgc_outer_project(dev(B), dev(bits.view(np.int16)), count, rho, m, n, ob.Gc, ob.ws)
    torch.cuda.synchronize()
    got = ob.Gc.cpu().numpy().reshape(count, rho, n)
    for c in range(count):
        assert relerr(got[c], orc.outer_project(B[c], G[c])) < 1e-5, c
    # and it equals, bit for bit, the projection of the same values handed over as floats
    ob2 = sgc.OuterBuffers(rho, m, n, count=count)
    sgc.sgc_outer_project(dev(B), dev(G), count, rho, m, n, ob2.Gc, ob2.ws)
    torch.cuda.synchronize()
    assert torch.equal(ob.Gc, ob2.Gc)


@pytest.mark.parametrize("rho,m,n,d,k", [
    (1, 2, 4, 4, 1), (5, 37, 24, 8, 2), (32, 300, 132, 64, 5), (64, 1000, 512, 2048, 31), (130, 64, 128, 1664, 40),
    (32, 1024, 1024, 2048, 31), (64, 1024, 512, 2048, 31), (96, 512, 384, 1024, 20), (16, 256, 128, 512, 7),
])
def test_outer_apply_matches_oracle(rho, m, n, d, k):
    say("outer_apply", rho, m, n, d, k)
    rng = np.random.default_rng(rho * 3 + m + n)
    C = rho * n // d
    B = rng.standard_normal((rho, m)).astype(np.float32)
    W = rng.standard_normal((m, n)).astype(np.float32)
    sel_m = np.stack([rng.permutation(d)[:k] for _ in range(C)]).astype(np.int32)
    sel_v = np.stack([rng.permutation(row) for row in sel_m]).astype(np.int32)
    if k > 1:
        sel_v[:, 0] = (sel_m[:, 0] + 1) % d                      # may miss the first moment's support
    x = rng.standard_normal((C, k)).astype(np.float32)
    z = rng.standard_normal((C, k)).astype(np.float32) ** 2 - 0.05   # some negative second moments
    h = sgc.hyper(alpha=2.0, lr=0.01, eps=1e-3)
    ob = sgc.OuterBuffers(rho, m, n)
    Wd = dev(W)
    sgc.sgc_outer_apply(Wd, dev(B), 1, rho, m, n, d, k, dev(sel_m), dev(x), dev(sel_v), dev(z), h, ob.ws)
    torch.cuda.synchronize()
    ref = orc.outer_apply(W, B, d, sel_m, x, sel_v, z, alpha=2.0, eps=1e-3, lr=0.01)
    assert relerr(Wd.cpu().numpy() - W, ref.astype(np.float64) - W) < TOL


@pytest.mark.parametrize("count,rho,m,n,d,k", [(3, 5, 37, 24, 8, 2), (4, 32, 256, 256, 2048, 31), (2, 70, 96, 128, 64, 4)])
def test_a_batch_equals_its_matrices_one_by_one(count, rho, m, n, d, k):
    """Bitwise: the batch index only moves the base pointers."""
    say("outer batch", count, rho, m, n)
    rng = np.random.default_rng(count + rho)
    B = dev(rng.standard_normal((count, rho, m)).astype(np.float32))
    G = dev(rng.standard_normal((count, m, n)).astype(np.float32))
    W = rng.standard_normal((count, m, n)).astype(np.float32)
    Cm = rho * n // d
    sel = dev(np.stack([rng.permutation(d)[:k] for _ in range(count * Cm)]).astype(np.int32))
    x = dev(rng.standard_normal((count * Cm, k)).astype(np.float32))
    z = dev((rng.standard_normal((count * Cm, k)) ** 2).astype(np.float32))
    h = sgc.hyper(alpha=2.0, lr=0.01)
    ob = sgc.OuterBuffers(rho, m, n, count=count)
    one = sgc.OuterBuffers(rho, m, n)
    sgc.sgc_outer_project(B, G, count, rho, m, n, ob.Gc, ob.ws)
    Wb = dev(W)
    sgc.sgc_outer_apply(Wb, B, count, rho, m, n, d, k, sel, x, sel, z, h, ob.ws)
    torch.cuda.synchronize()
    for c in range(count):
        sgc.sgc_outer_project(B[c], G[c], 1, rho, m, n, one.Gc, one.ws)
        W1 = dev(W[c])
        lo, hi = c * Cm, (c + 1) * Cm
        sgc.sgc_outer_apply(W1, B[c], 1, rho, m, n, d, k, sel[lo:hi], x[lo:hi], sel[lo:hi], z[lo:hi], h, one.ws)
        torch.cuda.synchronize()
        assert torch.equal(ob.Gc[c], one.Gc), c
        assert torch.equal(Wb[c], W1), c
    ref = orc.outer_project(B[1].cpu().numpy(), G[1].cpu().numpy())
    assert relerr(ob.Gc[1].cpu().numpy(), ref) < 1e-5


def test_outer_apply_of_an_empty_update_leaves_the_weights():
    rho, m, n, d, k = 4, 40, 64, 32, 3
    rng = np.random.default_rng(0)
    W = rng.standard_normal((m, n)).astype(np.float32)
    B = rng.standard_normal((rho, m)).astype(np.float32)
    C = rho * n // d
    sel = np.tile(np.arange(k, dtype=np.int32), (C, 1))
    zero = np.zeros((C, k), np.float32)
    ob = sgc.OuterBuffers(rho, m, n)
    Wd = dev(W)
    sgc.sgc_outer_apply(Wd, dev(B), 1, rho, m, n, d, k, dev(sel), dev(zero), dev(sel), dev(zero), sgc.hyper(), ob.ws)
    torch.cuda.synchronize()
    assert np.array_equal(Wd.cpu().numpy(), W)


def cesgc_case(m, n, rho, d, r, k, seed):
    basis = synth.orthonormal_rows(seed, max(rho, 8) * 2, m)
    B = np.ascontiguousarray(basis[:rho])
    At = synth.gaussian_matrix(seed + 1, d, r)
    A = sgc.Matrix(d, r, At=dev(At))
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    return basis, B, At, A


@pytest.mark.parametrize("m,n,rho,d,r,k,steps", [
    (96, 128, 4, 64, 32, 4, 3),
    (512, 1024, 32, 2048, 220, 31, 2),       # the paper's CESGC setting (rank 32, chunks of 2048, 31 kept, r = 7 k)
    (4096, 4096, 32, 2048, 220, 31, 1),      # the same on a full attention matrix (the benchmark's shape, one matrix)
], ids=["tiny", "paper_setting", "paper_setting_4096x4096"])
def test_cesgc_steps_stage_wise(m, n, rho, d, r, k, steps):
    basis, B, At, A = cesgc_case(m, n, rho, d, r, k, 3)
    C = rho * n // d
    h = sgc.hyper(alpha=2.0, lr=1e-2)   # a step well above the rounding of W, so the change itself is compared
    ob = sgc.OuterBuffers(rho, m, n)
    buf = sgc.StepBuffers(C, d, r, k)
    rng = np.random.default_rng(1)
    W = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
    Wd, Bd = dev(W), dev(B)
    m_prev = np.zeros((C, r), np.float32)
    v_prev = np.zeros((C, r), np.float32)
    for t in range(1, steps + 1):
        say("  cesgc step", t)
        G = synth.matrix_gradient(3, t, m, n, basis)
        W_prev = Wd.cpu().numpy()
        sgc.step_cesgc(dev(G), Wd, Bd, ob, buf, A, t, h)
        torch.cuda.synchronize()
        Gc = ob.Gc.cpu().numpy()
        assert relerr(Gc, orc.outer_project(B, G)) < 1e-5
        # Alg. 2 on the GPU's compressed gradient
        idx, val = orc.topk(Gc.reshape(C, d), k)
        assert np.array_equal(buf.idx.cpu().numpy(), idx) and np.array_equal(buf.val.cpu().numpy(), val)
        p, q = orc.project(idx, val, At)
        gp, gq = buf.p.cpu().numpy(), buf.q.cpu().numpy()
        for c in range(C):
            assert relerr(gp[c], p[c]) < 1e-5 and relerr(gq[c], q[c]) < 1e-5
        rm, rv, rmh, rvh = orc.adam(gp, gq, m_prev, v_prev, t)
        m_prev, v_prev = buf.m.cpu().numpy(), buf.v.cpu().numpy()
        assert relerr(m_prev, rm) < 1e-6 and relerr(v_prev, rv) < 1e-6
        hat = buf.hat.cpu().numpy()
        rsel, rx = orc.omp_batch(hat, At, k)
        sel, x = buf.sel.cpu().numpy(), buf.x.cpu().numpy()
        assert np.array_equal(sel, rsel)
        for nn in range(2 * C):
            assert relerr(x[nn], rx[nn]) < TOL
        ref = orc.outer_apply(W_prev, B, d, sel[:C], x[:C], sel[C:], x[C:], alpha=2.0, lr=1e-2)
        assert relerr(Wd.cpu().numpy() - W_prev, ref.astype(np.float64) - W_prev) < TOL


def test_cesgc_with_identity_projection_equals_the_plain_step():
    """B = I: both paths must move the weights identically up to the rounding of the products."""
    m, n, d, r, k = 32, 256, 512, 128, 6
    C = m * n // d
    At = synth.gaussian_matrix(9, d, r)
    A = sgc.Matrix(d, r, At=dev(At))
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    rng = np.random.default_rng(4)
    G = rng.standard_t(3.0, size=(m, n)).astype(np.float32)
    W = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
    h = sgc.hyper(alpha=2.0)
    ob = sgc.OuterBuffers(m, m, n)
    buf1, buf2 = sgc.StepBuffers(C, d, r, k), sgc.StepBuffers(C, d, r, k)
    W1, W2 = dev(W), dev(W).reshape(-1).clone()
    sgc.step_cesgc(dev(G), W1, dev(np.eye(m, dtype=np.float32)), ob, buf1, A, 1, h)
    sgc.step(dev(G).reshape(-1), W2, buf2, A, 1, h)
    torch.cuda.synchronize()
    assert torch.equal(ob.Gc.reshape(-1), dev(G).reshape(-1))          # products with 0 and 1 are exact
    assert torch.equal(buf1.sel, buf2.sel) and torch.equal(buf1.x, buf2.x)
    assert relerr(W1.cpu().numpy().ravel() - W.ravel(), W2.cpu().numpy() - W.ravel()) < TOL


def test_llama_attention_matrix_full_size_sampled():
    """The bench shape (4096 x 4096 weights, rank 32): Gc on sampled entries, the weight change on
    sampled rows, each from the oracle's definition entry by entry."""
    m = n = 4096
    rho, d, k = 32, 2048, 31
    rng = np.random.default_rng(11)
    B = synth.orthonormal_rows(5, rho, m)
    G = rng.standard_t(3.0, size=(m, n)).astype(np.float32) * np.float32(1e-3)
    ob = sgc.OuterBuffers(rho, m, n)
    Bd = dev(B)
    sgc.sgc_outer_project(Bd, dev(G), 1, rho, m, n, ob.Gc, ob.ws)
    torch.cuda.synchronize()
    Gc = ob.Gc.cpu().numpy()
    cols = np.array([0, 1, 127, 128, 2049, 4095])
    ref = B.astype(np.float64) @ G[:, cols].astype(np.float64)
    assert np.abs(Gc[:, cols] - ref).max() < 1e-5 * np.abs(ref).max()
    C = rho * n // d
    sel_m = np.stack([rng.permutation(d)[:k] for _ in range(C)]).astype(np.int32)
    x = rng.standard_normal((C, k)).astype(np.float32)
    z = (rng.standard_normal((C, k)) ** 2).astype(np.float32)
    W = rng.standard_normal((m, n)).astype(np.float32)
    Wd = dev(W)
    h = sgc.hyper(alpha=2.0, lr=0.01, eps=1e-3)
    sgc.sgc_outer_apply(Wd, Bd, 1, rho, m, n, d, k, dev(sel_m), dev(x), dev(sel_m), dev(z), h, ob.ws)
    torch.cuda.synchronize()
    N = np.zeros((C, d))
    for c in range(C):
        N[c, sel_m[c]] = 2.0 * x[c].astype(np.float64) / (np.sqrt(z[c].astype(np.float64)) + 1e-3)
    N = N.reshape(rho, n)
    rows = np.array([0, 31, 32, 1000, 4095])
    ref = -0.01 * B[:, rows].astype(np.float64).T @ N
    got = Wd.cpu().numpy()[rows].astype(np.float64) - W[rows]
    assert np.abs(got - ref).max() < TOL * np.abs(ref).max()
