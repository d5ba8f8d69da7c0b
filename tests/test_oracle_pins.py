"""Pins of the CPU oracle against things that are not the oracle: brute force, library
routines, published test vectors, closed forms and invariants. CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2502_00311_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- top-k
def brute_topk(g, k):
    """Sparsify_k by a full stable sort on (-|g|, position) (Sec. 4.2)."""
    mag = np.abs(g.astype(np.float64))
    order = np.lexsort((np.arange(g.size), -mag))[:k]
    pos = np.sort(order)
    return pos.astype(np.int32), g[pos]


@pytest.mark.parametrize("d,k", [(1, 1), (7, 3), (64, 64), (1000, 17), (4096, 32), (5003, 256)])
def test_topk_matches_full_sort(d, k):
    rng = np.random.default_rng(d * 31 + k)
    g = rng.standard_t(3, size=(5, d)).astype(np.float32)
    idx, val = orc.topk(g, k)
    for c in range(g.shape[0]):
        pos, v = brute_topk(g[c], k)
        assert np.array_equal(idx[c], pos)
        assert np.array_equal(val[c], v)


def test_topk_ties_lower_position_wins_and_sign_is_kept():
    g = np.array([[1.0, -2.0, 2.0, -2.0, 0.5, 2.0, -0.0, 0.0]], np.float32)
    idx, val = orc.topk(g, 3)
    assert idx.tolist() == [[1, 2, 3]]
    assert val.tolist() == [[-2.0, 2.0, -2.0]]
    idx, val = orc.topk(np.zeros((1, 6), np.float32), 2)
    assert idx.tolist() == [[0, 1]]
    # quantised values: many ties at the threshold
    rng = np.random.default_rng(5)
    g = rng.integers(-4, 5, size=(3, 300)).astype(np.float32)
    idx, val = orc.topk(g, 40)
    for c in range(3):
        pos, v = brute_topk(g[c], 40)
        assert np.array_equal(idx[c], pos) and np.array_equal(val[c], v)


@pytest.mark.parametrize("d,k", [(64, 8), (5000, 64), (16384, 64), (70000, 100)])
def test_topk_orders_values_one_ulp_apart_around_the_kth_place(d, k):
    """Many entries one unit in the last place apart on both sides of the k-th largest magnitude (and
    exact ties at it): the order must be that of the full bit pattern, down to the lowest mantissa bit."""
    g = synth.ulp_cluster_gradients(1, 3, d, k)
    idx, val = orc.topk(g, k)
    for c in range(3):
        pos, v = brute_topk(g[c], k)
        assert np.array_equal(idx[c], pos)
        assert np.array_equal(val[c].view(np.uint32), v.view(np.uint32))
        # the threshold really sits among neighbours one ulp apart: kept and dropped magnitudes touch
        kept = np.abs(g[c, pos]).min().view(np.uint32)
        dropped = np.abs(np.delete(g[c], pos)).max().view(np.uint32)
        assert kept >= dropped and int(kept) - int(dropped) <= 1


def test_topk_bf16_matches_full_sort_on_widened_values():
    rng = np.random.default_rng(11)
    g32 = rng.standard_t(2.5, size=(4, 3000)).astype(np.float32)
    bits = synth.f32_to_bf16_bits(g32)
    wide = synth.bf16_bits_to_f32(bits)
    idx, val = orc.topk(bits, 100)
    for c in range(4):
        pos, v = brute_topk(wide[c], 100)
        assert np.array_equal(idx[c], pos)
        assert np.array_equal(val[c], v)


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is halfway between bf16 1.0 and 1+2^-7: ties to even -> 1.0; 1+3*2^-8 -> 1+2^-6
    x = np.array([1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8, 1.0 + 2.0**-8 + 2.0**-20], np.float32)
    back = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    assert back.tolist() == [1.0, 1.0 + 2.0**-6, 1.0 + 2.0**-7]


def test_chunked_vs_global_sparsification_bound():
    """Thm. 1: E||chunked - global||^2 <= 2 (1 - s/d) G_max, G_max = ||G||^2 here."""
    rng = np.random.default_rng(3)
    c, dc, sc = 8, 512, 16
    for _ in range(5):
        G = rng.standard_t(3, size=c * dc).astype(np.float32)
        idx, val = orc.topk(G.reshape(c, dc), sc)
        chunked = np.zeros(c * dc)
        for i in range(c):
            chunked[i * dc + idx[i]] = val[i]
        gi, gv = orc.topk(G.reshape(1, -1), c * sc)
        glob = np.zeros(c * dc)
        glob[gi[0]] = gv[0]
        lhs = np.sum((chunked - glob) ** 2)
        assert lhs <= 2 * (1 - c * sc / (c * dc)) * np.sum(G.astype(np.float64) ** 2)


# ---------------------------------------------------------------------- projection
def test_projection_equals_dense_matvec():
    rng = np.random.default_rng(0)
    d, r, k, C = 700, 96, 23, 4
    At = synth.gaussian_matrix(9, d, r)
    g = rng.standard_normal((C, d)).astype(np.float32)
    idx, val = orc.topk(g, k)
    p, q = orc.project(idx, val, At)
    A = At.astype(np.float64).T  # r x d
    for c in range(C):
        gs = np.zeros(d)
        gs[idx[c]] = val[c]
        gs2 = np.zeros(d)
        gs2[idx[c]] = (val[c] * val[c]).astype(np.float64)  # float square, as a float G^2 holds
        assert np.allclose(p[c], A @ gs, rtol=0, atol=1e-6 * np.abs(A @ gs).max())
        assert np.allclose(q[c], A @ gs2, rtol=0, atol=1e-6 * np.abs(A @ gs2).max())
    # a transposed operand or an index slip would not survive a one-hot gradient
    one = np.zeros((1, d), np.float32)
    one[0, 123] = -3.0
    idx, val = orc.topk(one, 1)
    p, q = orc.project(idx, val, At)
    assert np.array_equal(p[0], (-3.0 * At[123].astype(np.float64)).astype(np.float32))
    assert np.array_equal(q[0], (9.0 * At[123].astype(np.float64)).astype(np.float32))


# -------------------------------------------------------------------------- Philox
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLD, "philox4x32_10_kat.txt")) if not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        w = [int(x, 16) for x in row]
        out = orc.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]


def test_normal_transform_against_exact_box_muller():
    rng = np.random.default_rng(1)
    w = rng.integers(0, 2**32, size=(20000, 2), dtype=np.uint64)
    # corners of the input space
    w[:8, 0] = [0, 1, 2**32 - 1, 2**31, 511, 512, 2**32 - 512, 2**9 * 3]
    w[:8, 1] = [0, 2**32 - 1, 2**29, 2**29 - 1, 2**31, 3 * 2**29 + 5, 2**30, 7 * 2**29]
    worst = 0.0
    for a, b in w:
        z = orc.normal_pair(a, b, 1.0).astype(np.float64)
        u = (((int(a) >> 9) << 1) | 1) * 2.0**-24
        oct_ = int(b) >> 29
        frac = ((int(b) >> 6) & 0x7FFFFF) + 0.5
        theta = (oct_ + frac * 2.0**-23) * (np.pi / 4)
        rad = np.sqrt(-2.0 * np.log(u))
        ex = np.array([rad * np.cos(theta), rad * np.sin(theta)])
        worst = max(worst, np.abs(z - ex).max() / max(1.0, rad))
    assert worst < 6e-7


def test_philox_matrix_layout_and_statistics():
    d, r = 512, 256
    At = orc.philox_matrix(0x1234567890ABCDEF, d, r)
    # layout: counter (i, j/4), words (0,1) -> rows 4b,4b+1 and (2,3) -> rows 4b+2,4b+3
    key = [0x90ABCDEF, 0x12345678]
    scale = np.float32(1.0 / np.sqrt(r))
    for i, jb in [(0, 0), (5, 3), (511, 63)]:
        wds = orc.philox4x32_10([i, jb, 0, 0], key)
        z01 = orc.normal_pair(wds[0], wds[1], scale)
        z23 = orc.normal_pair(wds[2], wds[3], scale)
        assert np.array_equal(At[i, 4 * jb:4 * jb + 4], np.concatenate([z01, z23]))
    # sub-blocks equal the corresponding rows of the full matrix
    assert np.array_equal(orc.philox_matrix(0x1234567890ABCDEF, d, r, 100, 7), At[100:107])
    # a different seed gives a different matrix
    assert not np.array_equal(orc.philox_matrix(2, d, r, 0, 4), At[:4])
    z = At.astype(np.float64).ravel() * np.sqrt(r)
    n = z.size
    assert abs(z.mean()) < 4 / np.sqrt(n)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs((z**4).mean() - 3) < 4 * np.sqrt(96 / n)
    from scipy import stats
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # rows and columns are uncorrelated: Gram of 64 columns is close to identity
    G = At[:64].astype(np.float64) @ At[:64].astype(np.float64).T
    assert np.abs(G - np.eye(64)).max() < 6 / np.sqrt(r)


# ---------------------------------------------------------------------------- Adam
def test_adam_hand_derived_steps():
    rows = [list(map(float, l.split())) for l in open(os.path.join(GOLD, "adam_step1_closed_form.txt")) if not l.startswith("#")]
    for p, q, m1, v1, mh1, vh1, m2s, v2s, m2c, v2c, mh2c, vh2c in rows:
        P = np.array([p], np.float32)
        Q = np.array([q], np.float32)
        z = np.zeros(1, np.float32)
        m, v, mh, vh = orc.adam(P, Q, z, z, 1)
        assert np.allclose([m[0], v[0], mh[0], vh[0]], [m1, v1, mh1, vh1], rtol=2e-6, atol=0)
        mm, vv, mh2, vh2 = orc.adam(P, Q, m, v, 2)
        assert np.allclose([mm[0], vv[0], mh2[0], vh2[0]], [m2s, v2s, p, q], rtol=2e-6, atol=0)
        mm, vv, mh2, vh2 = orc.adam(3 * P, 5 * Q, m, v, 2)
        assert np.allclose([mm[0], vv[0], mh2[0], vh2[0]], [m2c, v2c, mh2c, vh2c], rtol=2e-6, atol=0)


def test_adam_moments_are_the_projection_of_dense_adam_moments():
    """Eq. 10: M_t = A sum_i h_i(beta1) G~_i, i.e. the compressed moment equals A times the
    dense AdamW first moment (Alg. 1) of the sparsified gradients; same for V with G~^2."""
    rng = np.random.default_rng(4)
    d, r, k = 600, 80, 12
    At = synth.gaussian_matrix(3, d, r)
    A = At.astype(np.float64).T
    m = np.zeros(r, np.float32)
    v = np.zeros(r, np.float32)
    Md = np.zeros(d)
    Vd = np.zeros(d)
    b1, b2 = 0.9, 0.999
    for t in range(1, 6):
        g = rng.standard_normal((1, d)).astype(np.float32)
        idx, val = orc.topk(g, k)
        p, q = orc.project(idx, val, At)
        m, v, mh, vh = orc.adam(p[0], q[0], m, v, t)
        gs = np.zeros(d)
        gs[idx[0]] = val[0]
        Md = b1 * Md + (1 - b1) * gs
        Vd = b2 * Vd + (1 - b2) * gs**2
        assert np.allclose(m, A @ Md, rtol=0, atol=5e-6 * np.abs(A @ Md).max())
        assert np.allclose(v, A @ Vd, rtol=0, atol=5e-6 * np.abs(A @ Vd).max())
        assert np.allclose(mh, A @ (Md / (1 - b1**t)), rtol=0, atol=5e-6 * np.abs(mh).max())
        assert np.allclose(vh, A @ (Vd / (1 - b2**t)), rtol=0, atol=5e-6 * np.abs(vh).max())


def test_state_counts_printed_in_the_paper():
    for line in open(os.path.join(GOLD, "paper_state_counts.txt")):
        if line.startswith("#"):
            continue
        kappa, c, sc, states = map(int, line.split())
        r = kappa * sc  # measurements per chunk
        m = np.zeros((c, r), np.float32)
        v = np.zeros((c, r), np.float32)
        assert m.size + v.size == states


# ----------------------------------------------------------------------------- OMP
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_omp_exact_recovery_of_sparse_signals(seed):
    """Sec. 4.3: a k-sparse x is reconstructed from y = A x when A is iid normal with enough
    measurements (here r >= 4 k ln d)."""
    d, k, r = 1024, 8, 256
    At = synth.gaussian_matrix(seed + 20, d, r)
    x, pos = synth.sparse_signal(seed, d, k)
    y = (At.astype(np.float64).T @ x).astype(np.float32)
    out = orc.omp(y, At, k)
    assert sorted(out["sel"].tolist()) == pos.tolist()
    rec = np.zeros(d)
    rec[out["sel"]] = out["x64"]
    assert np.abs(rec - x).max() < 1e-5
    assert np.linalg.norm(out["res"]) < 1e-5 * np.linalg.norm(y)


def exhaustive_best_support(y, A, k):
    best, arg = np.inf, None
    for S in itertools.combinations(range(A.shape[1]), k):
        sol, *_ = np.linalg.lstsq(A[:, S], y, rcond=None)
        rn = np.linalg.norm(y - A[:, S] @ sol)
        if rn < best:
            best, arg = rn, S
    return arg, best


@pytest.mark.parametrize("d,k,r,seed", [(12, 1, 6, 0), (16, 2, 8, 1), (20, 3, 10, 2), (18, 3, 9, 3)])
def test_omp_equals_exhaustive_search_on_tiny_problems(d, k, r, seed):
    At = synth.gaussian_matrix(seed + 50, d, r)
    A = At.astype(np.float64).T
    x, pos = synth.sparse_signal(seed + 9, d, k)
    y = (A @ x).astype(np.float32)
    S, rn = exhaustive_best_support(y.astype(np.float64), A, k)
    assert rn < 1e-6 and list(S) == pos.tolist()
    out = orc.omp(y, At, k)
    assert sorted(out["sel"].tolist()) == list(S)
    sol, *_ = np.linalg.lstsq(A[:, out["sel"]], y.astype(np.float64), rcond=None)
    assert np.allclose(out["x64"], sol, rtol=1e-9, atol=1e-12)


def test_omp_first_pick_is_best_single_atom_fit_with_unequal_column_norms():
    """The selection rule divides by the column norm (App. B): the first pick is the atom whose
    one-atom least-squares fit leaves the smallest residual, whatever the column scales."""
    rng = np.random.default_rng(8)
    d, r = 200, 40
    At = synth.gaussian_matrix(4, d, r) * rng.uniform(0.05, 20, size=(d, 1)).astype(np.float32)
    A = At.astype(np.float64).T
    for t in range(10):
        y = rng.standard_normal(r).astype(np.float32)
        out = orc.omp(y, At, 1)
        resid = [np.linalg.norm(y - A[:, i] * (A[:, i] @ y) / (A[:, i] @ A[:, i])) for i in range(d)]
        assert out["sel"][0] == int(np.argmin(resid))


def test_omp_invariants_in_the_noisy_regime():
    """Each iteration is the least-squares fit on the chosen support: residual orthogonal to the
    selected columns, residual norm non-increasing, values equal to a library least squares, and
    every pick maximises the normalised correlation with the previous residual."""
    rng = np.random.default_rng(12)
    d, r, k = 400, 64, 10
    At = synth.gaussian_matrix(6, d, r)
    A = At.astype(np.float64).T
    nrm = np.linalg.norm(A, axis=0)
    assert np.allclose(orc.colnorms(At), nrm, rtol=1e-14)
    y = rng.standard_normal(r).astype(np.float32)  # not sparse at all
    full = orc.omp(y, At, k, want_top2=True)
    prev = np.linalg.norm(y)
    res = y.astype(np.float64)
    for j in range(1, k + 1):
        score = np.abs(A.T @ res) / nrm
        score[full["sel"][: j - 1]] = -1
        assert full["sel"][j - 1] == int(np.argmax(score))
        top = np.sort(score)[::-1][:2]
        assert np.allclose(full["top2"][j - 1], top, rtol=1e-10)
        pre = orc.omp(y, At, j)
        assert np.array_equal(pre["sel"], full["sel"][:j])
        S = pre["sel"]
        sol, *_ = np.linalg.lstsq(A[:, S], y.astype(np.float64), rcond=None)
        assert np.allclose(pre["x64"], sol, rtol=1e-9, atol=1e-12)
        res = y - A[:, S] @ sol
        assert np.allclose(pre["res"], res, atol=1e-12)
        assert np.abs(A[:, S].T @ pre["res"]).max() < 1e-10 * np.linalg.norm(y)
        assert np.linalg.norm(pre["res"]) <= prev + 1e-12
        prev = np.linalg.norm(pre["res"])


def test_omp_forced_prefix_and_zero_input():
    rng = np.random.default_rng(13)
    d, r, k = 300, 48, 6
    At = synth.gaussian_matrix(7, d, r)
    y = rng.standard_normal(r).astype(np.float32)
    full = orc.omp(y, At, k)
    again = orc.omp(y, At, k, forced=full["sel"][:4])
    assert np.array_equal(again["sel"], full["sel"]) and np.array_equal(again["x"], full["x"])
    other = orc.omp(y, At, 3, forced=np.array([5, 9], np.int32))
    assert other["sel"][:2].tolist() == [5, 9] and other["sel"][2] not in (5, 9)
    zero = orc.omp(np.zeros(r, np.float32), At, 4)
    assert zero["sel"].tolist() == [0, 1, 2, 3] and not zero["x"].any()
    sel, x = orc.omp_batch(np.stack([y, np.zeros(r, np.float32)]), At, k)
    assert np.array_equal(sel[0], full["sel"]) and np.array_equal(x[0], full["x"])
    assert sel[1].tolist() == list(range(k))


def test_single_pick_after_a_given_prefix():
    """oracle.omp_pick (one iteration of the definition after a given prefix) against numpy: a library least
    squares on an ARBITRARY prefix (not one OMP would choose), the residual, and the argmax of the
    normalised correlation over the unselected positions; and against oracle.omp's own picks."""
    rng = np.random.default_rng(21)
    d, r = 500, 80
    At = synth.gaussian_matrix(8, d, r) * rng.uniform(0.2, 5.0, size=(d, 1)).astype(np.float32)  # unequal norms
    A = At.astype(np.float64).T
    nrm = np.linalg.norm(A, axis=0)
    y = rng.standard_normal(r).astype(np.float32)
    for n_prefix in (0, 1, 7, 40):
        prefix = rng.choice(d, size=n_prefix, replace=False).astype(np.int32)
        got = orc.omp_pick(y, At, prefix)
        res = y.astype(np.float64)
        if n_prefix:
            sol, *_ = np.linalg.lstsq(A[:, prefix], y.astype(np.float64), rcond=None)
            res = res - A[:, prefix] @ sol
        score = np.abs(A.T @ res) / nrm
        score[prefix] = -1
        assert got["lam"] == int(np.argmax(score))
        assert np.allclose(got["top2"], np.sort(score)[::-1][:2], rtol=1e-10)
        assert np.allclose(got["res"], res, atol=1e-12)
    full = orc.omp(y, At, 12)
    for j in range(12):
        assert orc.omp_pick(y, At, full["sel"][:j])["lam"] == full["sel"][j]
    # exact ties go to the lowest unselected position; a repeated prefix position is refused
    assert orc.omp_pick(np.zeros(r, np.float32), At, np.array([0, 2], np.int32))["lam"] == 1
    with pytest.raises(ValueError):
        orc.omp_pick(y, At, np.array([3, 3], np.int32))


def test_philox_matrix_filled_by_threads_is_the_same_matrix():
    assert np.array_equal(orc.philox_matrix_threads(77, 1000, 36, workers=3), orc.philox_matrix(77, 1000, 36))


# ----------------------------------------------------------------------- full step
def test_apply_formula_by_hand():
    # eq. 11 with alpha=2, eps=0.5, lr=0.1: N = 2*x/(sqrt(z)+0.5)
    d = 8
    W = np.arange(8, dtype=np.float32).reshape(1, 8)
    sel_m = np.array([[6, 1, 3]], np.int32)
    x_m = np.array([[3.0, -1.0, 2.0]], np.float32)
    sel_v = np.array([[1, 6, 5]], np.int32)
    x_v = np.array([[4.0, -9.0, 1.0]], np.float32)
    out = orc.apply(W, d, sel_m, x_m, sel_v, x_v, alpha=2.0, eps=0.5, lr=0.1)
    exp = np.arange(8, dtype=np.float64)
    exp[6] -= 0.1 * 2 * 3.0 / (0.0 + 0.5)      # negative second moment -> 0
    exp[1] -= 0.1 * 2 * -1.0 / (2.0 + 0.5)
    exp[3] -= 0.1 * 2 * 2.0 / (0.0 + 0.5)      # missing second moment -> 0
    assert np.allclose(out.ravel(), exp, rtol=1e-6)


@pytest.mark.parametrize("shared", [False, True])
def test_first_step_closed_form_in_exact_recovery_regime(shared):
    """With zero initial moments Mhat_1 = p and Vhat_1 = q (Alg. 2), so when OMP recovers the
    k-sparse G~ and G~^2 exactly, N_1 = alpha G~/(|G~| + eps) on the top-k support (eq. 11)."""
    w = synth.shrink(synth.CFG1, C=3, d=2048, r=512, k=8)
    g = synth.gradients(w, 1)
    At = synth.gaussian_matrix(1, w.d, w.r)
    W0 = synth.weights(w)
    z = np.zeros((w.C, w.r), np.float32)
    alpha, eps, lr = 2.0, 1e-8, 1e-3
    out = orc.step(g, W0, z, z, 1, At, w.k, alpha=alpha, eps=eps, lr=lr, shared_support=shared)
    assert np.allclose(out["mhat"], out["p"], rtol=2e-6, atol=0)
    assert np.allclose(out["vhat"], out["q"], rtol=2e-6, atol=0)
    exp = W0.astype(np.float64).copy().reshape(w.C, w.d)
    for c in range(w.C):
        assert sorted(out["sel_m"][c].tolist()) == out["idx"][c].tolist()
        assert sorted(out["sel_v"][c].tolist()) == out["idx"][c].tolist()
        gv = out["val"][c].astype(np.float64)
        exp[c, out["idx"][c]] -= lr * alpha * gv / (np.abs(gv) + eps)
    dW = out["W"].reshape(w.C, w.d).astype(np.float64) - W0.reshape(w.C, w.d)
    ref = exp - W0.reshape(w.C, w.d)
    assert np.abs(dW - ref).max() < 1e-4 * np.abs(ref).max()
    # untouched positions are bit-identical
    mask = np.ones((w.C, w.d), bool)
    for c in range(w.C):
        mask[c, out["idx"][c]] = False
    assert np.array_equal(out["W"].reshape(w.C, w.d)[mask], W0.reshape(w.C, w.d)[mask])


# --------------------------------------------------------------------------- shared-support recovery
@pytest.mark.parametrize("d,r,k,seed", [(50, 20, 1, 0), (300, 64, 7, 1), (1000, 128, 32, 2)])
def test_lstsq_on_a_support_equals_the_library_routine(d, r, k, seed):
    rng = np.random.default_rng(seed)
    At = synth.gaussian_matrix(seed + 40, d, r)
    sel = rng.permutation(d)[:k].astype(np.int32)
    y = rng.standard_normal(r).astype(np.float32)
    ref, *_ = np.linalg.lstsq(At[sel].astype(np.float64).T, y.astype(np.float64), rcond=None)
    got = orc.lstsq_support(y, At, sel)
    assert np.abs(got - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("seed", [0, 1])
def test_shared_support_recovers_both_moments_of_a_sparse_pair(seed):
    """Two k-sparse vectors with the same non-zero positions (G~ and G~^2 in Sec. 4.3) measured with
    the same A: the support comes from the first alone and both are reconstructed, each aligned with
    the selection order."""
    d, k, r = 1024, 8, 256
    At = synth.gaussian_matrix(seed + 60, d, r)
    x, pos = synth.sparse_signal(seed, d, k)
    z = x * x * 3.0
    A64 = At.astype(np.float64).T
    ym = (A64 @ x).astype(np.float32)[None]
    yv = (A64 @ z).astype(np.float32)[None]
    sel, xs, zs = orc.omp_shared(ym, yv, At, k)
    assert sorted(sel[0].tolist()) == pos.tolist()
    assert np.array_equal(sel[0], orc.omp(ym[0], At, k)["sel"])
    assert np.abs(xs[0] - x[sel[0]]).max() < 1e-5 * np.abs(x).max()
    assert np.abs(zs[0] - z[sel[0]]).max() < 1e-5 * np.abs(z).max()


def test_shared_support_fit_in_the_noisy_regime_is_the_projection_onto_the_support():
    """z is the least-squares fit of the SECOND right-hand side: its residual is orthogonal to the
    selected columns, and it differs from the fit of the first."""
    d, k, r = 400, 12, 48
    rng = np.random.default_rng(5)
    At = synth.gaussian_matrix(77, d, r)
    ym = rng.standard_normal((2, r)).astype(np.float32)
    yv = rng.standard_normal((2, r)).astype(np.float32)
    sel, xs, zs = orc.omp_shared(ym, yv, At, k)
    for c in range(2):
        As = At[sel[c]].astype(np.float64).T
        for y, sol in ((ym[c], xs[c]), (yv[c], zs[c])):
            ref, *_ = np.linalg.lstsq(As, y.astype(np.float64), rcond=None)
            assert np.abs(sol - ref).max() < 1e-5 * np.abs(ref).max()
        res = yv[c].astype(np.float64) - As @ orc.lstsq_support(yv[c], At, sel[c])
        assert np.abs(As.T @ res).max() < 1e-10 * np.linalg.norm(yv[c])
        assert np.abs(zs[c] - xs[c]).max() > 1e-3


# --------------------------------------------------------------------------- SGCA re-projection
def test_reprojection_equals_dense_matvec_and_scales():
    rng = np.random.default_rng(11)
    d, r, k, N = 700, 48, 9, 3
    At2 = synth.gaussian_matrix(9, d, r)
    sel = np.stack([rng.permutation(d)[:k] for _ in range(N)]).astype(np.int32)   # selection order, not sorted
    x = rng.standard_normal((N, k)).astype(np.float32)
    out = orc.reproject(sel, x, At2, scale=0.271)
    for n in range(N):
        dense = np.zeros(d)
        dense[sel[n]] = x[n]
        ref = 0.271 * (At2.astype(np.float64).T @ dense)
        assert np.abs(out[n] - ref).max() < 1e-6 * np.abs(ref).max()


@pytest.mark.parametrize("shared", [False, True])
def test_sgca_keeps_the_moments_aligned_with_the_new_matrix(shared):
    """App. C: after M <- A' OMP_A(M) the state is the projection, with the NEW matrix, of the same
    dense moment (eq. 10 with A' in place of A), and stays so over the following steps. Gradients
    with one fixed k-sparse support keep every recovery exact."""
    d, r, k, C = 1024, 256, 8, 2
    A1 = synth.gaussian_matrix(31, d, r)
    A2 = synth.gaussian_matrix(32, d, r)
    rng = np.random.default_rng(2)
    support = np.sort(rng.permutation(d)[:k])
    m = np.zeros((C, r), np.float32)
    v = np.zeros((C, r), np.float32)
    W = np.zeros(C * d, np.float32)
    Md = np.zeros((C, d))
    Vd = np.zeros((C, d))
    b1, b2 = 0.9, 0.999
    At = A1
    for t in range(1, 5):
        g = np.zeros((C, d), np.float32)
        g[:, support] = rng.standard_normal((C, k)).astype(np.float32) + 3.0 * np.sign(rng.standard_normal((C, k))).astype(np.float32)
        out = orc.step(g, W, m, v, t, At, k, shared_support=shared, At_new=A2 if t == 2 else None)
        Md = b1 * Md + (1 - b1) * g.astype(np.float64)
        Vd = b2 * Vd + (1 - b2) * g.astype(np.float64) ** 2
        if t == 2:
            At = A2
        A64 = At.astype(np.float64).T
        for c in range(C):
            assert sorted(out["sel_m"][c].tolist()) == support.tolist()
            assert np.abs(out["m"][c] - A64 @ Md[c]).max() < 2e-5 * np.abs(A64 @ Md[c]).max(), t
            assert np.abs(out["v"][c] - A64 @ Vd[c]).max() < 2e-5 * np.abs(A64 @ Vd[c]).max(), t
        m, v, W = out["m"], out["v"], out["W"]


# --------------------------------------------------------------------------- CESGC outer projection
def test_outer_projection_by_hand():
    # Sec. 4.4: Gc = B G; update W - lr B^T N. One row B = (0.6, 0.8), G = [[1, 2], [3, 4]].
    B = np.array([[0.6, 0.8]], np.float32)
    G = np.array([[1.0, 2.0], [3.0, 4.0]], np.float32)
    Gc = orc.outer_project(B, G)
    assert np.allclose(Gc, [[0.6 + 2.4, 1.2 + 3.2]], rtol=1e-6)
    # one chunk of d = 2, k = 1: x = 2 at position 1, z = 4 there: N = (0, 1 * 2 / (2 + 0.5)) = (0, 0.8)
    W = np.array([[10.0, 20.0], [30.0, 40.0]], np.float32)
    out = orc.outer_apply(W, B, 2, np.array([[1]], np.int32), np.array([[2.0]], np.float32),
                          np.array([[1]], np.int32), np.array([[4.0]], np.float32), alpha=1.0, eps=0.5, lr=0.5)
    assert np.allclose(out, [[10.0, 20.0 - 0.5 * 0.6 * 0.8], [30.0, 40.0 - 0.5 * 0.8 * 0.8]], rtol=1e-6)


def test_outer_projection_equals_the_library_product():
    rng = np.random.default_rng(3)
    rho, m, n = 5, 37, 24          # all different: a transposed operand or a swapped size fails
    B = rng.standard_normal((rho, m)).astype(np.float32)
    G = rng.standard_normal((m, n)).astype(np.float32)
    ref = B.astype(np.float64) @ G.astype(np.float64)
    assert np.abs(orc.outer_project(B, G) - ref).max() < 1e-6 * np.abs(ref).max()
    # back-projection: d = 8 -> 15 chunks of the 5 x 24 compressed space, k = 2
    d, k = 8, 2
    C = rho * n // d
    sel_m = np.stack([rng.permutation(d)[:k] for _ in range(C)]).astype(np.int32)
    sel_v = sel_m[:, ::-1].copy()
    x = rng.standard_normal((C, k)).astype(np.float32)
    z = np.abs(rng.standard_normal((C, k))).astype(np.float32) + 0.1
    W = rng.standard_normal((m, n)).astype(np.float32)
    out = orc.outer_apply(W, B, d, sel_m, x, sel_v, z, alpha=2.0, eps=1e-3, lr=0.01)
    N = np.zeros((C, d))
    for c in range(C):
        zz = dict(zip(sel_v[c].tolist(), z[c].astype(np.float64)))
        for t in range(k):
            N[c, sel_m[c, t]] = 2.0 * float(x[c, t]) / (np.sqrt(zz[int(sel_m[c, t])]) + 1e-3)
    ref = W.astype(np.float64) - 0.01 * B.astype(np.float64).T @ N.reshape(rho, n)
    assert np.abs(out - ref).max() < 1e-6 * np.abs(ref).max()


def test_identity_outer_projection_is_the_plain_sgc_step():
    """B = I (rho = m): CESGC is SGC on the gradient read row-major."""
    w = synth.shrink(synth.CFG1, C=4, d=512, r=128, k=6)
    m_rows, n = 8, 256                                  # 8 x 256 weights = 4 chunks of 512
    g = synth.gradients(w, 1)
    At = synth.gaussian_matrix(1, w.d, w.r)
    W0 = synth.weights(w)
    z = np.zeros((w.C, w.r), np.float32)
    plain = orc.step(g, W0, z, z, 1, At, w.k, alpha=2.0)
    eye = np.eye(m_rows, dtype=np.float32)
    ces = orc.step_cesgc(g.reshape(m_rows, n), W0.reshape(m_rows, n), eye, z, z, 1, At, w.d, w.k, alpha=2.0)
    assert np.array_equal(ces["Gc"].ravel(), g.ravel())
    assert np.array_equal(ces["sel_m"], plain["sel_m"]) and np.array_equal(ces["x_v"], plain["x_v"])
    assert np.array_equal(ces["W"].ravel(), plain["W"].ravel())


def test_outer_projection_with_orthonormal_rows():
    """B B^T = I: compressing a gradient that lies in the row space of B loses nothing, and the
    weight change, compressed again, is the update N itself."""
    rho, m, n, d, k = 4, 64, 32, 16, 3
    B = synth.orthonormal_rows(0, rho, m)
    rng = np.random.default_rng(5)
    X = rng.standard_normal((rho, n)).astype(np.float32)
    G = (B.astype(np.float64).T @ X).astype(np.float32)
    assert np.abs(orc.outer_project(B, G) - X).max() < 1e-6
    C = rho * n // d
    sel = np.stack([rng.permutation(d)[:k] for _ in range(C)]).astype(np.int32)
    x = rng.standard_normal((C, k)).astype(np.float32)
    zv = np.ones((C, k), np.float32)
    W = np.zeros((m, n), np.float32)
    out = orc.outer_apply(W, B, d, sel, x, sel, zv, alpha=1.0, eps=0.0, lr=1.0)
    N = np.zeros((C, d))
    for c in range(C):
        N[c, sel[c]] = x[c]
    back = B.astype(np.float64) @ (-out.astype(np.float64))
    assert np.abs(back - N.reshape(rho, n)).max() < 1e-6


def test_synthetic_matrix_gradient_has_the_given_leading_directions():
    """The input recipe of the CESGC workload: the first rows of the basis span what a truncated SVD
    of the gradient returns (checked against the library SVD on a small case)."""
    m, n, rho = 96, 128, 4
    basis = synth.orthonormal_rows(2, 12, m)
    G = synth.matrix_gradient(2, 1, m, n, basis)
    U = np.linalg.svd(G.astype(np.float64), full_matrices=False)[0][:, :rho]
    P_svd = U @ U.T
    P_b = basis[:rho].astype(np.float64).T @ basis[:rho].astype(np.float64)
    assert np.abs(P_svd - P_b).max() < 0.15


# --------------------------------------------------------------------------- CESGC: the refresh of B
def _factors(rng, m, n, sigma):
    """G = U diag(sigma) V^T with orthonormal columns U [m, q], V [n, q] built by Gram-Schmidt (QR) of
    random matrices: the decomposition is known without calling the routine under test."""
    q = len(sigma)
    U, _ = np.linalg.qr(rng.standard_normal((m, q)))
    V, _ = np.linalg.qr(rng.standard_normal((n, q)))
    return U, V, (U * sigma) @ V.T


def test_refresh_returns_the_factors_a_matrix_was_built_from():
    # Sec. 4.4: B = the leading left singular vectors, as rows. Distinct singular values: unique up to sign.
    rng = np.random.default_rng(41)
    sigma = np.array([9.0, 5.0, 3.0, 2.0, 0.5, 0.1])
    U, V, G = _factors(rng, 20, 31, sigma)
    B, s = orc.outer_refresh(G, 4)
    assert B.shape == (4, 20)
    assert np.abs(s - sigma[:4]).max() < 1e-12
    for i in range(4):
        u = U[:, i] * np.sign(U[np.argmax(np.abs(U[:, i])), i])
        assert np.abs(B[i] - u).max() < 1e-12, i           # a transposed or column-sliced result fails here


def test_refresh_rows_are_orthonormal_and_capture_the_most_energy():
    # Eckart-Young: among all rho x m matrices with orthonormal rows, B maximises ||B G||_F, and the
    # maximum is the root of the sum of the rho largest squared singular values
    rng = np.random.default_rng(42)
    G = rng.standard_normal((15, 40)) * (0.8 ** np.arange(15))[:, None]
    B, s = orc.outer_refresh(G, 5)
    assert np.abs(B @ B.T - np.eye(5)).max() < 1e-12
    best = np.linalg.norm(B @ G)
    assert abs(best - np.sqrt((s ** 2).sum())) < 1e-10
    evals = np.sort(np.linalg.eigvalsh(G @ G.T))[::-1]     # another route to the singular values
    assert np.abs(s ** 2 - evals[:5]).max() < 1e-10 * evals[0]
    for trial in range(20):
        Q, _ = np.linalg.qr(rng.standard_normal((15, 5)))
        assert np.linalg.norm(Q.T @ G) <= best + 1e-12


def test_refresh_of_a_diagonal_matrix_picks_the_largest_entries():
    G = np.zeros((5, 7))
    for i, val in enumerate([2.0, -7.0, 0.5, 4.0, 1.0]):
        G[i, i] = val
    B, s = orc.outer_refresh(G, 3)
    assert np.array_equal(s, [7.0, 4.0, 2.0])
    assert np.array_equal(np.argmax(np.abs(B), axis=1), [1, 3, 0])
    assert np.abs(np.abs(B).sum(axis=1) - 1).max() < 1e-15 and (B.sum(axis=1) > 0).all()


# --------------------------------------------------------------------------- App. B: the recurrences
def test_appendix_b_recurrences_reach_the_definition():
    """App. B (Alg. 3) never forms a residual: it carries the correlation vector p, the images
    b_t = A^H q_t of the orthonormal directions and the inverse Cholesky factor F, and states
    p <- p - b_j a_j, b_j = gamma_j (G_:lambda - B c), a_j = gamma_j p_lambda (p before the update),
    gamma_j = 1/sqrt(G_ll - c.c), c = F^H w, x = F a. Written out here in double exactly as stated (with
    F_1 = gamma_1, the only reading under which x = F a is the least-squares solution), it must make the
    oracle's selections, reproduce its least-squares values and keep p equal to A^H (y - A_Lambda x):
    the oracle follows the plain definition, so this pins both it and the reading of App. B the GPU
    engines use."""
    rng = np.random.default_rng(77)
    d, r, k = 300, 48, 10
    At = (rng.standard_normal((d, r)) / np.sqrt(r)).astype(np.float32)
    y = rng.standard_normal(r).astype(np.float32)
    ref = orc.omp(y, At, k)
    A = At.astype(np.float64).T                       # r x d
    G = A.T @ A
    norms = np.sqrt(np.diag(G))
    p = A.T @ y.astype(np.float64)
    F = np.zeros((k, k))
    a = np.zeros(k)
    B = np.zeros((d, k))
    lam_list = []
    for j in range(k):
        score = np.abs(p) / norms
        score[lam_list] = -1.0
        lam = int(np.argmax(score))
        assert lam == ref["sel"][j], j
        w = G[lam_list, lam]
        c = F[:j, :j].T @ w
        gamma = 1.0 / np.sqrt(G[lam, lam] - c @ c)
        b = gamma * (G[:, lam] - B[:, :j] @ c)
        F[:j, j] = -gamma * (F[:j, :j] @ c)
        F[j, j] = gamma
        a[j] = gamma * p[lam]
        p = p - b * a[j]
        B[:, j] = b
        lam_list.append(lam)
        x = F[:j + 1, :j + 1] @ a[:j + 1]
        res = y.astype(np.float64) - A[:, lam_list] @ x
        assert np.abs(p - A.T @ res).max() < 1e-12 * np.abs(y).max() * 10
    assert np.abs(x - ref["x64"]).max() < 1e-10 * np.abs(ref["x64"]).max()
    assert np.abs(res - ref["res"]).max() < 1e-10
