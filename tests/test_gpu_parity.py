"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: positions (top-k, OMP support in selection order) and the generated matrix bit-exact;
projections, moments, recovered values and weight updates within 1e-4 of the per-vector maximum
(max|gpu-ref| / max|ref| per chunk vector)."""
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


def rowwise_relerr(a, ref):
    return max(relerr(a[i], ref[i]) for i in range(len(ref)))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def make_matrix(mode, seed, d, r):
    """(sgc.Matrix with device buffers and inverse norms, host At for the oracle)"""
    if mode == "stored":
        At = synth.gaussian_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=dev(At))
    else:
        At = orc.philox_matrix(seed, d, r)
        A = sgc.Matrix(d, r, At=None, seed=seed)
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    return A, At


# ------------------------------------------------------------------ generated matrix
def test_generated_matrix_is_bit_identical_to_the_oracle():
    for seed, r, row0, rows in [(1, 64, 0, 300), (0xDEADBEEF12345678, 1024, 16000, 40), (7, 8, 5, 1)]:
        say("matrix_fill", seed, r, row0, rows)
        out = torch.empty((rows, r), dtype=torch.float32, device=DEV)
        sgc.sgc_matrix_fill(seed, r, row0, rows, out)
        ref = orc.philox_matrix(seed, row0 + rows, r, row0, rows)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("mode", ["stored", "philox"])
def test_column_norms(mode):
    A, At = make_matrix(mode, 3, 777, 96)
    ref = 1.0 / orc.colnorms(At)
    assert relerr(A.inv_colnorm.cpu().numpy(), ref) < 1e-6


# ------------------------------------------------------------------------------ top-k
def run_topk_project(g, k, A):
    C, d = g.shape
    gd = dev(g)
    idx = torch.empty((C, k), dtype=torch.int32, device=DEV)
    val = torch.empty((C, k), dtype=torch.float32, device=DEV)
    p = torch.empty((C, A.r), dtype=torch.float32, device=DEV)
    q = torch.empty((C, A.r), dtype=torch.float32, device=DEV)
    sgc.sgc_sparsify_project(gd, C * d, d, k, A, idx, val, p, q)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), val.cpu().numpy(), p.cpu().numpy(), q.cpu().numpy()


@pytest.mark.parametrize("C,d,k,r,mode", [
    (3, 1, 1, 4, "stored"), (4, 7, 3, 8, "stored"), (5, 1000, 17, 32, "philox"), (2, 4096, 32, 256, "stored"),
    (3, 5003, 256, 256, "stored"), (2, 16384, 64, 1024, "philox"), (2, 20001, 100, 128, "stored"),
    (2, 65536, 256, 2048, "stored"), (2, 65537, 300, 512, "philox"), (1, 70001, 129, 256, "philox"),
    (3, 16385, 64, 64, "philox"), (2, 4100, 4, 8, "philox"),
])
def test_sparsify_project_matches_oracle(C, d, k, r, mode):
    say("sparsify_project", C, d, k, r, mode)
    rng = np.random.default_rng(d + k)
    g = (rng.standard_t(3, size=(C, d)) * 1e-3).astype(np.float32)
    A, At = make_matrix(mode, 11, d, r)
    idx, val, p, q = run_topk_project(g, k, A)
    ridx, rval = orc.topk(g, k)
    assert np.array_equal(idx, ridx)
    assert np.array_equal(val.view(np.uint32), rval.view(np.uint32))
    rp, rq = orc.project(ridx, rval, At)
    assert rowwise_relerr(p, rp) < TOL and rowwise_relerr(q, rq) < TOL


def test_topk_ties_zeros_and_quantised_values():
    rng = np.random.default_rng(2)
    A, At = make_matrix("stored", 5, 3000, 64)
    g = rng.integers(-3, 4, size=(6, 3000)).astype(np.float32)   # thousands of ties at the threshold
    g[1] = 0.0                                                   # all-zero chunk
    g[2] = 1.0                                                   # all equal
    g[3, ::2] *= -1
    g[4] = np.where(rng.random(3000) < 0.5, -0.0, 0.0)           # signed zeros
    for k in (1, 37, 64):
        idx, val, p, q = run_topk_project(g, k, A)
        ridx, rval = orc.topk(g, k)
        assert np.array_equal(idx, ridx)
        assert np.array_equal(val.view(np.uint32), rval.view(np.uint32))


@pytest.mark.parametrize("d,k,r", [
    (64, 8, 8), (5000, 64, 64), (16384, 64, 64),      # the register-resident single-pass kernel
    (32768, 64, 128), (65536, 100, 512),              # two and four pieces merged in a second pass
    (65536, 256, 256), (70000, 100, 128),             # the single pass for long chunks, the general kernel
])
def test_topk_values_one_ulp_apart_around_the_kth_place(d, k, r):
    """The k-th largest magnitude sits in a cluster of values one unit in the last place apart (with ties):
    any comparison that drops the lowest mantissa bit, or compares rounded values, picks a different set."""
    say("topk one-ulp cluster", d, k, r)
    g = synth.ulp_cluster_gradients(2, 5, d, k)
    A, At = make_matrix("stored", 13, d, r)
    idx, val, p, q = run_topk_project(g, k, A)
    ridx, rval = orc.topk(g, k)
    assert np.array_equal(idx, ridx)
    assert np.array_equal(val.view(np.uint32), rval.view(np.uint32))


@pytest.mark.parametrize("d,k,r", [
    (16392, 1, 8),        # two pieces, the smallest possible scratch (r = 2 k would do: 8 >= 2)
    (32768, 64, 128),     # two pieces, r = S k exactly
    (32768, 64, 124),     # one candidate short of the scratch: the single-pass kernel
    (49152, 100, 300),    # three pieces
    (65536, 128, 512),    # four pieces, the largest k of the two-pass path, r = S k exactly
    (65536, 129, 1024),   # one more: single pass
    (65536, 1, 8),        # the paper's memory-efficient setting
    (40000, 30, 512),     # 40000 % 12 != 0: single pass
    (131072, 100, 800),   # eight pieces
    (262144, 64, 1024),   # sixteen pieces, 1024 candidates to merge
    (262144, 65, 2048),   # 1040 candidates: the general kernel
])
def test_topk_long_chunks_two_pass(d, k, r):
    """Chunks of 16385 .. 65536 floats are cut in up to four pieces whose candidates are merged in a second
    pass (p and q serve as scratch until the projection writes them). Heavy tails, thousands of ties at
    the threshold, an all-zero and an all-equal chunk, ties across the piece boundaries, NaN patterns."""
    say("topk two-pass", d, k, r)
    rng = np.random.default_rng(d + 3 * k)
    C = 7
    g = (rng.standard_t(3, size=(C, d)) * 1e-3).astype(np.float32)
    g[1] = rng.integers(-2, 3, size=d).astype(np.float32)        # ties everywhere, also across pieces
    g[2] = 0.0
    g[3] = -1.5
    g[4, : d // 2] = 0.0                                         # the whole result lies in the last pieces
    g[5, d // 3:] = 0.0                                          # ... in the first
    bits = g.view(np.uint32)
    bits[6, 5] = 0x7fc00000                                      # NaN patterns order above everything, by bits
    bits[6, d - 1] = 0xffc00001
    bits[6, d // 2] = 0x7f800000
    A, At = make_matrix("stored", 12, d, r)
    idx, val, p, q = run_topk_project(g, k, A)
    ridx, rval = orc.topk(g, k)
    assert np.array_equal(idx, ridx)
    assert np.array_equal(val.view(np.uint32), rval.view(np.uint32))
    rp, rq = orc.project(ridx[:6], rval[:6], At)
    assert rowwise_relerr(p[:6], rp) < TOL and rowwise_relerr(q[:6], rq) < TOL


def test_topk_nan_inf_and_subnormal_patterns():
    """Order is defined on the bit pattern with the sign cleared: NaN patterns above infinity,
    subnormals below every normal value. Chunks: NaNs and infinities among normal values; only
    subnormals and zeros (the k-th largest is subnormal); plain values next to them in one launch."""
    rng = np.random.default_rng(8)
    C, d, k = 4, 16384, 64
    g = rng.standard_normal((C, d)).astype(np.float32)
    bits = g.view(np.uint32)
    bits[0, 5] = 0x7fc00000; bits[0, 9000] = 0xffc00123; bits[0, 77] = 0x7f800000; bits[0, 16383] = 0xff800000
    g[1] = 0.0
    sub = rng.integers(1, 0x007fffff, size=200).astype(np.uint32)
    bits[1, rng.permutation(d)[:200]] = sub | (rng.integers(0, 2, size=200).astype(np.uint32) << 31)
    bits[2, 100:140] = 0x7f800000   # 40 infinities, tie among themselves
    gd = dev(g)
    A, At = make_matrix("stored", 3, d, 64)
    idx = torch.empty((C, k), dtype=torch.int32, device=DEV)
    val = torch.empty((C, k), dtype=torch.float32, device=DEV)
    p = torch.empty((C, 64), dtype=torch.float32, device=DEV)
    sgc.sgc_sparsify_project(gd, C * d, d, k, A, idx, val, p, None)
    torch.cuda.synchronize()
    ridx, rval = orc.topk(g, k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.array_equal(val.cpu().numpy().view(np.uint32), rval.view(np.uint32))


@pytest.mark.parametrize("C,d,k", [(3, 3000, 100), (2, 16384, 64), (2, 262144, 1024)])
def test_topk_bf16(C, d, k):
    say("topk bf16", C, d, k)
    w = synth.shrink(synth.CFG5, C=C, d=d, k=k, r=1024)
    bits = synth.gradients(w, 1)
    A, At = make_matrix("philox", 9, d, 1024) if d <= 16384 else (None, None)
    if A is None:  # large d: a small stored matrix would not match d; use a generated one without norms
        A = sgc.Matrix(d, 1024, At=None, seed=9)
    gd = dev(bits.view(np.int16))
    idx = torch.empty((C, k), dtype=torch.int32, device=DEV)
    val = torch.empty((C, k), dtype=torch.float32, device=DEV)
    p = torch.empty((C, 1024), dtype=torch.float32, device=DEV)
    q = torch.empty((C, 1024), dtype=torch.float32, device=DEV)
    sgc.sgc_sparsify_project(gd, C * d, d, k, A, idx, val, p, q)
    ridx, rval = orc.topk(bits, k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.array_equal(val.cpu().numpy().view(np.uint32), rval.view(np.uint32))
    if At is not None:
        rp, rq = orc.project(ridx, rval, At)
        assert rowwise_relerr(p.cpu().numpy(), rp) < TOL and rowwise_relerr(q.cpu().numpy(), rq) < TOL


@pytest.mark.parametrize("d,k", [
    (2048, 1), (2048, 256), (2056, 37), (4104, 100), (16384, 256), (16392, 5), (20008, 300), (65536, 1024),
    (262144, 1), (262144, 777), (100000, 1024), (1000, 10), (20004, 64),
])
def test_topk_bf16_edge_cases(d, k):
    """bfloat16 chunks through the two-sweep kernel (d % 8 == 0) and the general one: heavy tails, ties at the
    threshold (certain with 8-bit mantissas), quantised and constant chunks (everything reaches the bound: the
    list overflows and the chunk falls back), zeros, a single large entry, NaN and infinity patterns, values
    only in the last / first part of the chunk."""
    say("topk bf16 edge", d, k)
    rng = np.random.default_rng(d * 7 + k)
    C = 9
    g = rng.standard_t(2.5, size=(C, d)).astype(np.float32)
    g[1] = rng.integers(-2, 3, size=d).astype(np.float32)
    g[2] = 0.0
    g[3] = -1.5
    g[4, : d // 2] = 0.0
    g[5, d // 3:] = 0.0
    g[6] = 0.0
    g[6, d // 2] = 3.0
    g[7] *= 1e-30                                            # tiny magnitudes: small exponents, still bfloat16 normals
    bits = synth.f32_to_bf16_bits(g)
    bits[8, 5] = 0x7fc0
    bits[8, d - 1] = 0xffc1
    bits[8, d // 2] = 0x7f80
    bits[8, 7] = 0xff80
    A = sgc.Matrix(d, 1024, At=None, seed=9)
    idx = torch.empty((C, k), dtype=torch.int32, device=DEV)
    val = torch.empty((C, k), dtype=torch.float32, device=DEV)
    p = torch.empty((C, 1024), dtype=torch.float32, device=DEV)
    sgc.sgc_sparsify_project(dev(bits.view(np.int16)), C * d, d, k, A, idx, val, p, None)
    torch.cuda.synchronize()
    ridx, rval = orc.topk(bits, k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.array_equal(val.cpu().numpy().view(np.uint32), rval.view(np.uint32))


def test_empty_batch_is_a_no_op():
    A, _ = make_matrix("stored", 5, 64, 16)
    e = torch.empty(0, device=DEV)
    ei = torch.empty(0, dtype=torch.int32, device=DEV)
    g = torch.zeros(4, device=DEV)  # valid pointer, n = 0
    sgc.sgc_sparsify_project(g, 0, 64, 4, A, ei.new_empty(4), e.new_empty(4), e.new_empty(4), e.new_empty(4))
    sgc.sgc_adam_compressed(g, g, g, g, g, g, 0, 1, sgc.hyper())
    sgc.sgc_apply(g, 0, 64, 4, ei.new_empty(4), g, ei.new_empty(4), g, sgc.hyper())
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------- Adam
@pytest.mark.parametrize("n", [5 * 96 + 3, 4 * (3 * 1024 + 700) + 2, 4 * 1024 * 4100 + 1],
                         ids=["small", "ragged_pass", "more_passes_than_workgroups"])
def test_adam_matches_oracle_over_steps(n):
    rng = np.random.default_rng(3)   # n: not a multiple of 4
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    md, vd = dev(m), dev(v)
    mh = torch.empty(n, device=DEV)
    vh = torch.empty(n, device=DEV)
    h = sgc.hyper()
    for t in range(1, 6):
        p = rng.standard_normal(n).astype(np.float32)
        q = (rng.standard_normal(n) ** 2).astype(np.float32)
        sgc.sgc_adam_compressed(dev(p), dev(q), md, vd, mh, vh, n, t, h)
        m, v, rmh, rvh = orc.adam(p, q, m, v, t)
        for a, b in [(md, m), (vd, v), (mh, rmh), (vh, rvh)]:
            assert relerr(a.cpu().numpy(), b) < 1e-6
    # closed form of the first step from zero state: mhat = p, vhat = q
    md.zero_()
    vd.zero_()
    sgc.sgc_adam_compressed(dev(p), dev(q), md, vd, mh, vh, n, 1, h)
    assert relerr(mh.cpu().numpy(), p) < 1e-6 and relerr(vh.cpu().numpy(), q) < 1e-6


# -------------------------------------------------------------------------------- OMP
def run_omp(Y, A, k):
    N, r = Y.shape
    yd = dev(Y)
    sel = torch.empty((N, k), dtype=torch.int32, device=DEV)
    x = torch.empty((N, k), dtype=torch.float32, device=DEV)
    nbytes = sgc.sgc_omp_workspace_bytes(N, A.d, r, k)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    sgc.sgc_recover_omp(yd, N, A, k, sel, x, ws)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), x.cpu().numpy()


@pytest.mark.parametrize("N,d,r,k,mode", [
    (1, 100, 16, 4, "stored"),       # one ragged tile
    (5, 1000, 96, 12, "stored"),     # 8 position tiles with a ragged tail, 3 depth steps
    (5, 1000, 96, 12, "philox"),
    (2, 4096, 256, 32, "stored"),    # cfg1 shape
    (130, 700, 64, 8, "philox"),     # two right-hand-side tiles, ragged
    (3, 2000, 100, 10, "stored"),    # depth not a multiple of the staging depth
    (2, 2048, 512, 320, "stored"),   # k > 256: sixteen rows of F per lane in the update kernel
    (3, 32768, 64, 5, "stored"),     # many full position tiles, few right-hand sides: the half-width pipelined tile
    (64, 32768, 128, 3, "stored"),   # the same tile completely filled
    (3, 20000, 1024, 4, "philox"),   # a generated matrix too large to write out (80 MB, few right-hand sides):
                                     # regenerated inside the contraction and the selection kernel
])
def test_omp_matches_oracle_on_noisy_right_hand_sides(N, d, r, k, mode):
    say("omp", N, d, r, k, mode)
    rng = np.random.default_rng(N * 7 + d)
    A, At = make_matrix(mode, 21, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    sel, x = run_omp(Y, A, k)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    assert rowwise_relerr(x, rx) < TOL


@pytest.mark.parametrize("N,d,r,k,mode", [
    (128, 512, 4, 2, "stored"),       # the smallest depth, exactly one tile of right-hand sides, full position tiles
    (300, 1000, 8, 3, "stored"),      # ragged either way
    (300, 1000, 8, 3, "philox"),      # generated matrix, consumed from the panel
    (257, 777, 12, 5, "stored"),      # one right-hand side in the second tile, odd sizes
    (600, 70000, 16, 4, "philox"),    # the largest depth of this kernel, two halves on two streams, 274 position tiles
    (130, 65536, 8, 1, "stored"),     # the paper's memory-efficient setting: one pick from eight measurements
])
def test_omp_with_very_few_measurements(N, d, r, k, mode):
    """r <= 16 and at least 128 right-hand sides: the contraction without matrix cores (a thread per
    right-hand side). Exact ties, a zero and a tiny right-hand side included."""
    say("omp narrow", N, d, r, k, mode)
    rng = np.random.default_rng(N * 11 + d)
    A, At = make_matrix(mode, 27, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    Y[1] = 0.0
    Y[2] *= 1e-20
    Y[3] = np.round(Y[3])                           # small integers: equal scores are likely
    sel, x = run_omp(Y, A, k)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    assert rowwise_relerr(x, rx) < TOL


@pytest.mark.parametrize("N,d,r,k,flags", [
    (600, 3000, 64, 6, 0),       # the generated matrix is written out once (it fits the cache-sized panel)
    (1030, 2500, 8192, 3, 0),    # long columns, 82 MB, many right-hand sides: two panels refilled in every iteration, the second one ragged
    (520, 2500, 8192, 3, 0),     # the same matrix with fewer right-hand sides: regenerated inside the contraction (128-wide tiles)
    (300, 16640, 1024, 4, 0),    # 68 MB, regenerated inside the contraction in tiles of 256 right-hand sides, the second one ragged
    (400, 20480, 1024, 52, 0),   # 80 MB, the same kernel with the column copies of 52 iterations
    (400, 20480, 1024, 52, sgc.MATRIX_FLAG_MATERIALIZE),  # no larger than the column copies (d <= N k): written out whole in their place
])
def test_omp_generated_matrix_with_many_right_hand_sides(N, d, r, k, flags):
    say("omp panels", N, d, r, k)
    rng = np.random.default_rng(N + d)
    A, At = make_matrix("philox", 33, d, r)
    A.flags = flags
    Y = rng.standard_normal((N, r)).astype(np.float32)
    Y[7] = 0.0
    sel, x = run_omp(Y, A, k)
    norm = orc.colnorms(At)
    for n in [0, 1, 7, 127, 128, 255, 256, N - 2, N - 1]:   # the oracle checks a sample of the right-hand sides
        ref = orc.omp(Y[n], At, k, norm=norm)
        assert np.array_equal(sel[n], ref["sel"]), n
        assert relerr(x[n], ref["x"]) < TOL
    assert all(len(set(row.tolist())) == k for row in sel)


@pytest.mark.parametrize("N,d,r,k,mode", [
    (8400, 2048, 64, 4, "stored"),    # two halves of 8 x 33 = 264 tiles of 256 x 128 each: eight workgroups take a second tile; ragged last tiles
    (40000, 1024, 64, 3, "stored"),   # halves of 4 x 157 = 628 tiles: two or three per workgroup
    (9000, 4096, 128, 5, "philox"),   # generated matrix written to the panel; halves of 16 x 36 = 576 tiles
    (5000, 768, 192, 6, "stored"),    # 3 x 40 = 120 tiles: fewer than 128, the general kernel (one tile per workgroup)
])
def test_contraction_with_more_tiles_than_compute_units(N, d, r, k, mode):
    """The float contraction on full tiles runs as one workgroup per CU that walks its tiles (the next tile's first
    stages are loaded during the last stages of the current one). Sampled right-hand sides against the oracle, chosen
    at the edges of tiles and of the shares of a workgroup; supports distinct everywhere."""
    say("omp many tiles", N, d, r, k, mode)
    rng = np.random.default_rng(N + 3 * d + k)
    A, At = make_matrix(mode, 35, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    Y[129] = 0.0
    sel, x = run_omp(Y, A, k)
    norm = orc.colnorms(At)
    sample = sorted(set([0, 1, 127, 128, 129, 255, 256, N // 3, N // 2, (N // 128) * 128 - 1, (N // 128) * 128 if N % 128 else N - 128,
                         N - 2, N - 1] + [int(v) for v in rng.integers(0, N, size=24)]))
    for n in sample:
        ref = orc.omp(Y[n], At, k, norm=norm)
        assert np.array_equal(sel[n], ref["sel"]), n
        assert relerr(x[n], ref["x"]) < TOL, n
    assert all(len(set(row.tolist())) == k for row in sel)
    assert sel.min() >= 0 and sel.max() < d


@pytest.mark.parametrize("N,d,r,k,mode", [
    (2, 4096, 256, 32, "stored"),     # configuration 1's shape with both moments: 64 workgroups of 64 rows
    (1, 4096, 256, 32, "stored"),
    (4, 1000, 96, 12, "stored"),      # ragged: the last workgroup holds fewer rows
    (3, 2048, 220, 31, "stored"),     # the CESGC chunk shape (r not a multiple of 64)
    (2, 37, 16, 16, "stored"),        # fewer positions than lanes, k = r
    (4, 5, 8, 5, "stored"),           # d barely above the batch: workgroups without rows, k = d
    (2, 6000, 64, 1, "philox"),       # generated matrix written to the workspace panel first; one iteration
    (2, 300, 128, 128, "stored"),     # the largest k of this path
    (4, 24000, 64, 8, "stored"),      # 6.5 MB of rows: too much for 64 workers, the launches serve it
    (3, 70000, 16, 16, "stored"),     # 5.6 MB of short rows: 87 KiB slices of 1094 rows in 64 workers
    (1, 1, 4, 1, "stored"),           # the smallest problem there is
    (4, 513, 2048, 8, "stored"),      # the longest columns (N r = 8192, k r = 16384): one row more than 64 slices of 8
    (1, 9000, 1024, 16, "philox"),    # generated, 35 MB: written to the panel, too large for the workers' LDS
    (2, 3000, 256, 64, "stored"),     # the largest k of this path, k r = 16384
])
def test_small_batch_single_launch_recovery(N, d, r, k, mode):
    """At most four right-hand sides on a small resident matrix are recovered in one launch (resident workgroups
    that keep their rows of At in LDS and meet at a barrier twice per iteration). Against the oracle, and
    against the three-launches-per-iteration form of the same recovery (SGC_MATRIX_FLAG_MULTI_LAUNCH)."""
    say("omp single launch", N, d, r, k, mode)
    rng = np.random.default_rng(N * 1000 + d + k)
    A, At = make_matrix(mode, 41, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    if N > 2:
        Y[1] = 0.0                                   # all-zero right-hand side: every position ties
        Y[2] = np.round(2 * Y[2])                    # small integers: equal float scores are likely
    sel, x = run_omp(Y, A, k)
    assert sel.min() >= 0                            # -1 would mean the launch gave up waiting for its workgroups
    rsel, rx = orc.omp_batch(Y, At, k)
    assert np.array_equal(sel, rsel)
    assert rowwise_relerr(x, rx) < TOL
    A.flags = sgc.MATRIX_FLAG_MULTI_LAUNCH
    sel2, x2 = run_omp(Y, A, k)
    assert np.array_equal(sel, sel2) and rowwise_relerr(x, x2) < 1e-6
    # twice in a row on the same workspace: the barrier words of the first call must not leak into the second
    A.flags = 0
    yd = dev(Y)
    s3 = torch.empty((N, k), dtype=torch.int32, device=DEV)
    x3 = torch.empty((N, k), dtype=torch.float32, device=DEV)
    ws = torch.empty(sgc.sgc_omp_workspace_bytes(N, d, r, k), dtype=torch.uint8, device=DEV)
    for _ in range(3):
        sgc.sgc_recover_omp(yd, N, A, k, s3, x3, ws)
    torch.cuda.synchronize()
    assert np.array_equal(s3.cpu().numpy(), sel) and np.array_equal(x3.cpu().numpy().view(np.uint32), x.view(np.uint32))


def test_omp_exact_recovery_zero_and_oversized_k():
    d, r, k = 1024, 256, 8
    A, At = make_matrix("stored", 20, d, r)
    A64 = At.astype(np.float64).T
    Y = np.zeros((4, r), np.float32)
    x0, pos0 = synth.sparse_signal(0, d, k)
    x1, pos1 = synth.sparse_signal(1, d, 5)       # sparser than k: the last 3 picks see only rounding noise
    Y[0] = (A64 @ x0).astype(np.float32)
    Y[1] = (A64 @ x1).astype(np.float32)
    Y[3] = 1e-30                                   # tiny but not zero
    sel, x = run_omp(Y, A, k)
    rsel, rx = orc.omp_batch(Y, At, k)
    assert sorted(sel[0].tolist()) == pos0.tolist() and np.array_equal(sel[0], rsel[0])
    assert relerr(x[0], rx[0]) < TOL
    # right-hand side sparser than k: the meaningful picks are unique, the rest must be valid
    assert np.array_equal(sel[1][:5], rsel[1][:5]) and sorted(sel[1][:5].tolist()) == pos1.tolist()
    assert len(set(sel[1].tolist())) == k and sel[1].min() >= 0 and sel[1].max() < d
    assert relerr(x[1][:5], rx[1][:5]) < TOL and np.abs(x[1][5:]).max() < 1e-5
    # all-zero right-hand side: ties resolve to the lowest unselected position, values 0
    assert sel[2].tolist() == list(range(k)) and not x[2].any()
    assert np.array_equal(sel[3], rsel[3]) and relerr(x[3], rx[3]) < TOL


@pytest.mark.parametrize("N", [128, 200])   # 200: a ragged second tile of right-hand sides
def test_omp_full_tiles_with_zero_and_sparse_right_hand_sides(N):
    """Full tiles of a stored matrix (the pipelined contraction): all-zero right-hand sides and ones
    sparser than k drive the residual to zero / rounding noise, where already selected positions can
    reach the top of a tile and must still never be selected twice."""
    d, r, k = 32768, 512, 8     # 128 position tiles: enough workgroups for the pipelined kernel to be chosen
    A, At = make_matrix("stored", 20, d, r)
    A64 = At.astype(np.float64).T
    rng = np.random.default_rng(12)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    Y[0] = 0.0
    Y[77] = 0.0
    sparse_rows = {}
    for n, ks in ((1, 8), (2, 3), (64, 5), (127, 1)):
        xs, pos = synth.sparse_signal(n, d, ks)
        Y[n] = (A64 @ xs).astype(np.float32)
        sparse_rows[n] = (ks, pos)
    sel, x = run_omp(Y, A, k)
    assert all(len(set(row.tolist())) == k for row in sel) and sel.min() >= 0 and sel.max() < d
    assert sel[0].tolist() == list(range(k)) and sel[77].tolist() == list(range(k)) and not x[0].any()
    norm = orc.colnorms(At)
    for n, (ks, pos) in sparse_rows.items():
        assert sorted(sel[n][:ks].tolist()) == pos.tolist(), n
        ref = orc.omp(Y[n], At, ks, norm=norm)
        assert np.array_equal(sel[n][:ks], ref["sel"]) and relerr(x[n][:ks], ref["x"]) < TOL
        assert np.abs(x[n][ks:]).max(initial=0.0) < 1e-5 * np.abs(x[n][:ks]).max()
    for n in (3, 50, 126, N - 2, N - 1):   # ordinary noisy right-hand sides in the same launch
        ref = orc.omp(Y[n], At, k, norm=norm)
        assert np.array_equal(sel[n], ref["sel"]) and relerr(x[n], ref["x"]) < TOL


def test_omp_largest_k_sampled_picks_and_values():
    """k = 1024, the largest the entry point accepts. A full oracle run costs k^4; instead sampled
    picks are checked one by one (oracle least squares on the GPU's prefix, then the argmax of the
    normalised correlation over the unselected positions) and the values on the full support."""
    N, d, r, k = 2, 1600, 1536, 1024
    say("omp k=1024")
    A, At = make_matrix("philox", 27, d, r)
    rng = np.random.default_rng(3)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    sel, x = run_omp(Y, A, k)
    assert all(len(set(row.tolist())) == k for row in sel)
    norm = orc.colnorms(At)
    A64 = At.astype(np.float64)
    for n in range(N):
        for j in (0, 1, 63, 64, 255, 256, 700, 1023):
            res = Y[n].astype(np.float64)
            if j:
                res = res - A64[sel[n, :j]].T @ orc.lstsq_support(Y[n], At, sel[n, :j])
            score = np.abs(A64 @ res) / norm
            score[sel[n, :j]] = -1.0
            assert int(np.argmax(score)) == sel[n, j], (n, j)
        assert relerr(x[n], orc.lstsq_support(Y[n], At, sel[n])) < TOL


def test_omp_is_deterministic():
    rng = np.random.default_rng(5)
    A, At = make_matrix("philox", 4, 3000, 128)
    Y = rng.standard_normal((7, 128)).astype(np.float32)
    a = run_omp(Y, A, 16)
    b = run_omp(Y, A, 16)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))


# ------------------------------------------------------------------------------ apply
def test_apply_matches_oracle():
    rng = np.random.default_rng(6)
    C, d, k = 5, 3000, 40
    W = rng.standard_normal(C * d).astype(np.float32)
    sel_m = np.stack([rng.choice(d, k, replace=False) for _ in range(C)]).astype(np.int32)
    sel_v = sel_m.copy()
    for c in range(C):
        rng.shuffle(sel_v[c])
        sel_v[c, :5] = [(s + 1) % d if (s + 1) % d not in sel_v[c] else s for s in sel_v[c, :5]]  # some absent
    x_m = rng.standard_normal((C, k)).astype(np.float32)
    x_m[0, 3] = 0.0
    x_v = (rng.standard_normal((C, k)) ** 2).astype(np.float32)
    x_v[:, ::7] *= -1  # negative recovered second moments
    h = sgc.hyper(alpha=2.0, eps=1e-3, lr=0.01)
    Wd = dev(W)
    sgc.sgc_apply(Wd, C, d, k, dev(sel_m), dev(x_m), dev(sel_v), dev(x_v), h)
    ref = orc.apply(W, d, sel_m, x_m, sel_v, x_v, alpha=2.0, eps=1e-3, lr=0.01)
    got = Wd.cpu().numpy()
    dW, rdW = got - W, ref - W
    assert rowwise_relerr(dW.reshape(C, d), rdW.reshape(C, d)) < TOL
    assert np.array_equal(got[rdW == 0], W[rdW == 0])


# -------------------------------------------------------------------------- full step
def gpu_steps(w, At_host, A, steps, h):
    """Run `steps` consecutive steps on the GPU; return per-step host copies of everything."""
    buf = sgc.StepBuffers(w.C, w.d, w.r, w.k)
    W = dev(synth.weights(w))
    outs = []
    for t in range(1, steps + 1):
        g = synth.gradients(w, t)
        gd = dev(g.view(np.int16) if w.grad == "bf16" else g)
        sgc.step(gd, W, buf, A, t, h)
        torch.cuda.synchronize()
        C = w.C
        outs.append(dict(idx=buf.idx.cpu().numpy(), val=buf.val.cpu().numpy(), p=buf.p.cpu().numpy(), q=buf.q.cpu().numpy(),
                         m=buf.m.cpu().numpy(), v=buf.v.cpu().numpy(), mhat=buf.hat[:C].cpu().numpy(), vhat=buf.hat[C:].cpu().numpy(),
                         sel_m=buf.sel[:C].cpu().numpy(), x_m=buf.x[:C].cpu().numpy(), sel_v=buf.sel[C:].cpu().numpy(),
                         x_v=buf.x[C:].cpu().numpy(), W=W.cpu().numpy(), g=g))
    return outs


def assert_support_equal_or_near_tie(sel, y, At, norm, what):
    """Bit-exact support in selection order; a difference is accepted only as a certified near-tie:
    replaying the GPU's own prefix in the oracle, its pick scores within 1e-6 of the best score."""
    k = sel.shape[0]
    ref = orc.omp(y, At, k, norm=norm)
    if np.array_equal(sel, ref["sel"]):
        return 0
    j = int(np.argmax(sel != ref["sel"]))
    replay = orc.omp(y, At, j + 1, norm=norm, forced=sel[:j], want_top2=True)
    best = replay["top2"][j, 0]
    a = At[sel[j]].astype(np.float64)
    mine = abs(a @ replay_residual(y, At, sel[:j])) / norm[sel[j]]
    assert mine >= (1 - 1e-6) * best, "%s: pick %d is not a near-tie (%g vs %g)" % (what, j, mine, best)
    say("   near-tie accepted in", what, "at pick", j)
    return 1


def replay_residual(y, At, prefix):
    if len(prefix) == 0:
        return y.astype(np.float64)
    return orc.omp(y, At, len(prefix), forced=prefix)["res"]


def check_steps_against_oracle(w, steps, alpha=1.0):
    """Every stage is compared with the oracle run on the same inputs the GPU stage consumed
    (the GPU's previous outputs), and the whole chain is compared with the oracle's own chain."""
    A, At = make_matrix(w.matrix, w.a_seed, w.d, w.r)
    norm = orc.colnorms(At)
    h = sgc.hyper(alpha=alpha)
    outs = gpu_steps(w, At, A, steps, h)
    C = w.C
    m = np.zeros((C, w.r), np.float32)
    v = np.zeros((C, w.r), np.float32)
    W = synth.weights(w)
    cm, cv, cW = m.copy(), v.copy(), W.copy()   # the oracle's own chain
    for t, o in enumerate(outs, start=1):
        say("  step", t)
        # stage 1: Sparsify + projection, from the gradient
        ridx, rval = orc.topk(o["g"], w.k)
        assert np.array_equal(o["idx"], ridx)
        assert np.array_equal(o["val"].view(np.uint32), rval.view(np.uint32))
        rp, rq = orc.project(ridx, rval, At)
        assert rowwise_relerr(o["p"], rp) < TOL and rowwise_relerr(o["q"], rq) < TOL
        # stage 2: moments, from the GPU's p, q and previous state
        rm, rv, rmh, rvh = orc.adam(o["p"], o["q"], m, v, t)
        for name, ref in (("m", rm), ("v", rv), ("mhat", rmh), ("vhat", rvh)):
            assert rowwise_relerr(o[name], ref) < 1e-6, name
        # stage 3: recovery, from the GPU's bias-corrected moments
        Y = np.concatenate([o["mhat"], o["vhat"]])
        rsel, rx = orc.omp_batch(Y, At, w.k)
        gsel = np.concatenate([o["sel_m"], o["sel_v"]])
        gx = np.concatenate([o["x_m"], o["x_v"]])
        assert np.array_equal(gsel, rsel), "recovered support"
        assert rowwise_relerr(gx, rx) < TOL
        # stage 4: update, from the GPU's recovered vectors
        rW = orc.apply(W, w.d, o["sel_m"], o["x_m"], o["sel_v"], o["x_v"], alpha=alpha)
        assert rowwise_relerr((o["W"] - W).reshape(C, w.d), (rW - W).reshape(C, w.d)) < TOL
        assert np.array_equal(o["W"][rW == W], W[rW == W])
        # whole chain, oracle-only state: positions exact (near-ties certified), values close
        chain = orc.step(o["g"], cW, cm, cv, t, At, w.k, alpha=alpha)
        for name in ("p", "q", "m", "v", "mhat", "vhat"):
            assert rowwise_relerr(o[name], chain[name]) < TOL, name
        ties = 0
        for c in range(C):
            ties += assert_support_equal_or_near_tie(o["sel_m"][c], chain["mhat"][c], At, norm, "OMP(mhat)")
            ties += assert_support_equal_or_near_tie(o["sel_v"][c], chain["vhat"][c], At, norm, "OMP(vhat)")
        if ties == 0:
            assert rowwise_relerr(o["x_m"], chain["x_m"]) < TOL and rowwise_relerr(o["x_v"], chain["x_v"]) < TOL
            # chain-level weight update. eq. 11 divides by sqrt(z) + eps: where a position of OMP(mhat) is absent
            # from OMP(vhat) (z = 0) or z is tiny, an allowed error in x or z is amplified by up to 1/eps, so a
            # tolerance relative to the chunk maximum means nothing there. The bound therefore carries the
            # amplification: the update may differ from the oracle chain's by what the tolerances already
            # granted to x and z (TOL of the chunk maxima) can move eq. 11 at that position, and no more.
            assert_update_within_propagated_tolerance(o, chain, W, cW, w, alpha)
        m, v, W = o["m"], o["v"], o["W"]
        cm, cv, cW = chain["m"], chain["v"], chain["W"]


def assert_update_within_propagated_tolerance(o, chain, W_before_gpu, W_before_ref, w, alpha, eps=1e-8, lr=1e-3):
    """|dW_gpu - dW_ref| at every position of every chunk is at most what errors of TOL * max|x| in x and
    TOL * max|z| in z move N = alpha x / (sqrt(max(z, 0)) + eps) there (evaluated at the corners of that box
    around the oracle chain's values), plus the float rounding of the weights; untouched positions are equal."""
    C, d = w.C, w.d
    dW = (o["W"].astype(np.float64) - W_before_gpu).reshape(C, d)
    rdW = (chain["W"].astype(np.float64) - W_before_ref).reshape(C, d)
    wmax = float(np.abs(W_before_ref).max())
    checked_tight = 0
    for c in range(C):
        x = np.zeros(d)
        z = np.zeros(d)
        x[chain["sel_m"][c]] = chain["x_m"][c]
        z[chain["sel_v"][c]] = chain["x_v"][c]
        dx = TOL * np.abs(chain["x_m"][c]).max()
        dz = TOL * np.abs(chain["x_v"][c]).max()
        pos = chain["sel_m"][c]

        def upd(xx, zz):
            return alpha * xx / (np.sqrt(np.maximum(zz, 0.0)) + eps)

        ref = upd(x[pos], z[pos])
        dev_max = np.zeros(len(pos))
        for sx in (-dx, dx):
            for sz in (-dz, dz):
                dev_max = np.maximum(dev_max, np.abs(upd(x[pos] + sx, z[pos] + sz) - ref))
        bound = lr * dev_max * 1.01 + 4.0 * np.spacing(np.float32(wmax)) + 1e-6 * lr * np.abs(ref)
        err = np.abs(dW[c, pos] - rdW[c, pos])
        assert (err <= bound).all(), "chunk %d: update off by %g where %g is allowed" % (c, (err - bound).max(), bound[np.argmax(err - bound)])
        # where z is well away from zero the bound is tight: about TOL of the largest update of those positions
        good = z[pos] > 100 * dz
        if good.any():
            checked_tight += int(good.sum())
            assert err[good].max() <= 20 * TOL * np.abs(rdW[c, pos][good]).max()
        rest = np.ones(d, bool)
        rest[pos] = False
        assert not dW[c, rest].any() and not rdW[c, rest].any()
    return checked_tight


def test_full_step_cfg1_as_specified():
    say("cfg1")
    check_steps_against_oracle(synth.CFG1, 1)
    # the whole chain on this configuration, weights included (this is also what smoke() checks)
    w = synth.CFG1
    A, At = make_matrix(w.matrix, w.a_seed, w.d, w.r)
    o = gpu_steps(w, At, A, 1, sgc.hyper())[0]
    z = np.zeros((w.C, w.r), np.float32)
    W0 = synth.weights(w)
    ref = orc.step(o["g"], W0, z, z, 1, At, w.k)
    assert relerr(o["W"] - W0, ref["W"] - W0) < TOL


@pytest.mark.parametrize("w,steps", [
    (synth.shrink(synth.CFG2, C=3, d=4096, r=256, k=32), 4),      # consecutive steps, persistent moments
    (synth.shrink(synth.CFG3, C=6, d=4096, r=256, k=16), 1),      # generated matrix, row-scaled gradients
    (synth.shrink(synth.CFG4, C=7, d=2048, r=128, k=8), 2),       # layer-scaled gradients
    (synth.shrink(synth.CFG5, C=2, d=8192, r=512, k=64), 1),      # bf16 gradients
    (synth.shrink(synth.CFG5, C=2, d=32768, r=1024, k=128), 1),   # the stress shape scaled down, run in full
    # the paper's own MESGC setting for one 4096 x 4096 weight (App. D: 256 chunks, sparsity 256, kappa = 8):
    # one non-zero per chunk of 65536 and eight measurements - the smallest r and k the method is run with
    (synth.shrink(synth.CFG2, C=256, d=65536, r=8, k=1), 3),
    (synth.shrink(synth.CFG3, C=256, d=65536, r=8, k=1), 1),      # the same with a generated matrix
], ids=["cfg2s", "cfg3s", "cfg4s", "cfg5s", "cfg5_scaled_down", "paper_mesgc", "paper_mesgc_generated"])
def test_full_step_on_shrunk_workloads(w, steps):
    say(w.name, w.C, w.d, w.r, w.k)
    check_steps_against_oracle(w, steps, alpha=2.0)


def test_resume_from_copied_state_is_bitwise_identical():
    w = synth.shrink(synth.CFG2, C=2, d=4096, r=256, k=16)
    A, At = make_matrix(w.matrix, w.a_seed, w.d, w.r)
    h = sgc.hyper()
    straight = gpu_steps(w, At, A, 10, h)[-1]
    first = gpu_steps(w, At, A, 5, h)[-1]
    buf = sgc.StepBuffers(w.C, w.d, w.r, w.k)
    buf.m.copy_(dev(first["m"]))
    buf.v.copy_(dev(first["v"]))
    W = dev(first["W"])
    for t in range(6, 11):
        sgc.step(dev(synth.gradients(w, t)), W, buf, A, t, h)
    torch.cuda.synchronize()
    assert np.array_equal(W.cpu().numpy().view(np.uint32), straight["W"].view(np.uint32))
    assert np.array_equal(buf.m.cpu().numpy().view(np.uint32), straight["m"].view(np.uint32))


# ------------------------------------------------------------- streams and instrumentation
def test_large_batch_two_streams_equals_single_stream_and_profile_counts():
    """A batch of 600 right-hand sides runs its two halves on two streams; with per-kernel timing
    enabled it runs on the caller's stream alone. Both must give bitwise the same result, and the
    timing collection must count one contraction and one selection/update scope per iteration."""
    N, d, r, k = 600, 3000, 64, 6
    rng = np.random.default_rng(77)
    A, At = make_matrix("philox", 33, d, r)
    Y = rng.standard_normal((N, r)).astype(np.float32)
    a = run_omp(Y, A, k)
    sgc.sgc_profile_enable(True)
    b = run_omp(Y, A, k)
    prof = sgc.sgc_profile_read()
    sgc.sgc_profile_enable(False)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))
    assert prof["omp_corr"][1] == k and prof["omp_select_update"][1] == k
    assert prof["omp_matrix_fill"][1] == 1 and prof["omp_corr"][0] > 0.0
    c = run_omp(Y, A, k)    # and again on two streams after the collection is switched off
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[1].view(np.uint32), c[1].view(np.uint32))


def test_measurement_count_not_a_multiple_of_four_by_zero_rows():
    """r = 217 (the paper's 7 x 31): the library wants r % 4 == 0; three zero measurement rows appended to a
    stored matrix change nothing, so the padded run must match the oracle's run at r = 217."""
    C, d, r, k = 3, 2048, 217, 31
    rpad = 220
    w = synth.shrink(synth.CFG2, C=C, d=d, r=rpad, k=k)
    At = synth.gaussian_matrix(12, d, r)                       # [d, 217]
    At_pad = np.zeros((d, rpad), np.float32)
    At_pad[:, :r] = At
    A = sgc.Matrix(d, rpad, At=dev(At_pad))
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    g = synth.gradients(w, 1)
    W0 = synth.weights(w)
    W = dev(W0)
    buf = sgc.StepBuffers(C, d, rpad, k)
    sgc.step(dev(g), W, buf, A, 1, sgc.hyper(alpha=2.0))
    torch.cuda.synchronize()
    assert not buf.p[:, r:].any() and not buf.m[:, r:].any()
    # stage-wise against the oracle at r = 217
    idx, val = orc.topk(g, k)
    assert np.array_equal(buf.idx.cpu().numpy(), idx)
    p, q = orc.project(idx, val, At)
    assert rowwise_relerr(buf.p.cpu().numpy()[:, :r], p) < 1e-5
    hat = buf.hat.cpu().numpy()[:, :r]
    rsel, rx = orc.omp_batch(hat, At, k)
    assert np.array_equal(buf.sel.cpu().numpy(), rsel)
    assert rowwise_relerr(buf.x.cpu().numpy(), rx) < TOL
