"""The library under HIP graph capture: a whole step (every entry point allocates nothing and records
no memset node) is captured once and replayed with new gradients; every replay must equal the eager
step bit for bit, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2502_00311_amd import sgc, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(*a):
    print(*a, flush=True)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.mark.parametrize("shared,C,d,r,k", [
    (False, 3, 4096, 256, 24), (True, 3, 4096, 256, 24),
    (False, 2, 4096, 256, 24),     # four right-hand sides: the single-launch recovery inside the capture
    (False, 300, 1024, 64, 4),     # 600 right-hand sides: the recovery forks onto its second stream inside the capture
], ids=["two_supports", "shared_support", "single_launch", "two_streams"])
def test_captured_step_replays_equal_eager_steps(shared, C, d, r, k):
    w = synth.shrink(synth.CFG2, C=C, d=d, r=r, k=k)
    C, d, r, k = w.C, w.d, w.r, w.k
    At = synth.gaussian_matrix(5, d, r)
    A = sgc.Matrix(d, r, At=dev(At))
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    h = sgc.hyper(alpha=2.0)
    grads = [dev(synth.gradients(w, t)) for t in range(1, 5)]
    W0 = dev(synth.weights(w))

    # eager reference: four steps from zero state (the step number is a host argument: the graph is
    # captured for step 2 and replayed as step 2 on every state it is given)
    ref = []
    buf = sgc.StepBuffers(C, d, r, k)
    for g in grads:
        buf.m.zero_()
        buf.v.zero_()
        W = W0.clone()
        sgc.step(g, W, buf, A, 2, h, shared_support=shared)
        torch.cuda.synchronize()
        ref.append((W.clone(), buf.m.clone(), buf.v.clone(), buf.sel.clone(), buf.x.clone()))

    gin = torch.empty_like(grads[0])
    Wg = W0.clone()
    gbuf = sgc.StepBuffers(C, d, r, k)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                 # warm-up on the capture stream, eager
        gin.copy_(grads[0])
        sgc.step(gin, Wg, gbuf, A, 2, h, shared_support=shared)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sgc.step(gin, Wg, gbuf, A, 2, h, shared_support=shared)
    for i, g in enumerate(grads):
        say("  replay", i)
        gin.copy_(g)                              # eager work between the replays
        gbuf.m.zero_()
        gbuf.v.zero_()
        Wg.copy_(W0)
        graph.replay()
        torch.cuda.synchronize()
        W, m, v, sel, x = ref[i]
        rows = C if shared else 2 * C
        assert torch.equal(Wg, W) and torch.equal(gbuf.m, m) and torch.equal(gbuf.v, v), i
        assert torch.equal(gbuf.sel[:rows], sel[:rows]) and torch.equal(gbuf.x, x), i


def test_captured_cesgc_renewal_and_recurrence_recovery_replay_equal_eager():
    """The renewal of B (a dozen kernels per round, all on the caller's stream) and the recovery with the
    correlation recurrence, each captured once and replayed on new inputs."""
    rng = np.random.default_rng(21)
    # --- renewal of B
    rho, m, n, rounds = 6, 128, 192, 5
    Gs = [dev((rng.standard_normal((m, n)) * (0.7 ** np.arange(m))[:, None]).astype(np.float32)) for _ in range(3)]
    start = dev(rng.standard_normal((rho, m)).astype(np.float32))
    ws = torch.empty(sgc.sgc_outer_refresh_workspace_bytes(1, rho, m, n), dtype=torch.uint8, device=DEV)
    ref = []
    for G in Gs:
        B = start.clone()
        sig = torch.empty(rho, device=DEV)
        sgc.sgc_outer_refresh(B, G, 1, rho, m, n, rounds, sig, ws)
        torch.cuda.synchronize()
        ref.append((B.clone(), sig.clone()))
    Gin, Bg, sg = torch.empty_like(Gs[0]), start.clone(), torch.empty(rho, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        Gin.copy_(Gs[0])
        sgc.sgc_outer_refresh(Bg, Gin, 1, rho, m, n, rounds, sg, ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sgc.sgc_outer_refresh(Bg, Gin, 1, rho, m, n, rounds, sg, ws, stream=side)
    for i, G in enumerate(Gs):
        say("  renewal replay", i)
        Gin.copy_(G)
        Bg.copy_(start)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Bg, ref[i][0]) and torch.equal(sg, ref[i][1]), i
    # --- recovery with the recurrence for the first iterations, the contraction after
    N, d, r, k, head = 40, 2048, 64, 6, 3
    A = sgc.Matrix(d, r, At=dev(synth.gaussian_matrix(8, d, r)))
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=DEV)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    A.gram = torch.empty((d, d), dtype=torch.float64, device=DEV)
    sgc.sgc_matrix_gram(A, A.gram)
    Ys = [dev(rng.standard_normal((N, r)).astype(np.float32)) for _ in range(3)]
    ows = torch.empty(sgc.sgc_omp_recurrence_workspace_bytes(N, d, r, k, head), dtype=torch.uint8, device=DEV)
    sel, x = torch.empty((N, k), dtype=torch.int32, device=DEV), torch.empty((N, k), device=DEV)
    ref = []
    for Y in Ys:
        sgc.sgc_recover_omp_recurrence(Y, N, A, k, sel, x, ows, head=head)
        torch.cuda.synchronize()
        ref.append((sel.clone(), x.clone()))
    Yin = torch.empty_like(Ys[0])
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        Yin.copy_(Ys[0])
        sgc.sgc_recover_omp_recurrence(Yin, N, A, k, sel, x, ows, stream=side, head=head)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2, stream=side):
        sgc.sgc_recover_omp_recurrence(Yin, N, A, k, sel, x, ows, stream=side, head=head)
    for i, Y in enumerate(Ys):
        say("  recurrence replay", i)
        Yin.copy_(Y)
        sel.zero_()
        x.zero_()
        graph2.replay()
        torch.cuda.synchronize()
        assert torch.equal(sel, ref[i][0]) and torch.equal(x, ref[i][1]), i
