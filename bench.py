#!/usr/bin/env python3
"""Benchmark of the SGC per-step hot path on one MI355X.

A step = one pass of the whole path (sparsify+project, compressed Adam, batched OMP on mhat and
vhat, apply) over one batch of synthetic gradient chunks, through the C ABI of libsgc.so. The
default workload is the second configuration of the benchmark definition: 64 chunks x d=65536,
r=2048, k=256, float gradients, one stored Gaussian A, consecutive steps with persistent moments.
Inputs (A, all gradients of the run) are resident in HBM before the timed region.

Prints ONE JSON line: whole-job throughput, the roofline of the dominant kernel (the OMP
correlation contraction, float MFMA) from HIP events recorded around every launch, and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense float matrix peak
# Vector-ALU issue peak in lane-instructions per second: 256 CUs x 128 lanes per clock x 2.4 GHz, i.e. the
# published 157.3 TFLOP/s vector figure at 2 flop per FMA. The register-only probe of plain (non-packed)
# v_fma_f32 (sgc_probe, reported under micro.probes in every default run) sustains 66 T/s on this machine,
# 108 lanes per CU and nominal clock, so the figure is reachable without packed instructions.
VALU_PEAK_TLANE = 78.6
PROJECT_INSTR_PER_QUAD = 200.0  # vector instructions per four generated entries of A in project_kernel (50 per normal)
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, keyed by
# workload name: (bytes, the summary under profiles/ that holds the run). Stored figures: they describe the
# kernel as it was when that profile was taken.
MEASURED_TRAFFIC = {"cfg4_llama7b_block": (4.360e9, "profiles/cfg4_kernel_trace_and_hbm_traffic.md: bytes leaving the L2s, served by the "
                                                  "memory-side cache where the 64 MiB matrix stays; algorithmic 2.44e8"),
                    "cfg5_stress_bf16": (6.22e8, "profiles/cfg5_kernel_trace_stats.md: the residuals re-read by 2048 workgroups; the 8 GiB "
                                                  "matrix is generated in the kernel and never read; algorithmic 2.6e7"),
                    "cfg2_64x65536": (5.528e8, "profiles/cfg2_corr_kernel_hbm_traffic.md"),
                    "cesgc_16x4096x4096_rank32": (1.390e8, "profiles/cesgc_16x4096x4096_kernel_trace_stats.md")}  # per matrix


def host_gradients(w, step, workers):
    """One step's gradient chunks, drawn on the host by `workers` threads (every chunk has its own seed, so the
    result does not depend on the split)."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from paper_2502_00311_amd import synth

    if w.C < 4 * workers:
        return synth.gradients(w, step)
    edges = np.linspace(0, w.C, 4 * workers + 1).astype(int)
    with ThreadPoolExecutor(workers) as ex:
        parts = list(ex.map(lambda i: synth.gradients(w, step, chunks=range(edges[i], edges[i + 1])), range(4 * workers)))
    return np.concatenate(parts, axis=0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", type=int, default=4,
                    help="configuration index 1..5 (default 4: the linear weights of one Llama-2-7B block, the largest "
                         "configuration, 202 M gradient elements); 6 = the paper's own MESGC setting (r = 8, k = 1) on "
                         "configuration 4's block")
    ap.add_argument("--chunks", type=int, default=0, help="override the number of chunks (0 = as defined)")
    ap.add_argument("--distinct-steps", type=int, default=0,
                    help="gradient draws kept resident and cycled through the steps (0 = one per step up to 4 GB of "
                         "gradients, i.e. 4 draws for configuration 4)")
    ap.add_argument("--event-steps", type=int, default=3,
                    help="steps of the second pass that records HIP events around every kernel launch (the roofline's "
                         "launch durations come from there)")
    ap.add_argument("--events-only", action="store_true",
                    help="profiling aid: every step of the run (warm-up included) is taken with HIP events around each "
                         "launch, which also keeps the recovery on one stream with whole-batch launches, so that a "
                         "rocprofv3 kernel trace of this command holds launches of one size per kernel; the timed pass, "
                         "variants, micro-runs and the CPU baseline are skipped")
    ap.add_argument("--probes-only", action="store_true", help="only the machine probes (sgc_probe), as one JSON line")
    ap.add_argument("--shared-support", action="store_true",
                    help="recover one support per chunk from mhat and fit vhat on it (sgc_recover_omp_shared) "
                         "instead of the two independent recoveries of Alg. 2")
    ap.add_argument("--materialize", action="store_true",
                    help="a generated matrix is written out once with sgc_matrix_fill (outside the timed region) "
                         "and handed over as a stored one: what a caller with HBM to spare would do")
    ap.add_argument("--whole-matrix", action="store_true",
                    help="a generated matrix of more than 64 MiB is written out once per call into the recovery's "
                         "workspace (SGC_MATRIX_FLAG_MATERIALIZE; needs d <= N k) instead of being regenerated inside "
                         "the contraction")
    ap.add_argument("--gram", action="store_true",
                    help="build the optional table of column inner products (sgc_matrix_gram, 8 d^2 bytes, once, "
                         "outside the timed region) and let the recovery use it")
    ap.add_argument("--recurrence", action="store_true",
                    help="recover with the correlation recurrence of App. B (sgc_recover_omp_recurrence; builds the "
                         "Gram table like --gram and needs N (k + 1) d more floats of workspace): a variant")
    ap.add_argument("--recurrence-head", type=int, default=0,
                    help="with --recurrence: the recurrence serves only the first H iterations, the contraction "
                         "the rest (0 = all k iterations, -1 = r/64, about where the two cost the same)")
    ap.add_argument("--screen-bf16", action="store_true",
                    help="screen the correlation contraction on the bfloat16 matrix cores (split operands, three "
                         "products); candidates are re-scored in double either way")
    ap.add_argument("--cesgc", action="store_true",
                    help="time the CESGC step (Sec. 4.4) instead: --cesgc-matrices weight matrices of 4096 x 4096 "
                         "(LLaMA-7B attention projections), rank 32, chunks of 2048, k = 31, r = 220")
    ap.add_argument("--cesgc-matrices", type=int, default=16)
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the extra runs reported next to the headline: the shared-support variant, the micro-runs "
                         "and the labelled secondary entry on configuration 2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (reference for the rocprofv3 FETCH_SIZE / "
                         "WRITE_SIZE counters)")
    ap.add_argument("--corr-depth-sweep", action="store_true",
                    help="instead of a step: the correlation contraction alone (24704 right-hand sides, d = 16384, the "
                         "shape of workload 4) at depths r = 128 .. 2048, with --screen-bf16 its bfloat16 form; the "
                         "slope is the time per stage of 32 depths, the intercept the fixed cost per launch")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (chunks are independent and would shard by "
              "chunk range, but no multi-GPU path is built); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2502_00311_amd import sgc, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sgc.lib()  # fails loudly if the HIP library is not built
    dev = "cuda:0"
    if args.probes_only:
        print(json.dumps({"probes": probe_runs(dev)}))
        return 0
    if args.events_only:
        args.no_variants = args.no_cpu_baseline = True
    if args.cesgc:
        return main_cesgc(args, dev)
    if args.corr_depth_sweep:
        return main_depth_sweep(args, dev)
    w = synth.CONFIGS[args.workload]
    if args.chunks:
        w = synth.shrink(w, C=args.chunks)
    if args.recurrence:
        if args.shared_support:
            print("bench.py: --recurrence goes with the two-support recovery", file=sys.stderr)
            return 2
        args.gram = True
    out = run_workload(args, w, dev, args.steps, args.warmup, variants=not args.no_variants,
                       baseline=not args.no_cpu_baseline)
    if not args.no_variants:
        # labelled micro-runs of the HBM-bound kernels at a size where launch latency does not hide them
        out["micro"] = micro_runs(dev)
        plain = not (args.shared_support or args.screen_bf16 or args.gram or args.recurrence or args.materialize or args.chunks or args.whole_matrix)
        if plain and args.workload != 2:
            # secondary entry: configuration 2 (64 chunks of 65536, r 2048, k 256, stored matrix streamed from HBM
            # in every iteration), a few steps, same code path
            torch.cuda.empty_cache()
            sec = run_workload(args, synth.CFG2, dev, min(args.steps, 5), 1, variants=False, baseline=False)
            out["secondary"] = {key: sec[key] for key in ("value", "unit", "steps", "warmup", "ms_per_step", "config", "roofline", "kernels")}
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(out))
    return 0


def run_workload(args, w, dev, K, Wm, variants, baseline):
    """Time K steps of workload w after Wm warm-up steps; returns the dictionary of the JSON line."""
    import numpy as np
    import torch
    from paper_2502_00311_amd import sgc, synth

    C, d, r, k = w.C, w.d, w.r, w.k
    workers = min(16, os.cpu_count() or 1)

    # ---- inputs, resident before timing ----
    At_host = None
    if w.matrix == "stored":
        At_host = synth.gaussian_matrix(w.a_seed, d, r)
        A = sgc.Matrix(d, r, At=torch.from_numpy(At_host).to(dev))
    elif args.materialize:
        At_dev = torch.empty((d, r), dtype=torch.float32, device=dev)
        sgc.sgc_matrix_fill(w.a_seed, r, 0, d, At_dev)
        A = sgc.Matrix(d, r, At=At_dev)
    else:
        A = sgc.Matrix(d, r, At=None, seed=w.a_seed)
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=dev)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    if args.screen_bf16:
        A.flags = sgc.MATRIX_FLAG_SCREEN_BF16
    if args.whole_matrix:
        A.flags |= sgc.MATRIX_FLAG_MATERIALIZE
    gram_ms = None
    head = args.recurrence_head
    if args.recurrence and head < 0:
        head = max(1, min(k, r // 64))
    if args.gram:
        A.gram = torch.empty((d, d), dtype=torch.float64, device=dev)
        torch.cuda.synchronize()
        tg = time.perf_counter()
        sgc.sgc_matrix_gram(A, A.gram)
        torch.cuda.synchronize()
        gram_ms = (time.perf_counter() - tg) * 1e3
    nsteps = max(K, Wm, 1)
    step_bytes = (2.0 if w.grad == "bf16" else 4.0) * C * d
    ndraw = args.distinct_steps or max(1, min(nsteps, int(4.0e9 // step_bytes)))
    ndraw = min(ndraw, nsteps)
    grads = []
    for t in range(1, ndraw + 1):
        g = host_gradients(w, t, workers)
        grads.append(torch.from_numpy(g.view(np.int16) if w.grad == "bf16" else g).to(dev))
        del g
    W0 = torch.from_numpy(synth.weights(w)).to(dev)
    Wt = W0.clone()
    buf = sgc.StepBuffers(C, d, r, k, device=dev, recurrence=(head or True) if args.recurrence else False,
                          screen=args.screen_bf16)
    h = sgc.hyper()

    def reset():
        buf.m.zero_()
        buf.v.zero_()
        Wt.copy_(W0)

    def run(n, shared=None):
        for t in range(1, n + 1):
            sgc.step(grads[(t - 1) % ndraw], Wt, buf, A, t, h, shared_support=args.shared_support if shared is None else shared)

    if args.events_only:
        sgc.sgc_profile_enable(True)
    run(Wm)
    torch.cuda.synchronize()
    reset()
    torch.cuda.synchronize()
    if not args.events_only:
        t0 = time.perf_counter()
        run(K)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / K

    # ---- a second pass with HIP events around every kernel launch (on the stream the kernels run on) ----
    Ke = K if args.events_only else max(1, min(K, args.event_steps))
    reset()
    torch.cuda.synchronize()
    sgc.sgc_profile_enable(True)
    t2 = time.perf_counter()
    run(Ke)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    prof = sgc.sgc_profile_read()
    sgc.sgc_profile_enable(False)
    if args.events_only:
        ms_per_step = (t3 - t2) * 1e3 / Ke
    value = C * d / (ms_per_step * 1e-3)
    corr_ms, corr_n = prof["omp_corr"]
    fill_ms, _ = prof["omp_matrix_fill"]
    # one launch covers all d positions (stored / in-kernel generated A) or one panel of them
    launches_per_iter = corr_n / (Ke * k)
    nrhs = C if args.shared_support else 2 * C
    flops_per_launch = 2.0 * d * r * nrhs / launches_per_iter
    avg_ms = corr_ms / max(corr_n, 1)
    achieved = flops_per_launch / (avg_ms * 1e-3) / 1e12
    peak = MFMA_F32_PEAK_TFLOPS
    kernel_name = "omp correlation contraction At*R (float 32x32x2 MFMA, fused argmax epilogue)"
    if args.screen_bf16:  # three bfloat16 products per float product, priced against the bfloat16 peak
        achieved *= 3.0
        peak = 2500.0
        kernel_name = "omp correlation contraction At*R (3 x bf16 32x32x16 MFMA on split operands, fused argmax epilogue)"
    traffic = None if (args.shared_support or args.screen_bf16 or args.chunks) else MEASURED_TRAFFIC.get(w.name)
    roofline = {
        "bound": "mfma", "kernel": kernel_name,
        "achieved": round(achieved, 3), "peak": peak, "unit": "TFLOP/s",
        "frac": round(achieved / peak, 4),
        "traffic": traffic[0] if traffic else None,
        "traffic_source": (traffic[1] + " (rocprofv3 --pmc runs of this command; a stored figure, not read in this run)") if traffic else None,
        "flops_per_launch": flops_per_launch, "avg_launch_ms": round(avg_ms, 5), "launches": corr_n,
        "event_steps": Ke,
    }
    if r <= 16 and 2 * C >= 128 and not args.recurrence:
        # very few measurements: the contraction runs on the vector ALUs (corr_narrow_kernel: r FMAs and about
        # 7 further instructions per score), and the top-k scan is the larger kernel of the step
        ops = float(d) * nrhs * (r + 7) * k
        rate = ops / (corr_ms / Ke * 1e-3)
        roofline = {"bound": "alu", "kernel": "omp correlation on the vector ALUs (r <= 16), lane-instructions per second",
                    "achieved": round(rate / 1e12, 3), "peak": VALU_PEAK_TLANE, "unit": "T lane-instr/s",
                    "frac": round(rate / (VALU_PEAK_TLANE * 1e12), 4), "traffic": None, "avg_launch_ms": round(avg_ms, 5), "launches": corr_n}
        tk_ms, tk_n = prof["topk"]
        if tk_n and tk_ms > corr_ms:
            gbps = ((2.0 if w.grad == "bf16" else 4.0) * C * d + 8.0 * C * k) / (tk_ms / tk_n * 1e-3) / 1e9
            roofline = {"bound": "hbm", "kernel": "top-k scan of the gradients (the dominant kernel at this shape)",
                        "achieved": round(gbps, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(gbps / 8000.0, 4),
                        "traffic": None, "avg_launch_ms": round(tk_ms / tk_n, 5), "launches": tk_n,
                        "omp_corr_alu_frac": round(rate / (VALU_PEAK_TLANE * 1e12), 4)}
    if args.recurrence:
        # no contraction inside the iterations: the class holds p0 = A^H y (once per call) and the k - 1 updates
        # of p, which stream the image vectors b_t (4 d j bytes at iteration j), a row of the table (8 d), the
        # new b (4 d written) and p (8 d) per right-hand side
        hd = head or k
        total = float(nrhs) * d * sum(4.0 * j + 20.0 for j in range(1, hd)) + 8.0 * nrhs * d
        if hd == k:
            gbps = total / (corr_ms / Ke * 1e-3) / 1e9
            roofline = {"bound": "hbm", "kernel": "correlation recurrence p <- p - b a (App. B), all its launches of a step",
                        "achieved": round(gbps, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(gbps / 8000.0, 4),
                        "traffic": None, "bytes_per_step": total, "ms_per_step": round(corr_ms / Ke, 3), "launches": corr_n}
        else:
            # both engines inside one class of launches: the contraction's flop over the whole class's time is a
            # lower bound of its rate
            flops = 2.0 * d * r * nrhs * (k - hd)
            tf = flops / (corr_ms / Ke * 1e-3) / 1e12
            roofline = {"bound": "mfma", "kernel": "recurrence for %d iterations, then the float contraction; rate = the "
                        "contraction's flop over the time of both" % hd,
                        "achieved": round(tf, 3), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tf / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None,
                        "recurrence_bytes_per_step": total, "ms_per_step": round(corr_ms / Ke, 3), "launches": corr_n}
    if fill_ms > 0 and roofline.get("bound") == "mfma":  # generated A produced by a separate fill kernel: the rate including that time
        if not args.recurrence:
            roofline["achieved_incl_matrix_fill"] = round(flops_per_launch * corr_n / ((corr_ms + fill_ms) * 1e-3) / 1e12, 3)
    kernels = {n: {"ms_per_step": round(ms / Ke, 4), "launches_per_step": cnt / Ke} for n, (ms, cnt) in prof.items()}
    # HBM-bound companions (algorithmic bytes / event time)
    bytes_adam = 32.0 * C * r
    bytes_topk = (2.0 if w.grad == "bf16" else 4.0) * C * d + 8.0 * C * k
    companions = [("adam", bytes_adam), ("topk", bytes_topk)]
    if w.matrix == "stored" or args.materialize:  # the gather of k rows of At per chunk, and p, q written
        companions.append(("project", 4.0 * C * k * r + 8.0 * C * k + 8.0 * C * r))
    for name, nbytes in companions:
        ms, cnt = prof[name]
        if cnt:
            kernels[name]["algorithmic_GBps"] = round(nbytes / (ms / cnt * 1e-3) / 1e9, 2)
            kernels[name]["frac_of_8TBps"] = round(nbytes / (ms / cnt * 1e-3) / 8e12, 3)
    if w.matrix != "stored" and not args.materialize and prof["project"][1]:
        # generated matrix: the projection is bound by the generator's vector arithmetic, PROJECT_INSTR_PER_QUAD
        # lane-instructions per four entries of A
        ms, cnt = prof["project"]
        rate = float(C) * k * (r / 4) * PROJECT_INSTR_PER_QUAD / (ms / cnt * 1e-3)
        kernels["project"]["T_lane_instr_per_s"] = round(rate / 1e12, 2)
        kernels["project"]["frac_of_valu_peak"] = round(rate / (VALU_PEAK_TLANE * 1e12), 3)
    # the least-squares update and residual against one read of the selected columns per iteration
    # (N r j 4 bytes at iteration j) plus one pass over the factor F (N j^2 / 2 doubles)
    su_ms, su_n = prof["omp_select_update"]
    if su_n:
        ls_bytes = sum(4.0 * nrhs * r * j + 4.0 * nrhs * j * j for j in range(1, k + 1))
        kernels["omp_select_update"]["algorithmic_GBps"] = round(ls_bytes / (su_ms / Ke * 1e-3) / 1e9, 1)
        kernels["omp_select_update"]["frac_of_8TBps"] = round(ls_bytes / (su_ms / Ke * 1e-3) / 8e12, 3)
        # what this formulation moves: the selected columns twice per iteration (inner products with the new
        # column, then the residual, which needs the solution those inner products lead to) plus the factor
        two = sum(8.0 * nrhs * r * j + 4.0 * nrhs * j * j for j in range(1, k + 1))
        kernels["omp_select_update"]["two_pass_GBps"] = round(two / (su_ms / Ke * 1e-3) / 1e9, 1)

    # how far the two supports of a chunk are apart after the last step (the paper treats them as identical, which holds
    # only in the exact-recovery regime): mean over the chunks of |support(mhat) symmetric-difference support(vhat)|
    supports = None
    if not args.shared_support:
        both = torch.cat([buf.sel[:C], buf.sel[C:2 * C]], dim=1).sort(dim=1).values
        common = (both[:, 1:] == both[:, :-1]).sum(dim=1).double()
        supports = {"k": k, "mean_symmetric_difference": round(float((2.0 * (k - common)).mean().item()), 3),
                    "after_steps": Ke}

    out = {
        "metric": "gradient elements/s per full SGC step (1 GPU)", "value": round(value, 1), "unit": "elements/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "chunks": C, "d": d, "r": r, "k": k, "grad": w.grad,
                   "matrix": "philox, materialised by the caller" if (args.materialize and w.matrix != "stored") else
                             ("philox, written out once per call into the workspace" if args.whole_matrix else w.matrix),
                   "rhs_per_omp_call": nrhs,
                   "gradient_draws": "%d distinct steps resident in HBM, cycled over the %d steps; moments persist" % (ndraw, K),
                   "recovery": "shared_support" if args.shared_support else "two_supports",
                   "gram_table": bool(args.gram),
                   "contraction": ("none inside the iterations (correlation recurrence)" if not head
                                   else "correlation recurrence for %d iterations, then float" % head) if args.recurrence
                   else ("bf16 split (3 products), float accumulate" if args.screen_bf16 else "float")},
        "roofline": roofline,
        "ms_per_step_with_events": round((t3 - t2) * 1e3 / Ke, 3),
        "timing": "events pass only (one stream, HIP events around every launch)" if args.events_only else "eager steps, no events",
        "gram_build_ms": None if gram_ms is None else round(gram_ms, 2),
        "supports": supports,
        "kernels": kernels,
    }

    # ---- variants, a few steps each (context, not the headline): the shared-support recovery (first
    #      widening), the Gram table where it is at most 2 GiB, and for a generated matrix of more than 64 MiB the option that writes it out once per
    #      call into the workspace instead of regenerating it inside the contraction ----
    if variants and not (args.shared_support or args.screen_bf16 or args.gram or args.recurrence or args.whole_matrix):
        nv = 1 if ms_per_step > 2000 else min(3, nsteps)

        def timed(shared):
            reset()
            if ms_per_step <= 2000:
                run(1, shared)
                reset()
            torch.cuda.synchronize()
            tv = time.perf_counter()
            run(nv, shared)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - tv) * 1e3 / nv
            return {"ms_per_step": round(ms, 3), "value": round(C * d / (ms * 1e-3), 1), "steps": nv}

        out["variants"] = {"shared_support": timed(True)}
        if d <= 16384:
            # App. B's precomputed table of column inner products (built once per matrix, 8 d^2 bytes): the
            # update's inner products become look-ups; the contraction stays
            A.gram = torch.empty((d, d), dtype=torch.float64, device=dev)
            torch.cuda.synchronize()
            tg = time.perf_counter()
            sgc.sgc_matrix_gram(A, A.gram)
            torch.cuda.synchronize()
            build_ms = (time.perf_counter() - tg) * 1e3
            out["variants"]["gram_table"] = dict(timed(False), table_build_ms=round(build_ms, 3), table_bytes=8 * d * d)
            A.gram = None
        if A.mode == sgc.MATRIX_PHILOX and 4.0 * d * r > 64 * 2 ** 20 and d <= 2 * C * k:
            A.flags = sgc.MATRIX_FLAG_MATERIALIZE
            out["variants"]["whole_matrix_in_workspace"] = timed(False)
            A.flags = 0

    del grads, buf, Wt, W0
    A.gram = None
    torch.cuda.empty_cache()
    if baseline:
        out["cpu_baseline"] = cpu_baseline(w, At_host, args.shared_support)
    return out


def probe_runs(dev):
    """What this machine delivers for the resources the kernels are bound by (sgc_probe; best of 5 launches):
    plain v_fma_f32 issue rate, float MFMA rate, streaming read, the Adam kernel's 4-read / 4-write pattern,
    and a plain copy."""
    import torch
    from paper_2502_00311_amd import sgc

    res = {}
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    nbytes = 2 << 30
    src = torch.empty(nbytes // 2, dtype=torch.uint8, device=dev)
    dst = torch.empty(nbytes // 2, dtype=torch.uint8, device=dev)
    src.fill_(1)

    def best(kind, blocks, iters, nb, rd=src):
        sgc.sgc_probe(kind, rd, dst, nb, blocks, iters)
        t = 1e30
        for _ in range(5):
            a.record()
            sgc.sgc_probe(kind, rd, dst, nb, blocks, iters)
            b.record()
            torch.cuda.synchronize()
            t = min(t, a.elapsed_time(b))
        return t

    iters, blocks = 5000, 8192          # 32 workgroups per CU: the rate no longer grows with the grid
    ms = best(sgc.PROBE_VALU, blocks, iters, 0)
    res["valu_fma_T_lane_instr_per_s"] = round(blocks * 256.0 * iters * 64 / (ms * 1e-3) / 1e12, 2)
    ms = best(sgc.PROBE_MFMA, 1024, iters, 0)
    res["mfma_f32_TFLOPs"] = round(1024 * 4.0 * iters * 16 * 4096 / (ms * 1e-3) / 1e12, 1)
    # 16 MFMAs + 64 v_fma per iteration against the two alone: if vector-ALU work rode in the shadow of the float
    # MFMAs the mix would take the MFMA time; on this chip it takes the sum
    t_m = ms
    t_v = best(sgc.PROBE_VALU, 1024, iters, 0)
    t_mix = best(sgc.PROBE_MFMA_VALU4, 1024, iters, 0)
    res["mfma_plus_valu_ms"] = {"mfma_alone": round(t_m, 3), "valu_alone": round(t_v, 3), "both_in_one_loop": round(t_mix, 3)}
    # the same question for wavefronts that share a SIMD: four wavefronts of MFMAs and four of FMAs per workgroup
    res["mfma_beside_valu_ms"] = {"mfma_wavefronts_alone": round(best(sgc.PROBE_SPLIT_MFMA, 1024, iters, 0), 3),
                                  "valu_wavefronts_alone": round(best(sgc.PROBE_SPLIT_VALU, 1024, iters, 0), 3),
                                  "both": round(best(sgc.PROBE_SPLIT_BOTH, 1024, iters, 0), 3)}
    ms = best(sgc.PROBE_READ, 4096, 0, nbytes // 2)
    res["read_GBps"] = round(nbytes / 2 / (ms * 1e-3) / 1e9, 1)
    ms = best(sgc.PROBE_RW44, 4096, 0, nbytes)
    res["rw_4read_4write_GBps"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    ms = best(sgc.PROBE_COPY, 4096, 0, nbytes)
    res["copy_GBps"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    del src, dst
    return res


def micro_runs(dev):
    """Top-k (+ projection with a generated matrix) on configuration 4's shape and the Adam update on
    64 M state elements: algorithmic bytes / HIP-event time per launch. Inputs: normal deviates drawn on
    the device (only the memory traffic matters here). Plus the machine probes."""
    import torch
    from paper_2502_00311_amd import sgc

    res = {"probes": probe_runs(dev)}
    reps = 10
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    # Adam: p, q, m, v read; m, v, mhat, vhat written = 32 B per element
    n = 64 << 20
    p, q = torch.randn(n, device=dev), torch.rand(n, device=dev)
    m, v = torch.zeros(n, device=dev), torch.zeros(n, device=dev)
    mh, vh = torch.empty(n, device=dev), torch.empty(n, device=dev)
    h = sgc.hyper()
    for _ in range(2):
        sgc.sgc_adam_compressed(p, q, m, v, mh, vh, n, 3, h)
    a.record()
    for _ in range(reps):
        sgc.sgc_adam_compressed(p, q, m, v, mh, vh, n, 3, h)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / reps
    gbps = 32.0 * n / (ms * 1e-3) / 1e9
    res["adam_64M_elements"] = {"ms": round(ms, 4), "algorithmic_GBps": round(gbps, 1),
                                "frac_of_8TBps": round(gbps / 8e3, 3),
                                "ceiling_probe_GBps": res["probes"]["rw_4read_4write_GBps"],
                                "frac_of_ceiling_probe": round(gbps / res["probes"]["rw_4read_4write_GBps"], 3)}
    del p, q, m, v, mh, vh
    return res


def main_depth_sweep(args, dev):
    """The contraction of the recovery alone at several depths (a labelled micro-measurement, not a step)."""
    import torch
    from paper_2502_00311_amd import sgc

    N, d, k = 24704, 16384, 4
    rows = []
    for r in (128, 256, 512, 1024, 2048):
        A = sgc.Matrix(d, r, At=None, seed=5)
        A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=dev)
        sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
        A.flags = sgc.MATRIX_FLAG_SCREEN_BF16 if args.screen_bf16 else 0
        Y = torch.randn((N, r), device=dev)
        sel = torch.empty((N, k), dtype=torch.int32, device=dev)
        x = torch.empty((N, k), device=dev)
        ws = torch.empty(sgc.sgc_omp_workspace_bytes(N, d, r, k), dtype=torch.uint8, device=dev)
        sgc.sgc_recover_omp(Y, N, A, k, sel, x, ws)                 # warm-up
        torch.cuda.synchronize()
        sgc.sgc_profile_enable(True)
        sgc.sgc_recover_omp(Y, N, A, k, sel, x, ws)
        torch.cuda.synchronize()
        ms, launches = sgc.sgc_profile_read()["omp_corr"]
        sgc.sgc_profile_enable(False)
        rows.append({"r": r, "stages": r // 32, "us_per_launch": round(ms / launches * 1e3, 1)})
        del ws, Y
    a, b = rows[-2], rows[-1]
    slope = (b["us_per_launch"] - a["us_per_launch"]) / (b["stages"] - a["stages"])
    print(json.dumps({"micro": "corr_depth_sweep", "rhs": N, "d": d, "contraction": "bf16 split" if args.screen_bf16 else "float",
                      "launches": rows, "us_per_stage": round(slope, 2),
                      "fixed_us": round(b["us_per_launch"] - slope * b["stages"], 1)}))
    return 0


def main_cesgc(args, dev):
    """CESGC (Sec. 4.4) on a batch of equal weight matrices that share the measurement matrix A: one
    batched outer projection into a common buffer of compressed gradients, ONE pass of Alg. 2 over all
    their chunks, one batched back-projection. B (rank 32, one per matrix) is an input, resident like A."""
    import numpy as np
    import torch
    from paper_2502_00311_amd import sgc, synth

    m = n = 4096
    rho, d, r, k = 32, 2048, 220, 31      # Table of App. D: rank 32, 64 chunks per matrix, s_c = 31, kappa = 7
    M = args.cesgc_matrices
    K, Wm = args.steps, args.warmup
    Cm = rho * n // d                     # chunks per matrix
    C = M * Cm
    At_host = synth.gaussian_matrix(1, d, r)
    A = sgc.Matrix(d, r, At=torch.from_numpy(At_host).to(dev))
    A.inv_colnorm = torch.empty(d, dtype=torch.float32, device=dev)
    sgc.sgc_matrix_colnorms(A, A.inv_colnorm)
    bases = [synth.orthonormal_rows(100 + j, 2 * rho, m) for j in range(M)]
    B_host = [np.ascontiguousarray(b[:rho]) for b in bases]
    Bs = torch.from_numpy(np.stack(B_host)).to(dev)                 # [M][rho][m]
    nsteps = max(K, Wm, 1)
    # a fresh gradient per matrix and step; the matrices of a step lie one after the other
    G = []
    for t in range(1, nsteps + 1):
        Gt = torch.empty((M, m, n), dtype=torch.float32, device=dev)
        for j in range(M):
            Gt[j].copy_(torch.from_numpy(synth.matrix_gradient(100 + j, t, m, n, bases[j])))
        G.append(Gt)
    rng = np.random.default_rng(7)
    W0 = torch.empty((M, m, n), dtype=torch.float32, device=dev)
    for j in range(M):
        W0[j].copy_(torch.from_numpy((0.02 * rng.standard_normal((m, n))).astype(np.float32)))
    Wt = W0.clone()
    buf = sgc.StepBuffers(C, d, r, k, device=dev)
    ob = sgc.OuterBuffers(rho, m, n, count=M, device=dev)
    h = sgc.hyper(alpha=2.0, lr=2e-5)

    def reset():
        buf.m.zero_()
        buf.v.zero_()
        Wt.copy_(W0)

    def run(nrun):
        for t in range(1, nrun + 1):
            sgc.step_cesgc(G[t - 1], Wt, Bs, ob, buf, A, t, h)

    run(Wm)
    torch.cuda.synchronize()
    reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K
    reset()
    torch.cuda.synchronize()
    sgc.sgc_profile_enable(True)
    run(K)
    torch.cuda.synchronize()
    prof = sgc.sgc_profile_read()
    sgc.sgc_profile_enable(False)
    kernels = {nm: {"ms_per_step": round(ms / K, 4), "launches_per_step": cnt / K} for nm, (ms, cnt) in prof.items()}
    # the two streaming kernels: algorithmic bytes per matrix / event time per matrix
    bytes_proj = 4.0 * m * n + 4.0 * rho * n + 4.0 * rho * m
    bytes_back = 8.0 * m * n + 4.0 * rho * n + 4.0 * rho * m
    proj_ms = prof["outer_project"][0] / (K * M)   # per matrix
    back_ms = prof["outer_apply"][0] / (K * M)
    kernels["outer_project"]["algorithmic_GBps"] = round(bytes_proj / (proj_ms * 1e-3) / 1e9, 1)
    kernels["outer_apply"]["algorithmic_GBps"] = round(bytes_back / (back_ms * 1e-3) / 1e9, 1)
    achieved = bytes_back / (back_ms * 1e-3) / 1e9
    corr_ms, corr_n = prof["omp_corr"]
    if corr_n:  # one launch per iteration here (HIP events keep the recovery on one stream)
        kernels["omp_corr"]["TFLOPs"] = round(2.0 * d * r * 2 * C / (corr_ms / corr_n * 1e-3) / 1e12, 1)
    out = {
        "metric": "gradient elements/s per full CESGC step (1 GPU)", "value": round(M * m * n / (ms_per_step * 1e-3), 1),
        "unit": "elements/s", "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cesgc_%dx4096x4096_rank32" % M, "matrices": M, "m": m, "n": n, "rank": rho,
                   "chunks": C, "d": d, "r": r, "k": k, "matrix": "stored", "rhs_per_omp_call": 2 * C},
        "roofline": {"bound": "hbm", "kernel": "CESGC back-projection W -= lr B^T N (zero fill + read-modify-write of W), per matrix of the batch",
                     "achieved": round(achieved, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(achieved / 8000.0, 4),
                     "traffic": (MEASURED_TRAFFIC.get("cesgc_%dx4096x4096_rank32" % M) or (None,))[0], "bytes_per_matrix": bytes_back, "avg_ms_per_matrix": round(back_ms, 5)},
        "kernels": kernels,
    }
    # the renewal of B (outside the step: the paper does it every fixed number of steps): all matrices in one
    # call, started from the B in use, a few rounds of the iteration plus the Rayleigh-Ritz step
    rounds = 4
    Bn = Bs.clone()
    sig = torch.empty((M, rho), dtype=torch.float32, device=dev)
    rws = torch.empty(sgc.sgc_outer_refresh_workspace_bytes(M, rho, m, n), dtype=torch.uint8, device=dev)
    sgc.sgc_outer_refresh(Bn, G[0], M, rho, m, n, rounds, sig, rws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        sgc.sgc_outer_refresh(Bn, G[0], M, rho, m, n, rounds, sig, rws)
    torch.cuda.synchronize()
    refresh_ms = (time.perf_counter() - t0) * 1e3 / 3
    sgc.sgc_profile_enable(True)
    sgc.sgc_outer_refresh(Bn, G[0], M, rho, m, n, rounds, sig, rws)
    torch.cuda.synchronize()
    rprof = sgc.sgc_profile_read()
    sgc.sgc_profile_enable(False)
    out["refresh"] = {"rounds": rounds, "matrices": M, "ms_per_call": round(refresh_ms, 3),
                      "ms_per_matrix": round(refresh_ms / M, 4),
                      "passes_over_G_ms": round(rprof["outer_project"][0], 3), "passes": int(rprof["outer_project"][1]),
                      "factor_and_transform_ms": round(rprof["outer_refresh"][0], 3),
                      "note": "not part of the timed step"}
    del rws
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        z = np.zeros((Cm, r), np.float32)
        G1 = G[0][0].cpu().numpy()
        Wc = W0[0].cpu().numpy()
        tc = time.perf_counter()
        orc.step_cesgc(G1, Wc, B_host[0], z, z, 1, At_host, d, k, alpha=2.0, lr=2e-5)
        tc = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": round(m * n / tc, 1), "unit": "elements/s", "cores": 1, "kind": "oracle",
                               "sample": "matrix 0 of step 1 (1 of %d matrices), the whole CESGC step; %.1f s" % (M, tc),
                               "host_cores": os.cpu_count()}
    print(json.dumps(out))
    return 0


def cpu_baseline(w, At_host, shared_support=False, budget_s=30.0):
    """The CPU oracle (single thread, as it stands) on a bounded sample of step 1 of the same workload: whole
    chunks spread evenly over the batch (for configuration 4 that is over its seven weight matrices), each run
    through the whole path - top-k, projection, Adam, OMP(mhat), OMP(vhat), apply - until about budget_s seconds
    of CPU work are spent. A configuration whose single recovery would take minutes is timed on its first
    iterations (every iteration scans all d columns, which dominates) and scaled to k."""
    import numpy as np
    from oracle import oracle as orc
    from paper_2502_00311_amd import synth

    if At_host is None:
        At_host = orc.philox_matrix(w.a_seed, w.d, w.r)
    norm = orc.colnorms(At_host)
    per_iter = 2.0 * w.d * w.r / 2.0e9          # seconds per iteration at ~2 Gflop/s, to plan the sample
    full = per_iter * w.k * 2 <= budget_s
    iters = w.k if full else max(4, int(budget_s / 2 / per_iter))
    iters = min(iters, w.k)
    want = max(1, min(w.C, 16, int(budget_s / max(per_iter * iters * 2, 1e-3))))
    chunks = sorted(set(int(c) for c in np.linspace(0, w.C - 1, want + 2)[1:-1])) if want < w.C else list(range(w.C))
    t_total, done = 0.0, []
    t_begin = time.perf_counter()
    for c in chunks:
        g = synth.gradients(w, 1, chunks=[c])
        Wc = synth.weights(w, chunks=[c])
        z = np.zeros((1, w.r), np.float32)
        t0 = time.perf_counter()
        idx, val = orc.topk(g, w.k)
        p, q = orc.project(idx, val, At_host)
        m, v, mh, vh = orc.adam(p, q, z, z, 1)
        t1 = time.perf_counter()
        om = orc.omp(mh[0], At_host, iters, norm=norm)
        t2 = time.perf_counter()
        if shared_support:
            ov = {"sel": om["sel"], "x": orc.lstsq_support(vh[0], At_host, om["sel"])}
        else:
            ov = orc.omp(vh[0], At_host, iters, norm=norm)
        t3 = time.perf_counter()
        orc.apply(Wc, w.d, om["sel"][None], om["x"][None], ov["sel"][None], np.asarray(ov["x"], np.float32)[None])
        t4 = time.perf_counter()
        scale = w.k / iters
        t_total += (t1 - t0) + (t2 - t1) * scale + (t3 - t2) * (1.0 if shared_support else scale) + (t4 - t3)
        done.append(c)
        if time.perf_counter() - t_begin > budget_s:
            break
    return {
        "value": round(w.d * len(done) / t_total, 2), "unit": "elements/s", "cores": 1, "kind": "oracle",
        "sample": "chunks %s of step 1 (%d of %d chunks), each through the whole path: top-k, projection, Adam, "
                  "OMP(mhat), %s, apply; %s; %.1f s of CPU work counted"
                  % (done, len(done), w.C, "least-squares fit of vhat on its support" if shared_support else "OMP(vhat)",
                     "all %d iterations timed" % w.k if iters == w.k else
                     "recoveries timed for %d of %d iterations and scaled" % (iters, w.k), t_total),
        "host_cores": os.cpu_count(),
    }


if __name__ == "__main__":
    sys.exit(main())
