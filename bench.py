#!/usr/bin/env python3
"""Benchmark of the signature-kernel hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic paths: one sigkernel_fwd call
followed by one sigkernel_bwd call (for the Gram workloads: sigkernel_gram without and with grad_K).
Inputs, outputs and workspace are resident in HBM before the timed region starts.

metric  = PDE cell-updates per second over forward + backward: cells / (t_fwd + t_bwd), where
          cells = pairs * 2^lam (L-1) * 2^lam (L-1) is counted once per step (each of the two calls
          sweeps every cell at least once; the backward call also replays the forward values).
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP64_VECTOR_PEAK_TFLOPS = 78.6   # MI355X: 256 CUs x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz


def algorithmic_flops_per_cell(d, time_aug, lam, backward):
    """Flops the method needs per refined cell (paper Eq. (1) and Section 3.4), independent of how this
    library schedules them: the stencil on every refined cell, and the coefficient polynomials plus the
    d-channel contractions once per coarse cell (4^lam refined cells).
      forward : 4 (stencil) + (7 (A, B) + 2 (d + time)) / 4^lam
      backward: 6 (adjoint recurrence) + 9 (local derivative and accumulation)
                + (10 (A, B, A', B') + 2 (d + time) (Delta) + 4 d (map to dx and dy)) / 4^lam
    The forward values the backward call recomputes are a design cost and are not counted."""
    de = d + (1 if time_aug else 0)
    per_coarse = 4.0 ** lam
    if not backward:
        return 4.0 + (7.0 + 2.0 * de) / per_coarse
    return 15.0 + (10.0 + 2.0 * de + 4.0 * d) / per_coarse


def timed_step(sk, step, i, every):
    """Step i of the timed region.  The library brackets its sweep launches with HIP events on the launch stream while
    event timing is on; a pair of events costs a few microseconds of idle GPU around the launch (measured on c2: 0.195
    ms per step with every launch bracketed, 0.180 ms with none), so only one step in `every` is bracketed.  The
    kernel durations are averages over those steps, taken inside the timed region."""
    on = every > 0 and i % every == 0
    if on:
        sk.sigkernel_event_timing(True)
    step()
    if on:
        sk.sigkernel_event_timing(False)


def bench_signature(args):
    """Side measurement (not the headline): batched truncated signatures by Horner's scheme (Section 2.3) and their
    gradients (Section 2.4) on the shapes (B, L, d, N) of the paper's Table 1.  A step is one signature_fwd call
    followed by one signature_bwd call that is handed the signatures.  Algorithmic work per path and segment,
    forward: for every level k one multiply-add per entry of the nested products of lengths 1..k, that is
    F = sum_{k=1..N} sum_{j=1..k} d^j multiply-adds (the divisions by k - j of the scheme are not counted);
    backward: the same step once more with the negated increment, and two multiply-adds of the adjoint for each
    multiply-add of the step: 3 F."""
    import numpy as np
    import torch
    from paper_2509_10613_amd import binding as sk
    from paper_2509_10613_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    (B, L, d, N), X = workloads.make_signature(args.workload)
    flags = sk.SK_FLAG_LEAD_LAG if args.lead_lag else 0
    D, n = (2 * d, 2 * (L - 1)) if args.lead_lag else (d, L - 1)
    x = torch.tensor(X, device=dev)
    entries = sk.signature_length(d, N, flags)
    out = torch.empty((B, entries), dtype=torch.float64, device=dev)
    G = torch.tensor(workloads.upstream_weights(78, (B, entries)), device=dev)
    gx = torch.empty_like(x)
    ws = torch.empty(max(256, sk.signature_workspace_bytes(B, L, d, N, flags, sk.SK_F64),
                         int(sk.load().signature_bwd_workspace_bytes(B, L, d, N, flags, sk.SK_F64, 1))),
                     dtype=torch.uint8, device=dev)

    def fwd_call():
        sk.signature_fwd(x, N, flags, ws=ws, out=out)

    def bwd_call():
        sk.signature_bwd(x, G, N, flags, sig=out, ws=ws, grad_x=gx)

    def step():
        fwd_call()
        bwd_call()

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        timed_step(sk, step, i, args.time_every)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    f_ms, nf, b_ms, nb = sk.sigkernel_event_timing_read()
    sec = (t1 - t0) / args.steps
    fma = sum(sum(D ** j for j in range(1, k + 1)) for k in range(1, N + 1))
    fwd_ms, bwd_ms = f_ms / max(nf, 1), b_ms / max(nb, 1)
    flops = 2.0 * 3.0 * fma * B * n            # the backward kernel, the dominant one
    achieved = flops / (bwd_ms * 1e-3) / 1e12
    fwd_frac = 2.0 * fma * B * n / (fwd_ms * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS
    desc = sk.signature_bwd_describe(B, L, d, N, flags, sk.SK_F64)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import signature as osig
        Gh = G.cpu().numpy()
        npaths, spent = 0, 0.0
        while spent < args.cpu_seconds and npaths < B:
            a = time.perf_counter()
            osig.signature(X[npaths:npaths + 1], N, flags)
            osig.signature_backward(X[npaths:npaths + 1], Gh[npaths:npaths + 1], N, flags)
            spent += time.perf_counter() - a
            npaths += 1
        cpu = {"value": npaths * n * (entries - 1) / spent, "unit": "entry updates/s", "cores": 1, "kind": "oracle",
               "sample": "%d paths of %s, fwd+bwd, %.1f s (numpy, full tensor products)" % (npaths, args.workload, spent)}
    print(json.dumps({
        "metric": "signature entry updates/s (truncated signatures by Horner's scheme, fwd+bwd), fp64, 1 MI355X",
        "value": B * n * (entries - 1) / sec, "unit": "entry updates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "%s: %d paths, L=%d, d=%d, truncation level %d%s, fp64, fwd+bwd" % (
            args.workload, B, L, d, N, ", lead-lag transformed" if args.lead_lag else ""),
            "entries_per_path": entries},
        "paths_per_s": B / sec, "horner_kernel_ms": fwd_ms, "horner_bwd_kernel_ms": bwd_ms,
        "fwd_kernel": sk.signature_describe(B, L, d, N, flags, sk.SK_F64).split("kernel=", 1)[1].split(" channels=", 1)[0],
        "fwd_frac_of_peak": fwd_frac,
        "roofline": {"bound": "alu", "kernel": desc.split("kernel=", 1)[1].split(" channels=", 1)[0],
                     "launch": dict(kv.split("=", 1) for kv in desc.split(" ") if "=" in kv and not kv.startswith("kernel=")),
                     "achieved": achieved, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / FP64_VECTOR_PEAK_TFLOPS, "avg_launch_ms": bwd_ms, "flops_per_launch": flops,
                     "traffic": None},
        "cpu_baseline": cpu}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", help="c2 (headline), c1/c3/c4/c5 for the other configurations, or "
                    "s1/s2/s3 for truncated signatures on the shapes of the paper's Table 1 (a side measurement)")
    ap.add_argument("--lead-lag", action="store_true",
                    help="apply the lead-lag transform on the fly (SK_FLAG_LEAD_LAG): a side measurement, not the headline")
    ap.add_argument("--symmetric", action="store_true",
                    help="Gram workloads: K(X, X) instead of K(X, Y) (a side measurement, not the headline)")
    ap.add_argument("--mmd", action="store_true",
                    help="Gram workloads: a step is one sigkernel_mmd2 call (value and both gradients): K(X,X), K(X,Y) "
                         "and K(Y,Y) with gradients (a side measurement, not the headline; no roofline figure)")
    ap.add_argument("--time-every", type=int, default=8,
                    help="bracket the sweep launches of one step in this many with HIP events (1: every step)")
    ap.add_argument("--no-keep-forward", action="store_true",
                    help="pair workloads: the backward call sweeps forward again instead of taking over the sweep of the "
                         "forward call before it (SK_FLAG_KEEP_FORWARD / SK_FLAG_HAVE_FORWARD)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy, so that a rocprofv3 --pmc run of this command "
                         "holds a kernel of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (pairs are independent; see DESIGN.md for how the "
              "path would shard); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.workload in ("s1", "s2", "s3"):
        return bench_signature(args)

    import numpy as np
    import torch
    from paper_2509_10613_amd import binding as sk
    from paper_2509_10613_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    w, X, Y = workloads.make(args.workload)
    lam, flags = w.lam, w.flags
    if args.lead_lag:
        flags |= sk.SK_FLAG_LEAD_LAG
    x = torch.tensor(X, device=dev)
    y = torch.tensor(Y, device=dev)
    if args.symmetric:
        assert w.kind == "gram", "--symmetric is for the Gram workloads"
        y, Y = x, X   # the same tensor selects the symmetric case
    cells = w.pairs * w.cells_per_pair * (4 if args.lead_lag else 1)   # the transformed paths have 2 (L - 1) steps
    gram = w.kind == "gram"
    f64 = sk.SK_F64

    if gram:
        W = torch.tensor(workloads.upstream_weights(77, (w.n_x, w.n_y)), device=dev)
        K = torch.empty((w.n_x, w.n_y), dtype=torch.float64, device=dev)
        gX = torch.empty_like(x)
        gY = torch.empty_like(y)
        # (as for the pair workloads below: the forward call keeps its sweep for the backward call where the launch
        # mode can; the tile kernels of c5 cannot and ignore the flags)
        keep = sk.SK_FLAG_KEEP_FORWARD if (w.backward and not args.no_keep_forward and not args.mmd) else 0
        have = sk.SK_FLAG_HAVE_FORWARD if keep else 0
        need = max(sk.sigkernel_workspace_bytes(sk.SK_OP_GRAM, w.n_x, w.n_y, w.L, w.L, w.d, lam, lam, flags | keep, f64),
                   sk.sigkernel_workspace_bytes(sk.SK_OP_GRAM_BWD, w.n_x, w.n_y, w.L, w.L, w.d, lam, lam, flags | have, f64))
        ws = torch.empty(need, dtype=torch.uint8, device=dev)

        def fwd_call():
            sk.sigkernel_gram(x, y, None, lam, lam, flags | keep, K=K, ws=ws)

        def bwd_call():
            sk.sigkernel_gram(x, y, W, lam, lam, flags | have, K=K, grad_X=gX, grad_Y=None if args.symmetric else gY, ws=ws)
    else:
        gk = torch.tensor(workloads.upstream_weights(77, (w.n_x,)), device=dev)
        k = torch.empty((w.n_x,), dtype=torch.float64, device=dev)
        k2 = torch.empty_like(k)
        gx = torch.empty_like(x)
        gy = torch.empty_like(y)
        # A step is a forward call followed by a backward call on the same paths and workspace, so the forward call
        # keeps its sweep for the backward call (launch modes without that form ignore the two flags).
        keep = sk.SK_FLAG_KEEP_FORWARD if (w.backward and not args.no_keep_forward) else 0
        have = sk.SK_FLAG_HAVE_FORWARD if keep else 0
        need = max(sk.sigkernel_workspace_bytes(sk.SK_OP_FWD, w.n_x, 0, w.L, w.L, w.d, lam, lam, flags | keep, f64),
                   sk.sigkernel_workspace_bytes(sk.SK_OP_BWD, w.n_x, 0, w.L, w.L, w.d, lam, lam, flags, f64))
        ws = torch.empty(need, dtype=torch.uint8, device=dev)

        def fwd_call():
            sk.sigkernel_fwd(x, y, lam, lam, flags | keep, k=k, ws=ws)

        def bwd_call():
            sk.sigkernel_bwd(x, y, gk, lam, lam, flags | have, grad_x=gx, grad_y=gy, k_out=k2, ws=ws)

    def step():
        fwd_call()
        if w.backward:
            bwd_call()

    if args.mmd:
        assert gram and not args.symmetric, "--mmd is for the Gram workloads"
        loss = torch.empty((1,), dtype=torch.float64, device=dev)
        need = int(sk.load().sigkernel_mmd2_workspace_bytes(w.n_x, w.n_y, w.L, w.L, w.d, lam, lam, flags, f64, 1))
        wsm = torch.empty(need, dtype=torch.uint8, device=dev)

        def step():   # noqa: F811
            sk._check(sk.load().sigkernel_mmd2(sk._ptr(x), sk._ptr(y), sk._ptr(loss), sk._ptr(gX), sk._ptr(gY), w.n_x,
                                               w.n_y, w.L, w.L, w.d, lam, lam, flags, f64, sk._ptr(wsm), wsm.numel(),
                                               sk._stream()))
        # entries of the three Gram matrices; the symmetric ones solve n <= m only
        cells = (w.n_x * w.n_x + w.n_x * w.n_y + w.n_y * w.n_y) * w.cells_per_pair * (4 if args.lead_lag else 1)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly --steps steps; in one step out of --time-every the sweep kernels are bracketed by HIP events
    # on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        timed_step(sk, step, i, args.time_every)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    fwd_ms, nf, bwd_ms, nb = sk.sigkernel_event_timing_read()
    sec_per_step = (t1 - t0) / args.steps

    # separate timings of the two calls (reported, not the headline)
    def time_call(fn, n):
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - a) / n

    if args.mmd:
        print(json.dumps({"metric": "PDE cell-updates/s (squared MMD with gradients: K(X,X), K(X,Y), K(Y,Y)), fp64, 1 MI355X",
                          "value": cells / sec_per_step, "unit": "cells/s", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": sec_per_step * 1e3, "higher_is_better": True,
                          "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
                          "config": {"workload": "%s as two path sets of %d and %d paths, L=%d, d=%d, dyadic order %d, "
                                                 "sigkernel_mmd2" % (w.name, w.n_x, w.n_y, w.L, w.d, lam),
                                     "cells_per_step": cells},
                          "sweep_launches_ms": (fwd_ms + bwd_ms) / args.steps, "roofline": None, "cpu_baseline": None}))
        return
    n_sep = max(3, args.steps // 4)
    t_fwd = time_call(fwd_call, n_sep)
    t_bwd = time_call(bwd_call, n_sep) if w.backward else None

    # roofline of the dominant kernel (the backward sweep when there is one)
    dom_back = bool(w.backward and nb > 0)
    dom_ms = (bwd_ms / nb) if dom_back else (fwd_ms / max(nf, 1))
    flops = cells * algorithmic_flops_per_cell(w.d * (2 if args.lead_lag else 1), bool(flags & 1), lam, dom_back)
    achieved = flops / (dom_ms * 1e-3) / 1e12
    # the sweep kernel's name as a profiler reports it, from the library's own launch plan
    if gram:
        desc = sk.sigkernel_describe(sk.SK_OP_GRAM_BWD if dom_back else sk.SK_OP_GRAM, w.n_x, w.n_y, w.L, w.L, w.d, lam,
                                     lam, flags | (have if dom_back else keep), f64)
    else:
        desc = sk.sigkernel_describe(sk.SK_OP_BWD if dom_back else sk.SK_OP_FWD, w.n_x, 0, w.L, w.L, w.d, lam, lam,
                                     flags | (have if dom_back else keep), f64)
    plan = dict(kv.split("=", 1) for kv in desc.split(" ") if "=" in kv and not kv.startswith("kernel="))
    kname = desc.split("kernel=", 1)[1].split(" grid=", 1)[0] if "kernel=" in desc else "?"
    roofline = {"bound": "alu", "kernel": kname, "launch": plan,
                "achieved": achieved, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / FP64_VECTOR_PEAK_TFLOPS, "avg_launch_ms": dom_ms,
                "flops_per_launch": flops, "traffic": None}
    fwd_kernel_ms = fwd_ms / max(nf, 1)
    # HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary (if any)
    tfile = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tfile):
        with open(tfile) as f:
            tj = json.load(f)
        ent = tj.get(w.name, {}).get("backward sweep" if dom_back else "forward sweep")
        if ent is not None:
            roofline["traffic"] = ent

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        nx = min(w.n_x, 128 if not gram else 12)
        ny = min(w.n_y, 128 if not gram else 12)
        Xs, Ys = X[:nx], Y[:ny]
        sample_pairs = nx * ny if gram else nx
        reps, spent = 0, 0.0
        while spent < args.cpu_seconds and reps < 2000:
            a = time.perf_counter()
            if gram:
                oracle.gram(Xs, Ys, None, lam, lam, flags)
                if w.backward:
                    oracle.gram(Xs, Ys, np.ones((nx, ny)), lam, lam, flags)
            else:
                oracle.fwd(Xs, Ys, lam, lam, flags)
                if w.backward:
                    oracle.bwd(Xs, Ys, np.ones(nx), lam, lam, flags)
            spent += time.perf_counter() - a
            reps += 1
        cpu = {"value": sample_pairs * w.cells_per_pair * (4 if args.lead_lag else 1) * reps / spent, "unit": "cells/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": "%d pairs of %s (fwd%s), %d repetitions, %.1f s" % (sample_pairs, w.name,
                                                                             "+bwd" if w.backward else "", reps, spent)}

    out = {
        "metric": "PDE cell-updates/s (%s), fp64, 1 MI355X" % ("fwd+bwd" if w.backward else "fwd"),
        "value": cells / sec_per_step,
        "unit": "cells/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "%s: %s, %d pairs, L=%d, d=%d, dyadic order %d%s, fp64, fwd%s" % (
            w.name, w.kind, w.pairs, w.L, w.d, lam,
            (", time-augmented" if flags & 1 else "") + (", lead-lag transformed" if args.lead_lag else "") +
            (", K(X,X)" if args.symmetric else ""),
            "+bwd" if w.backward else ""), "cells_per_step": cells,
            "forward_sweep_kept_for_backward": bool(keep) and (
                sk.keeps_forward(w.n_x, w.L, w.L, w.d, lam, lam, flags, f64, gram_M=w.n_y if gram else None))},
        "evals_per_s": w.pairs / sec_per_step,
        # K(X, X): the library solves the pairs n <= m only (k(x, y) = k(y, x) bit for bit) and copies the rest
        "pairs_solved": (w.n_x * (w.n_x + 1) // 2) if args.symmetric else w.pairs,
        "solved_cells_per_s": (cells * ((w.n_x + 1) / (2.0 * w.n_x)) if args.symmetric else cells) / sec_per_step,
        "fwd_call_ms": t_fwd * 1e3,
        "bwd_call_ms": None if t_bwd is None else t_bwd * 1e3,
        "fwd_cells_per_s": cells / t_fwd,
        "bwd_cells_per_s": None if t_bwd is None else cells / t_bwd,
        "fwd_sweep_kernel_ms": fwd_kernel_ms,
        "bwd_sweep_kernel_ms": (bwd_ms / nb) if nb else None,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
