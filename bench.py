#!/usr/bin/env python3
"""Benchmark of the signature-kernel hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic paths: the forward call followed by the
backward call, as a training step makes them (pairs: sigkernel_fwd then sigkernel_bwd; Gram workloads: sigkernel_gram
without and with grad_K).  Inputs, outputs and workspace are resident in HBM before the timed region starts.

The headline is configuration 5, the largest one: K(X, Y) and K(X, X) of two sets of 1024 paths, forward and
backward, as ONE step (four calls, 2 x 1024^2 kernel evaluations).  The other configurations are timed in the same
run with the same --steps / --warmup and listed under "configs"; `--workload cN` measures one configuration alone
(what the rocprofv3 summaries under profiles/ are made with).

metric  = PDE cell-updates per second over forward + backward: cells / (seconds per step), where
          cells = pairs * 2^lam (L-1) * 2^lam (L-1) is counted once per step (each of the two calls sweeps every
          cell at least once; the backward call also recovers the forward values).  For K(X, X) all N^2 entries are
          counted; the library solves the N (N + 1) / 2 pairs n <= m and copies the rest (k(x, y) = k(y, x) bit for
          bit), and the rate over the cells actually solved is reported next to it.
After the timed region the outputs of the last step are compared with the CPU oracle on sampled pairs / rows
("parity_checked"); a mismatch fails the run.
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

FP64_VECTOR_PEAK_TFLOPS = 78.6    # MI355X: 256 CUs x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz
FP32_VECTOR_PEAK_TFLOPS = 157.3   # packed fp32; the sweeps run in fp64 whatever the caller's type
TOL = {"f64": 1e-10, "f32": 1e-4}
KEEP_LIMIT = 1 << 30   # a forward call keeps its sweep for the backward call if that takes at most this many bytes of
                       # workspace more than the backward call needs anyway


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


def bench_signature(args):
    """Side measurement (not the headline): batched truncated signatures by Horner's scheme (Section 2.3) and their
    gradients (Section 2.4) on the shapes (B, L, d, N) of the paper's Table 1.  A step is one signature_fwd call
    followed by one signature_bwd call that is handed the signatures.  Algorithmic work per path and segment,
    forward: for every level k one multiply-add per entry of the nested products of lengths 1..k, that is
    F = sum_{k=1..N} sum_{j=1..k} d^j multiply-adds (the divisions by k - j of the scheme are not counted);
    backward: the same step once more with the negated increment, and two multiply-adds of the adjoint for each
    multiply-add of the step: 3 F."""
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

    def step():
        sk.signature_fwd(x, N, flags, ws=ws, out=out)
        sk.signature_bwd(x, G, N, flags, sig=out, ws=ws, grad_x=gx)

    copy_calibration(args, torch, dev)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        on = args.time_every > 0 and i % args.time_every == 0
        if on:
            sk.sigkernel_event_timing(1)
        step()
        if on:
            sk.sigkernel_event_timing(0)
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


def copy_calibration(args, torch, dev):
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst


class Part:
    """One forward call + one backward call on the same paths: a pair batch, or one Gram matrix of a step."""

    def __init__(self, tag, label, fwd, bwd, pairs, pairs_solved, desc_fwd, desc_bwd, ws):
        self.tag, self.label, self.fwd, self.bwd = tag, label, fwd, bwd
        self.pairs, self.pairs_solved = pairs, pairs_solved
        self.desc_fwd, self.desc_bwd = desc_fwd, desc_bwd
        self.ws = ws

    def pairs_solved_twice(self):
        """Pairs the last backward call handed to the replay kernel because the inverse recurrence drifted (the
        launch description says where in the workspace the call counts them): 0 means the timed path was the fast one."""
        import torch
        if not self.bwd or "drifted_pairs_counter_at=" not in self.desc_bwd:
            return None
        at = int(self.desc_bwd.split("drifted_pairs_counter_at=", 1)[1].split()[0])
        torch.cuda.synchronize()
        return int(self.ws[at:at + 4].view(torch.int32)[0])


def make_case(name, io, args, sk, workloads, torch, dev):
    """Buffers and calls of one configuration.  Returns a dict with the parts of a step, the counted cells and a
    parity() closure that compares the outputs the last step left with the oracle."""
    import numpy as np
    w, X, Y = workloads.make(name)
    tdt = torch.float64 if io == "f64" else torch.float32
    sdt = sk.SK_F64 if io == "f64" else sk.SK_F32
    lam, flags = w.lam, w.flags
    if args.lead_lag:
        flags |= sk.SK_FLAG_LEAD_LAG
    ll4 = 4 if args.lead_lag else 1      # the transformed paths have 2 (L - 1) steps
    x = torch.tensor(X, device=dev, dtype=tdt)
    y = torch.tensor(Y, device=dev, dtype=tdt)
    Xr, Yr = x.cpu().numpy().astype(np.float64), y.cpu().numpy().astype(np.float64)   # as the GPU sees them
    gram = w.kind == "gram"
    keep_ok = w.backward and not args.no_keep_forward
    parts = []
    checks = []
    tol = TOL[io]

    def values_ok(got, ref):
        return bool(np.all(np.isfinite(got)) and np.max(np.abs(got - ref) / np.maximum(1.0, np.abs(ref))) <= tol)

    def grads_ok(got, ref):
        return bool(np.all(np.isfinite(got)) and np.max(np.abs(got - ref)) <= tol * max(1.0, np.max(np.abs(ref))))

    def host(t):
        return t.detach().cpu().numpy().astype(np.float64)

    if gram:
        import oracle   # noqa: F401  (only the parity closure and the cpu_baseline leg use it)
        sets = [("K(X,Y)", x, y, Xr, Yr, False)]
        if name == "c5" and not args.symmetric and not args.no_xx:
            sets.append(("K(X,X)", x, x, Xr, Xr, True))       # configuration 5 asks for both
        if args.symmetric:
            sets = [("K(X,X)", x, x, Xr, Xr, True)]
        for tag, (label, xa, ya, Xa, Ya, sym) in enumerate(sets, start=1):
            N, M = xa.shape[0], ya.shape[0]
            Wn = workloads.upstream_weights(77 + tag, (N, M))
            W = torch.tensor(Wn, device=dev, dtype=tdt)
            Wr = host(W)
            K = torch.empty((N, M), dtype=tdt, device=dev)
            K2 = torch.empty_like(K)
            gX = torch.empty_like(xa)
            gY = None if sym else torch.empty_like(ya)
            # the forward call keeps its sweep for the backward call where that costs at most KEEP_LIMIT bytes of
            # workspace (the rule of the autograd wrappers; the solo kernels keep checkpoints per pair, 7 GB for c3)
            keep = sk.SK_FLAG_KEEP_FORWARD if keep_ok else 0
            if keep and not args.keep_forward_any_size and sk.sigkernel_workspace_bytes(
                    sk.SK_OP_GRAM, N, M, w.L, w.L, w.d, lam, lam, flags | keep, sdt) > KEEP_LIMIT + sk.sigkernel_workspace_bytes(
                    sk.SK_OP_GRAM_BWD, N, M, w.L, w.L, w.d, lam, lam, flags, sdt):
                keep = 0
            have = sk.SK_FLAG_HAVE_FORWARD if keep else 0
            need = max(sk.sigkernel_workspace_bytes(sk.SK_OP_GRAM, N, M, w.L, w.L, w.d, lam, lam, flags | keep, sdt),
                       sk.sigkernel_workspace_bytes(sk.SK_OP_GRAM_BWD, N, M, w.L, w.L, w.d, lam, lam, flags | have, sdt))
            ws = torch.empty(need, dtype=torch.uint8, device=dev)

            def fwd(xa=xa, ya=ya, K=K, ws=ws, keep=keep):
                sk.sigkernel_gram(xa, ya, None, lam, lam, flags | keep, K=K, ws=ws)

            def bwd(xa=xa, ya=ya, W=W, K2=K2, gX=gX, gY=gY, ws=ws, have=have):
                sk.sigkernel_gram(xa, ya, W, lam, lam, flags | have, K=K2, grad_X=gX, grad_Y=gY, ws=ws)

            solved = N * (N + 1) // 2 if sym else N * M
            parts.append(Part(tag, label, fwd, bwd, N * M, solved,
                              sk.sigkernel_describe(sk.SK_OP_GRAM, N, M, w.L, w.L, w.d, lam, lam, flags | keep, sdt),
                              sk.sigkernel_describe(sk.SK_OP_GRAM_BWD, N, M, w.L, w.L, w.d, lam, lam, flags | have, sdt), ws))

            def check(label=label, Xa=Xa, Ya=Ya, Wr=Wr, K=K, K2=K2, gX=gX, gY=gY, sym=sym, N=N, M=M):
                # sampled rows (and columns) of the Gram matrix and of its gradients: one oracle row of M pairs each
                import oracle
                rng = np.random.default_rng(13)
                rows = [0, N - 1, int(rng.integers(1, N - 1))]
                Kh, K2h, gXh = host(K), host(K2), host(gX)
                ok = True
                for n in rows:
                    Kr, g1, _ = oracle.gram(Xa[n:n + 1], Ya, Wr[n:n + 1], lam, lam, flags)
                    ref = g1[0]
                    if sym:   # the total derivative: path n is also the second argument in column n
                        ref = ref + oracle.gram(Xa, Xa[n:n + 1], Wr[:, n:n + 1], lam, lam, flags)[2][0]
                    ok = ok and values_ok(Kh[n], Kr[0]) and values_ok(K2h[n], Kr[0]) and grads_ok(gXh[n], ref)
                if not sym:
                    gYh = host(gY)
                    for m in [0, M - 1, int(rng.integers(1, M - 1))]:
                        Kr, _, g2 = oracle.gram(Xa, Ya[m:m + 1], Wr[:, m:m + 1], lam, lam, flags)
                        ok = ok and values_ok(Kh[:, m], Kr[:, 0]) and grads_ok(gYh[m], g2[0])
                return ok
            checks.append(check)
    else:
        B = w.n_x
        gkn = workloads.upstream_weights(77, (B,))
        gk = torch.tensor(gkn, device=dev, dtype=tdt)
        k = torch.empty((B,), dtype=tdt, device=dev)
        k2 = torch.empty_like(k)
        gx = torch.empty_like(x)
        gy = torch.empty_like(y)
        # A step is a forward call followed by a backward call on the same paths and workspace, so the forward call
        # keeps its sweep for the backward call (launch modes without that form ignore the two flags).
        keep = sk.SK_FLAG_KEEP_FORWARD if keep_ok else 0
        if keep and not args.keep_forward_any_size and sk.sigkernel_workspace_bytes(
                sk.SK_OP_FWD, B, 0, w.L, w.L, w.d, lam, lam, flags | keep, sdt) > KEEP_LIMIT + sk.sigkernel_workspace_bytes(
                sk.SK_OP_BWD, B, 0, w.L, w.L, w.d, lam, lam, flags, sdt):
            keep = 0
        have = sk.SK_FLAG_HAVE_FORWARD if keep else 0
        need = max(sk.sigkernel_workspace_bytes(sk.SK_OP_FWD, B, 0, w.L, w.L, w.d, lam, lam, flags | keep, sdt),
                   sk.sigkernel_workspace_bytes(sk.SK_OP_BWD, B, 0, w.L, w.L, w.d, lam, lam, flags, sdt))
        ws = torch.empty(need, dtype=torch.uint8, device=dev)

        def fwd():
            sk.sigkernel_fwd(x, y, lam, lam, flags | keep, k=k, ws=ws)

        def bwd():
            sk.sigkernel_bwd(x, y, gk, lam, lam, flags | have, grad_x=gx, grad_y=gy, k_out=k2, ws=ws)

        parts.append(Part(1, "pairs", fwd, bwd if w.backward else None, B, B,
                          sk.sigkernel_describe(sk.SK_OP_FWD, B, 0, w.L, w.L, w.d, lam, lam, flags | keep, sdt),
                          sk.sigkernel_describe(sk.SK_OP_BWD, B, 0, w.L, w.L, w.d, lam, lam, flags | have, sdt), ws))

        def check():
            import oracle
            # long paths: the oracle keeps a whole grid per pair, so a sample of the pairs (first, middle, last)
            sample = list(range(B)) if w.cells_per_pair * B <= 1 << 27 else [0, B // 2, B - 1]
            gkr = host(gk)
            if not w.backward:
                return values_ok(host(k)[sample], oracle.fwd(Xr[sample], Yr[sample], lam, lam, flags))
            kr, gxr, gyr = oracle.bwd(Xr[sample], Yr[sample], gkr[sample], lam, lam, flags)
            ok = values_ok(host(k)[sample], kr) and values_ok(host(k2)[sample], kr)
            gxh, gyh = host(gx), host(gy)
            for i, b in enumerate(sample):
                ok = ok and grads_ok(gxh[b], gxr[i]) and grads_ok(gyh[b], gyr[i])
            return ok and bool(np.all(np.isfinite(gxh)) and np.all(np.isfinite(gyh)))
        checks.append(check)

    cells_per_pair = w.cells_per_pair * ll4
    return {"w": w, "io": io, "X": Xr, "Y": Yr, "flags": flags, "parts": parts, "gram": gram,
            "cells": sum(p.pairs for p in parts) * cells_per_pair,
            "cells_solved": sum(p.pairs_solved for p in parts) * cells_per_pair,
            "cells_per_pair": cells_per_pair,
            "parity": lambda: all(c() for c in checks)}


def kernel_name(desc):
    return desc.split("kernel=", 1)[1].split(" grid=", 1)[0] if "kernel=" in desc else "?"


def keeps_forward(desc_fwd):
    """Whether the forward call's launch plan is the first half of the backward pass (its sweep is kept)."""
    return " kept_sweep_half=1 " in desc_fwd


def run_case(case, args, sk, torch):
    """Warm-up, the timed region of exactly --steps steps, the event-timed kernel durations and the parity check of
    one configuration.  Returns the result record."""
    w, parts = case["w"], case["parts"]

    def step(timed=False):
        for p in parts:
            if timed:
                sk.sigkernel_event_timing(p.tag)
            p.fwd()
            if p.bwd:
                p.bwd()
            if timed:
                sk.sigkernel_event_timing(0)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    sk.sigkernel_event_timing_read()      # nothing from before the timed region
    # timed region: exactly --steps steps; in one step out of --time-every the sweep kernels are bracketed by HIP
    # events on the launch stream (a pair of events costs a few microseconds of idle GPU around the launch - on c2
    # 0.195 ms per step with every launch bracketed against 0.180 ms with none - so not in every step)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.time_every > 0 and i % args.time_every == 0)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps

    # per part: average duration of the forward and of the backward sweep kernel, and the algorithmic work of each
    d_eff = w.d * (2 if args.lead_lag else 1)
    ta = bool(case["flags"] & 1)
    launches = []
    for p in parts:
        f_ms, nf, b_ms, nb = sk.sigkernel_event_timing_read(p.tag)
        cells_launch = p.pairs_solved * case["cells_per_pair"]
        rec = {"part": p.label, "pairs": p.pairs, "pairs_solved": p.pairs_solved,
               "fwd_kernel": kernel_name(p.desc_fwd), "fwd_kernel_ms": f_ms / max(nf, 1),
               "fwd_flops": cells_launch * algorithmic_flops_per_cell(d_eff, ta, w.lam, False)}
        if p.bwd:
            rec.update({"pairs_solved_twice": p.pairs_solved_twice(),
                        "bwd_kernel": kernel_name(p.desc_bwd), "bwd_kernel_ms": b_ms / max(nb, 1),
                        "bwd_flops": cells_launch * algorithmic_flops_per_cell(d_eff, ta, w.lam, True)})
        launches.append(rec)
    # roofline of the dominant kernel (the backward sweep when there is one), over all its launches of a step:
    # algorithmic flops per launch (the average launch) / average launch duration
    side = "bwd" if parts[0].bwd else "fwd"
    flops = sum(r[side + "_flops"] for r in launches) / len(launches)
    dom_ms = sum(r[side + "_kernel_ms"] for r in launches) / len(launches)
    achieved = flops / (dom_ms * 1e-3) / 1e12
    desc = parts[0].desc_bwd if side == "bwd" else parts[0].desc_fwd
    plan = dict(kv.split("=", 1) for kv in desc.split(" ") if "=" in kv and not kv.startswith("kernel="))
    roofline = {"bound": "alu", "kernel": kernel_name(desc), "launch": plan, "launches_per_step": len(launches),
                "achieved": achieved, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / FP64_VECTOR_PEAK_TFLOPS, "avg_launch_ms": dom_ms, "flops_per_launch": flops,
                "traffic": None}
    for r in launches:
        for s in ("fwd", "bwd"):
            if s + "_flops" in r:
                r[s + "_frac"] = r.pop(s + "_flops") / (r[s + "_kernel_ms"] * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS
    if case["io"] == "f32":
        roofline["frac_of_fp32_vector_peak"] = achieved / FP32_VECTOR_PEAK_TFLOPS
    # HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary (if any)
    tfile = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tfile) and not args.lead_lag:
        with open(tfile) as f:
            tj = json.load(f)
        ent = tj.get(w.name if case["io"] == "f64" else w.name + "_f32", {}).get("backward sweep" if side == "bwd" else "forward sweep")
        if ent is not None:
            roofline["traffic"] = ent
            roofline["traffic_taken_at"] = tj.get("taken_at")

    parity = None
    if not args.no_parity:
        torch.cuda.synchronize()
        parity = case["parity"]()

    lam = w.lam
    label = "%s: %s, %d pairs, L=%d, d=%d, dyadic order %d%s, %s, fwd%s" % (
        w.name, w.kind if len(parts) == 1 else "K(X,Y) and K(X,X) in one step", sum(p.pairs for p in parts), w.L, w.d, lam,
        (", time-augmented" if ta else "") + (", lead-lag transformed" if args.lead_lag else "") +
        (", K(X,X)" if args.symmetric else ""),
        "fp64" if case["io"] == "f64" else "fp32 arrays (fp64 sweeps)", "+bwd" if parts[0].bwd else "")
    return {"workload": label, "name": w.name, "io_dtype": case["io"], "ms_per_step": sec * 1e3,
            "cells_per_step": case["cells"], "value": case["cells"] / sec,
            "evals_per_s": sum(p.pairs for p in parts) / sec,
            "pairs_solved": sum(p.pairs_solved for p in parts),
            "solved_cells_per_s": case["cells_solved"] / sec,
            "forward_sweep_kept_for_backward": any(keeps_forward(p.desc_fwd) for p in parts),
            "launches": launches, "roofline": roofline, "parity_checked": parity}


def cpu_baseline(case, args):
    """The oracle as it stands (gcc -O2, OpenMP over pairs / rows) on the host cores, on a bounded sample."""
    import numpy as np
    import oracle
    w, X, Y, flags = case["w"], case["X"], case["Y"], case["flags"]
    lam = w.lam
    if case["gram"]:
        n = min(w.n_x, 64)
        Xs, Ys = X[:n], Y[:n]
        sample_pairs = n * n * len(case["parts"])
        what = " and ".join(p.label for p in case["parts"]) + " of the first %d paths" % n
    else:
        n = min(w.n_x, 128)
        Xs, Ys = X[:n], Y[:n]
        sample_pairs = n
        what = "%d pairs" % n
    reps, spent = 0, 0.0
    while spent < args.cpu_seconds and reps < 2000:
        a = time.perf_counter()
        if case["gram"]:
            for p in case["parts"]:
                Ya = Xs if p.label == "K(X,X)" else Ys
                oracle.gram(Xs, Ya, None, lam, lam, flags)
                if w.backward:
                    oracle.gram(Xs, Ya, np.ones((n, n)), lam, lam, flags)
        else:
            oracle.fwd(Xs, Ys, lam, lam, flags)
            if w.backward:
                oracle.bwd(Xs, Ys, np.ones(n), lam, lam, flags)
        spent += time.perf_counter() - a
        reps += 1
    return {"value": sample_pairs * case["cells_per_pair"] * reps / spent, "unit": "cells/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%s of %s (fwd%s; every pair solved, no use of symmetry), %d repetitions, %.1f s" % (
                what, w.name, "+bwd" if w.backward else "", reps, spent)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    help="default: c5 (headline) with c1..c4 and the fp32 leg of c3 listed under 'configs'; c1..c5: that "
                         "configuration alone; s1/s2/s3: truncated signatures on the shapes of the paper's Table 1 (a "
                         "side measurement)")
    ap.add_argument("--dtype", default="f64", choices=["f64", "f32"],
                    help="element type of the caller's arrays (the sweeps run in fp64 either way)")
    ap.add_argument("--lead-lag", action="store_true",
                    help="apply the lead-lag transform on the fly (SK_FLAG_LEAD_LAG): a side measurement, not the headline")
    ap.add_argument("--symmetric", action="store_true",
                    help="Gram workloads: K(X, X) alone instead of K(X, Y) (a side measurement, not the headline)")
    ap.add_argument("--no-xx", action="store_true", help="c5: K(X, Y) alone (a side measurement)")
    ap.add_argument("--mmd", action="store_true",
                    help="Gram workloads: a step is one sigkernel_mmd2 call (value and both gradients): K(X,X), K(X,Y) "
                         "and K(Y,Y) with gradients (a side measurement, not the headline; no roofline figure)")
    ap.add_argument("--time-every", type=int, default=4,
                    help="bracket the sweep launches of one step in this many with HIP events (1: every step)")
    ap.add_argument("--no-keep-forward", action="store_true",
                    help="the backward call sweeps forward again instead of taking over the sweep of the forward call "
                         "before it (SK_FLAG_KEEP_FORWARD / SK_FLAG_HAVE_FORWARD)")
    ap.add_argument("--keep-forward-any-size", action="store_true",
                    help="keep the forward sweep whatever workspace that takes (c3: 7 GB of checkpoints per pair for a "
                         "step that is 10 % shorter); by default only if it adds at most 1 GiB to the backward call's workspace")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true", help="skip the comparison with the oracle after the timed region")
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

    import torch
    from paper_2509_10613_amd import binding as sk
    from paper_2509_10613_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    head_name = args.workload or "c5"
    copy_calibration(args, torch, dev)

    if args.mmd:
        w, X, Y = workloads.make(head_name)
        assert w.kind == "gram" and not args.symmetric, "--mmd is for the Gram workloads"
        x, y = torch.tensor(X, device=dev), torch.tensor(Y, device=dev)
        flags = w.flags | (sk.SK_FLAG_LEAD_LAG if args.lead_lag else 0)
        loss = torch.empty((1,), dtype=torch.float64, device=dev)
        gX, gY = torch.empty_like(x), torch.empty_like(y)
        need = int(sk.load().sigkernel_mmd2_workspace_bytes(w.n_x, w.n_y, w.L, w.L, w.d, w.lam, w.lam, flags, sk.SK_F64, 1))
        wsm = torch.empty(need, dtype=torch.uint8, device=dev)

        def step():
            sk._check(sk.load().sigkernel_mmd2(sk._ptr(x), sk._ptr(y), sk._ptr(loss), sk._ptr(gX), sk._ptr(gY), w.n_x,
                                               w.n_y, w.L, w.L, w.d, w.lam, w.lam, flags, sk.SK_F64, sk._ptr(wsm),
                                               wsm.numel(), sk._stream()))
        # entries of the three Gram matrices; the symmetric ones solve n <= m only
        cells = (w.n_x * w.n_x + w.n_x * w.n_y + w.n_y * w.n_y) * w.cells_per_pair * (4 if args.lead_lag else 1)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / args.steps
        print(json.dumps({"metric": "PDE cell-updates/s (squared MMD with gradients: K(X,X), K(X,Y), K(Y,Y)), fp64, 1 MI355X",
                          "value": cells / sec, "unit": "cells/s", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True,
                          "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
                          "config": {"workload": "%s as two path sets of %d and %d paths, L=%d, d=%d, dyadic order %d, "
                                                 "sigkernel_mmd2" % (w.name, w.n_x, w.n_y, w.L, w.d, w.lam),
                                     "cells_per_step": cells},
                          "roofline": None, "cpu_baseline": None}))
        return

    head_case = make_case(head_name, args.dtype, args, sk, workloads, torch, dev)
    head = run_case(head_case, args, sk, torch)
    cpu = None if args.no_cpu_baseline else cpu_baseline(head_case, args)
    del head_case
    torch.cuda.empty_cache()

    # the other configurations, same protocol, in the same line (only in the default run)
    others = []
    if args.workload is None and not (args.lead_lag or args.symmetric or args.no_xx):
        for name, io in (("c1", "f64"), ("c2", "f64"), ("c3", "f64"), ("c3", "f32"), ("c4", "f64")):
            case = make_case(name, io, args, sk, workloads, torch, dev)
            r = run_case(case, args, sk, torch)
            del case
            torch.cuda.empty_cache()
            others.append({"workload": r["workload"], "ms_per_step": r["ms_per_step"], "cells_per_s": r["value"],
                           "evals_per_s": r["evals_per_s"], "kernel": r["roofline"]["kernel"],
                           "avg_launch_ms": r["roofline"]["avg_launch_ms"], "frac": r["roofline"]["frac"],
                           "fwd_kernel_ms": r["launches"][0]["fwd_kernel_ms"],
                           "forward_sweep_kept_for_backward": r["forward_sweep_kept_for_backward"],
                           "parity_checked": r["parity_checked"]})

    parity_all = None if args.no_parity else bool(head["parity_checked"] and all(o["parity_checked"] for o in others))
    out = {
        "metric": "PDE cell-updates/s (fwd+bwd; config 5: K(X,Y) and K(X,X) of 1024 x 1024 paths, L=64, d=16), fp64, 1 MI355X"
                  if head["name"] == "c5" and len(head["launches"]) == 2 and args.dtype == "f64" else
                  "PDE cell-updates/s (%s; %s), %s, 1 MI355X" % ("fwd+bwd" if "bwd_kernel" in head["launches"][0] else "fwd",
                                                              head["name"], "fp64" if args.dtype == "f64" else "fp32 arrays"),
        "value": head["value"],
        "unit": "cells/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": head["workload"], "cells_per_step": head["cells_per_step"], "io_dtype": head["io_dtype"],
                   "forward_sweep_kept_for_backward": head["forward_sweep_kept_for_backward"]},
        "evals_per_s": head["evals_per_s"],
        "pairs_solved": head["pairs_solved"],
        "solved_cells_per_s": head["solved_cells_per_s"],
        "launches": head["launches"],
        "roofline": head["roofline"],
        "cpu_baseline": cpu,
        "parity_checked": parity_all,
        "configs": others,
    }
    print(json.dumps(out))
    if parity_all is False:
        print("bench.py: outputs of the timed calls do not match the oracle", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
