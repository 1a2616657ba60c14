#!/usr/bin/env python3
"""Headline benchmark: one RevFFN block, forward + inverse + backward, at the Qwen1.5-MoE-A2.7B
layer shape (batch 4 x seq 512, bf16 storage, fp32 accumulation) on ONE MI355X.

A "step" is one pass of the whole hot path over one batch: revffn_forward, revffn_inverse
(rebuilding the input from the output) and revffn_backward (recomputing activations from the
rebuilt input, all weight gradients written).  Inputs and weights are resident in HBM before
the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def cpu_baseline(wl, W32, x1, x2, dy1, dy2, n_inv_iters, symmetric=False):
    """Time the fp64 oracle (as it stands) on the same batch."""
    import numpy as np
    from oracle import revffn_oracle as O
    S = wl.S
    cores = len(os.sched_getaffinity(0))
    W = O.as_f64(W32)                         # promotion of the stored weights is not timed
    cfg = O.Config(wl.d_model, wl.n_heads, wl.head_dim, wl.n_experts, wl.top_k, wl.d_expert, wl.d_shared,
                   n_inv_iters=n_inv_iters, symmetric=symmetric)
    nb = min(wl.B, 4)                         # whole sequences; a few seconds each
    a, b, ga, gb = (np.ascontiguousarray(t[:nb * S]) for t in (x1, x2, dy1, dy2))
    t0 = time.perf_counter()
    y1, y2 = O.forward(a, b, W, cfg, nb, S)
    O.grads_reconstructed(y1, y2, ga, gb, W, cfg, nb, S)
    dt = time.perf_counter() - t0
    return {"value": nb * S / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"forward + inverse + backward of {nb} of the {wl.B} sequences (S={S}) of the same batch, "
                      f"full-size weights, numpy float64, {dt:.1f} s"}


def bench_stack(args, wl):
    """Stack of wl.n_blocks blocks: forward keeping only the last state, then the backward sweep that
    rebuilds every block's input from its output (no cached activations).  Reports tokens/s, peak HBM
    bytes and the reconstruction drift at the stack input."""
    import numpy as np
    import torch
    import synth
    import paper_2512_20920_amd as R
    from paper_2512_20920_amd import harness as Hn

    t_setup = time.perf_counter()
    L = wl.n_blocks
    Wds, Gs = [], []
    for l in range(L):
        Wd = Hn.upload_weights(synth.make_weights(wl, block=l, f64=False), wl.dtype)
        Wds.append(Wd)
        Gs.append(Hn.alloc_grads(Wd, fp32=args.fp32_grads))
    x1, x2, dy1, dy2 = synth.make_inputs(wl)
    sdt = "f32" if args.fp32_streams else wl.dtype
    x1d, x2d, dy1d, dy2d = Hn.upload(x1, sdt), Hn.upload(x2, sdt), Hn.upload(dy1, wl.dtype), Hn.upload(dy2, wl.dtype)
    new = lambda dt=sdt: torch.empty((wl.T, wl.h), dtype=Hn.torch_dtype(dt), device="cuda")
    y1d, y2d, s1, s2, g1, g2 = new(), new(), new(), new(), new(wl.dtype), new(wl.dtype)
    ctx = R.Context(Hn.make_config(wl, n_inv_iters=args.inv_iters, fp32_streams=args.fp32_streams, symmetric=args.symmetric, fp32_grads=args.fp32_grads), wl.B, wl.S)
    if args.inv_tol > 0:
        ctx.set_inverse_tolerance(args.inv_tol, args.inv_max_iters, args.inv_block)
    ws = (R.Weights * L)(*[R.binding._struct(R.Weights, w) for w in Wds])
    gs = (R.Grads * L)(*[R.binding._struct(R.Grads, g) for g in Gs])
    stream = torch.cuda.current_stream()
    if args.stored:
        # the non-reversible comparison: one context (one block's activations) per layer and every block boundary
        # state kept; forward fills them, the backward walk reads them (no inverse, no recomputation)
        ctxs = [ctx] + [R.Context(Hn.make_config(wl, n_inv_iters=args.inv_iters, fp32_streams=args.fp32_streams, symmetric=args.symmetric, fp32_grads=args.fp32_grads),
                                  wl.B, wl.S) for _ in range(L - 1)]
        states = [(x1d, x2d)] + [(new(), new()) for _ in range(L)]
        wstructs = [R.binding._struct(R.Weights, w) for w in Wds]
        gstructs = [R.binding._struct(R.Grads, g) for g in Gs]
        h1, h2 = new(wl.dtype), new(wl.dtype)
    t_setup = time.perf_counter() - t_setup

    def step():
        if args.stored:
            for l in range(L):
                R.revffn_forward(ctxs[l], wstructs[l], states[l][0], states[l][1], states[l + 1][0], states[l + 1][1],
                                 wl.B, wl.S, wl.h, stream)
            ga, gb = dy1d, dy2d
            for l in range(L - 1, -1, -1):
                na, nb = (g1, g2) if ga is not g1 else (h1, h2)           # ping-pong gradient buffers
                R.revffn_backward_stored(ctxs[l], wstructs[l], states[l][0], states[l][1], states[l + 1][0], ga, gb,
                                         na, nb, gstructs[l], wl.B, wl.S, wl.h, stream)
                ga, gb = na, nb
            return
        R.binding._check(ctx.lib.revffn_stack_forward(ctx.handle, ws, L, x1d.data_ptr(), x2d.data_ptr(), y1d.data_ptr(),
                                                      y2d.data_ptr(), wl.B, wl.S, wl.h, stream.cuda_stream))
        s1.copy_(y1d); s2.copy_(y2d); g1.copy_(dy1d); g2.copy_(dy2d)      # the sweep works in place
        R.binding._check(ctx.lib.revffn_stack_backward(ctx.handle, ws, gs, L, s1.data_ptr(), s2.data_ptr(), g1.data_ptr(),
                                                       g2.data_ptr(), wl.B, wl.S, wl.h, stream.cuda_stream))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.inv_tol > 0:
        ctx.set_inverse_tolerance(args.inv_tol, args.inv_max_iters, args.inv_block)   # (restarts the iteration statistics)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    inv_calls, inv_total = ctx.inverse_stats()[:2]
    drift1 = 0.0 if args.stored else float((s1.float() - x1d.float()).abs().max())
    drift2 = 0.0 if args.stored else float((s2.float() - x2d.float()).abs().max())
    weights_bytes = sum(t.numel() * t.element_size() for w in Wds for t in w.values() if t is not None)
    out = {
        "metric": ("RevFFN 24-block stack forward + stored-activation backward (non-reversible comparison), tokens/s"
                   if args.stored else "RevFFN 24-block stack forward + reconstructing backward sweep, tokens/s"),
        "value": wl.T / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {L} RevFFN blocks at the Qwen1.5-MoE-A2.7B layer shape, B={wl.B} S={wl.S}",
                   "n_inv_iters": args.inv_iters, "setup_s": round(t_setup, 1),
                   "residual_streams": "f32" if args.fp32_streams else wl.dtype,
                   "block": "symmetric comparison block" if args.symmetric else "RevFFN (Eq. 1-2)",
                   **({"inv_tol": args.inv_tol, "inv_max_iters": args.inv_max_iters,
                       "mean_iters_per_inverse": inv_total / max(inv_calls, 1)} if args.inv_tol > 0 else {})},
        "peak_hbm_bytes": int(torch.cuda.max_memory_allocated()) + int(ctx.workspace_bytes(wl.B, wl.S)) * (L if args.stored else 1),
        "weights_bytes": int(weights_bytes), "gradient_bytes": int(sum(t.numel() * t.element_size() for g in Gs for t in g.values() if t is not None)),
        "activation_workspace_bytes": int(ctx.workspace_bytes(wl.B, wl.S)) * (L if args.stored else 1),
        "activations": "stored: one workspace per block + every block boundary state" if args.stored else "reversible: one workspace",
        "reconstruction_drift_at_stack_input": {"max_abs_x1": drift1, "max_abs_x2": drift2,
                                                "note": "max |rebuilt - true| after walking all blocks down"},
        "csrc_sha16": csrc_hash(),
    }
    print(json.dumps(out))


def csrc_hash():
    """First 16 hex digits of the SHA-256 over the kernel sources: stamps a measurement with the kernels it was
    taken from."""
    import glob
    import hashlib
    hsh = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2512_20920_amd", "csrc")
    for path in sorted(glob.glob(os.path.join(base, "*.hip")) + glob.glob(os.path.join(base, "*.h"))):
        hsh.update(os.path.basename(path).encode())
        hsh.update(open(path, "rb").read())
    return hsh.hexdigest()[:16]


def measured_traffic(workload, family):
    """HBM bytes per launch of a kernel family (fetched + written), from the committed rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE summary of this workload.  None when there is no such summary, or when it was measured with other
    kernel sources than the ones in this tree (its `csrc_sha16` stamp differs): a stale figure is not reported."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic__{workload}.json")
    try:
        with open(path) as f:
            doc = json.load(f)
        if doc.get("csrc_sha16") != csrc_hash():
            return None
        fam = doc["families"].get(family)
    except (OSError, ValueError, KeyError):
        return None
    return None if fam is None else fam["fetch_bytes_per_launch"] + fam["write_bytes_per_launch"]


def routing_report(wl, W32, y1_host):
    """Near-ties and flips of the timed workload's routing (part of the CPU leg: it runs the oracle's router on the
    stream-1 values the GPU stored).  A near-tie is a token whose top-k logit margin or a gap between selected
    logits is <= 1e-3; a flip is a token whose GPU selection differs from the oracle's."""
    import numpy as np
    from oracle import revffn_oracle as O
    cfg = O.Config(wl.d_model, wl.n_heads, wl.head_dim, wl.n_experts, wl.top_k, wl.d_expert, wl.d_shared)
    f = lambda a: np.asarray(a, dtype=np.float64)
    um = O.rmsnorm(y1_host, f(W32["norm_m"]), cfg.rms_eps) @ f(W32["pup_m"]).T
    z = um @ f(W32["w_router"]).T
    if W32.get("b_router") is not None:
        z = z + f(W32["b_router"])
    idx, _, _ = O.route(z, cfg)
    margin = O.topk_margin(z, cfg.top_k)
    zsel = np.take_along_axis(z, idx.astype(np.int64), axis=-1)
    gaps = np.min(-np.diff(zsel, axis=-1), axis=-1) if cfg.top_k > 1 else np.full(len(margin), np.inf)
    return idx, int(((margin <= 1e-3) | (gaps <= 1e-3)).sum())


def time_steps(torch, step, stream, K):
    """K steps, each between its own pair of events on `stream`; returns (median ms, mean ms)."""
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    evs[0].record(stream)
    for i in range(K):
        step()
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(K))
    med = per[K // 2] if K % 2 else 0.5 * (per[K // 2 - 1] + per[K // 2])
    return med, evs[0].elapsed_time(evs[K]) / K


def family_roofline(p):
    """Algorithmic flops and bytes per launch over the average launch duration; the bound is whichever published
    peak the family's work sits closer to (families without flops are memory-bound)."""
    avg_ms = p["ms"] / p["launches"]
    tflops = p["flops"] / p["launches"] / (avg_ms * 1e-3) / 1e12
    gbs = p["bytes"] / p["launches"] / (avg_ms * 1e-3) / 1e9
    if tflops / PEAK_BF16_TFLOPS >= gbs / PEAK_HBM_GBS:
        return {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": tflops / PEAK_BF16_TFLOPS}
    return {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}


def bench_block(args, wl, headline):
    """One single-block workload.  headline: the full record (both call forms, per-kernel pass, routing report, CPU
    leg); otherwise a compact record (timed steps and the per-kernel pass)."""
    import torch
    import synth
    import paper_2512_20920_amd as R
    from paper_2512_20920_amd import harness as Hn

    t_setup = time.perf_counter()
    W32 = synth.make_weights(wl, f64=False)
    x1, x2, dy1, dy2 = synth.make_inputs(wl)
    Wd = Hn.upload_weights(W32, wl.dtype)
    adapters = ("pup_a", "pdn_a", "pup_m", "pdn_m")
    frozen = {"all": (), "stage1": tuple(n for n in R.WEIGHT_FIELDS if n not in adapters),
              "stage2": ("w_router", "b_router")}[args.train]
    G = Hn.alloc_grads(Wd, skip=frozen, fp32=args.fp32_grads)
    sdt = "f32" if args.fp32_streams else wl.dtype
    x1d, x2d, dy1d, dy2d = Hn.upload(x1, sdt), Hn.upload(x2, sdt), Hn.upload(dy1, wl.dtype), Hn.upload(dy2, wl.dtype)
    new = lambda dt=sdt: torch.empty((wl.T, wl.h), dtype=Hn.torch_dtype(dt), device="cuda")
    y1d, y2d, r1d, r2d, dx1d, dx2d = new(), new(), new(), new(), new(wl.dtype), new(wl.dtype)
    ctx = R.Context(Hn.make_config(wl, n_inv_iters=args.inv_iters, fp32_streams=args.fp32_streams, symmetric=args.symmetric, fp32_grads=args.fp32_grads), wl.B, wl.S)
    wstruct = R.binding._struct(R.Weights, Wd)
    gstruct = R.binding._struct(R.Grads, G)
    stream = torch.cuda.current_stream()
    t_setup = time.perf_counter() - t_setup

    def step_fused():
        # forward, then the sweep step: inverse (input rebuilt from the output) + backward at the rebuilt input
        R.revffn_forward(ctx, wstruct, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h, stream)
        R.revffn_inverse_backward(ctx, wstruct, y1d, y2d, r1d, r2d, dy1d, dy2d, dx1d, dx2d, gstruct,
                                  wl.B, wl.S, wl.h, None, stream)

    def step_three():
        # the three calls as the boundary names them: the MoE half is evaluated by the inverse and again by backward
        R.revffn_forward(ctx, wstruct, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h, stream)
        R.revffn_inverse(ctx, wstruct, y1d, y2d, r1d, r2d, wl.B, wl.S, wl.h, None, stream)
        R.revffn_backward(ctx, wstruct, r1d, r2d, y1d, dy1d, dy2d, dx1d, dx2d, gstruct, wl.B, wl.S, wl.h, stream)

    step = step_three if args.separate_calls else step_fused
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        # the same calls recorded once (helper streams and their event dependencies included) and replayed
        eager_stream, stream = stream, torch.cuda.Stream()       # step() enqueues on `stream`
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):
            with torch.cuda.graph(graph, stream=stream):
                step()
        stream = eager_stream
        run_step = graph.replay
        for _ in range(2):
            run_step()
        torch.cuda.synchronize()
    # timed region: exactly K steps, each between its own event pair, nothing else on the stream
    ms_per_step, ms_mean = time_steps(torch, run_step, stream, args.steps)
    other_ms = None
    if headline and not args.graph and not args.no_other_form:
        other = step_fused if args.separate_calls else step_three
        for _ in range(2):
            other()
        other_ms, _ = time_steps(torch, other, stream, args.steps)
    # per-kernel pass: the same K steps again with a HIP event pair around every launch, on the stream it is launched
    # on, and with the helper streams off so that no two kernels overlap and each duration is that kernel's alone.
    # The event pairs cost about a tenth of a step, so they stay out of the region above.
    prof, ms_per_step_events = {}, None
    if not args.no_kernel_events:
        ctx.set_helper_streams(False)
        ctx.profile_enable(True)
        _, ms_per_step_events = time_steps(torch, step, stream, args.steps)
        prof = ctx.profile_read()
        ctx.profile_enable(False)
        ctx.set_helper_streams(os.environ.get("REVFFN_NO_STREAMS") is None)

    # the family with the most time in the per-kernel pass goes into the `roofline` object
    dom = max(prof, key=lambda k: prof[k]["ms"]) if prof else None
    roofline = None
    if dom:
        p = prof[dom]
        roofline = family_roofline(p)
        roofline.update({"kernel": dom, "launches_per_step": p["launches"] / args.steps,
                         "avg_launch_us": p["ms"] / p["launches"] * 1e3,
                         "share_of_step": p["ms"] / args.steps / ms_per_step_events,
                         "ms_per_step_kernel_pass": ms_per_step_events,
                         "traffic": measured_traffic(wl.name, dom)})
    kernels = {}
    for k, v in prof.items():
        r = family_roofline(v)
        kernels[k] = {"ms_per_step": round(v["ms"] / args.steps, 5), "launches_per_step": v["launches"] / args.steps,
                      "tflops": round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2),
                      "gbs": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1),
                      "bound": r["bound"], "frac": round(r["frac"], 4)}
        t = measured_traffic(wl.name, k) if headline else None
        if t is not None:
            kernels[k]["traffic"] = t
    launches = sum(v["launches"] for v in prof.values()) / args.steps if prof else None
    if not headline:
        out = {"ms_per_step": ms_per_step, "tokens_per_s": wl.T / (ms_per_step * 1e-3), "steps": args.steps,
               "launches_per_step": launches, "setup_s": round(t_setup, 1),
               "kernels": {k: {"ms_per_step": v["ms_per_step"], "bound": v["bound"], "frac": v["frac"]}
                           for k, v in kernels.items() if v["ms_per_step"] >= 0.02}}
        ctx.close()
        return out

    calls = "forward+inverse+backward" if args.separate_calls else "forward+inverse_backward"
    out = {
        "metric": "RevFFN block fwd+inverse+bwd tokens/s at Qwen1.5-MoE shape",
        "value": wl.T / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "ms_per_step_mean": ms_mean,
        "timing": "median of the K steps, each between its own HIP event pair",
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: 1 RevFFN block, d={wl.d_model}, {wl.n_heads} heads x {wl.head_dim}, "
                               f"{wl.n_experts} experts top-{wl.top_k} I={wl.d_expert}, shared {wl.d_shared}, "
                               f"B={wl.B} S={wl.S}, weights N(0,0.02) inputs N(0,1) seed {wl.seed}",
                   "n_inv_iters": args.inv_iters, "residual_streams": "f32" if args.fp32_streams else wl.dtype, "launch": "HIP graph replay" if args.graph else "eager", "block": "symmetric comparison block" if args.symmetric else "RevFFN (Eq. 1-2)", "weight_gradients": "f32" if args.fp32_grads else wl.dtype, "trained": args.train, "calls": calls, "setup_s": round(t_setup, 1)},
        "roofline": roofline, "kernels": kernels, "launches_per_step": launches, "csrc_sha16": csrc_hash(),
    }
    if headline and not args.no_merged and not args.symmetric:
        # passes that need no gradients (static weights): adapters multiplied into the pre-trained weights once
        Md = Hn.alloc_merged(wl)
        mstruct = R.binding._m(Md)
        merge = lambda: R.revffn_merge_adapters(ctx, wstruct, mstruct, stream)
        fwd_u = lambda: R.revffn_forward(ctx, wstruct, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h, stream)
        inv_u = lambda: R.revffn_inverse(ctx, wstruct, y1d, y2d, r1d, r2d, wl.B, wl.S, wl.h, None, stream)
        fwd_m = lambda: R.revffn_forward_merged(ctx, wstruct, mstruct, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h, stream)
        inv_m = lambda: R.revffn_inverse_merged(ctx, wstruct, mstruct, y1d, y2d, r1d, r2d, wl.B, wl.S, wl.h, None, stream)
        rec = {}
        for name, fn, k in (("merge_ms", merge, 3), ("forward_ms", fwd_u, args.steps), ("forward_merged_ms", fwd_m, args.steps),
                            ("inverse_ms", inv_u, args.steps), ("inverse_merged_ms", inv_m, args.steps)):
            for _ in range(2):
                fn()
            rec[name] = round(time_steps(torch, fn, stream, k)[0], 4)
        rec["note"] = ("section 3.2 with static weights: W.P_up and P_dn.W formed once by merge (merge_ms), then forward and "
                       "inverse without adapter GEMMs; not part of `value`")
        out["merged_adapters"] = rec
        del Md
    if other_ms is not None:
        # both call forms: the fused sweep step (MoE half evaluated once) and the literal three calls
        out["three_call_ms_per_step" if not args.separate_calls else "fused_ms_per_step"] = other_ms
    if not args.no_cpu_baseline:
        idx = torch.empty((wl.T, wl.top_k), dtype=torch.int32, device="cuda")
        R.revffn_forward(ctx, wstruct, x1d, x2d, y1d, y2d, wl.B, wl.S, wl.h, stream)
        R.revffn_get_routing(ctx, idx)
        torch.cuda.synchronize()
        idx_o, ties = routing_report(wl, W32, Hn.download(y1d))
        out["routing"] = {"tokens": wl.T, "ties": ties, "flips": int((idx.cpu().numpy() != idx_o).any(axis=-1).sum()),
                          "note": "near-ties (margin <= 1e-3 in the oracle's fp64 logits) and GPU-vs-oracle selection "
                                  "differences of the timed workload"}
        out["cpu_baseline"] = cpu_baseline(wl, W32, x1, x2, dy1, dy2, args.inv_iters, args.symmetric)
    ctx.close()
    return out


def gemm_sweep():
    """One dense GEMM kernel (128x128 tiles) at growing k: a single tile, and 2048 x 2048 outputs (one tile per CU).
    The k = 64 rows are the fixed cost of a launch in a stream; the slope is the time of one k-step."""
    import torch
    import paper_2512_20920_amd as R
    rows = []
    for (M, N) in ((128, 128), (2048, 2048)):
        for K in (64, 256, 1024, 2048, 4096, 8192):
            a = torch.randn((M, K), device="cuda").bfloat16()
            b = torch.randn((N, K), device="cuda").bfloat16()
            c = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
            st = torch.cuda.current_stream()
            f = lambda: R.revffn_op_gemm(1, 2 + 256 * 2, a, b, c, M, N, K, K, K, N, False, False, False, st)
            for _ in range(3):
                f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(100):
                f()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 10.0
            rows.append({"M": M, "N": N, "K": K, "us_per_launch": round(us, 2), "tflops": round(2.0 * M * N * K / us / 1e6, 1)})
    print(json.dumps({"gemm_sweep": "C[M,N] = A[M,K] B[N,K]^T, bf16, 128x128 tiles, 100 launches back to back on one stream",
                      "rows": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="qwen_b4s512")
    ap.add_argument("--inv-iters", type=int, default=1, help="fixed-point iterations of the inverse (paper: 1)")
    ap.add_argument("--inv-tol", type=float, default=0.0,
                    help="stack workloads: > 0 = iterate each inverse until successive iterates differ by at most this "
                         "(decided on the device), at most --inv-max-iters times")
    ap.add_argument("--inv-max-iters", type=int, default=8)
    ap.add_argument("--inv-block", type=int, default=0,
                    help="with --inv-tol: positions per block of the stopping rule (0 = the whole call stops together)")
    ap.add_argument("--train", choices=["all", "stage1", "stage2"], default="all",
                    help="which weight gradients are asked for (the others are NULL and their GEMMs skipped): all; "
                         "stage1 = the four projection adapters only; stage2 = everything but the router (paper section 3.3)")
    ap.add_argument("--graph", action="store_true",
                    help="single-block workloads: capture one step into a HIP graph and time K replays of it")
    ap.add_argument("--fp32-grads", action="store_true", help="float32 weight-gradient buffers (dtype otherwise)")
    ap.add_argument("--symmetric", action="store_true",
                    help="the symmetric comparison block (queries from stream 2 too; closed-form inverse) instead of Eq. 1")
    ap.add_argument("--fp32-streams", action="store_true",
                    help="keep the residual streams x1, x2, y1, y2 in float32 (weights, activations, gradients stay bf16)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stored", action="store_true",
                    help="stack workloads: the non-reversible comparison (activations of every block kept, "
                         "revffn_backward_stored) instead of the reconstructing sweep")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three plain 256 MiB device-to-device copies (the known-size reference for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters) and exit")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="skip the second pass with per-launch HIP events (no roofline object)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="time revffn_inverse + revffn_backward as two calls (MoE half evaluated twice) as the headline "
                         "instead of revffn_inverse_backward (the other form is reported beside it either way)")
    ap.add_argument("--no-other-form", action="store_true",
                    help="skip the pass that times the other call form (used under the profiler, so that every step of "
                         "the run launches the same kernels)")
    ap.add_argument("--gemm-sweep", action="store_true",
                    help="time one dense GEMM kernel at growing k (launch floor and time per k-step) and exit")
    ap.add_argument("--no-merged", action="store_true", help="skip the forward/inverse timings with pre-merged adapters")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="headline workload only: skip the compact records of the skewed-routing and long-sequence workloads")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    if args.copy_calibration:
        a = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        a.fill_(1)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": a.numel(), "copies": 3}))
        return
    if args.gemm_sweep:
        return gemm_sweep()
    wl = synth.WORKLOADS[args.workload]
    if wl.n_blocks > 1:
        return bench_stack(args, wl)
    out = bench_block(args, wl, headline=True)
    if args.workload == "qwen_b4s512" and not args.no_other_workloads and not args.graph:
        # the other single-block workloads, compact (same step, same timing rule), so that one run records them
        others = {}
        for name in ("qwen_zipf_b2s2048", "qwen_b1s8192"):
            torch.cuda.empty_cache()
            others[name] = bench_block(args, synth.WORKLOADS[name], headline=False)
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
