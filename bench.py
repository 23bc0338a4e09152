#!/usr/bin/env python3
"""Benchmark of the mixed-precision MoE layer on one MI355X.

A step is one pass of the whole hot path over one batch: dx_route (top-k,
routing weights, permutation, and the hotness counters, which the context is
configured to update inside the routing kernel) -> dx_moe_forward for one
30B-shaped MoE layer at decode batch 32 (workload C2).  Steps rotate over `--layers` independent layers'
weights (default 48, the model's depth, ~26 GB) so that no step finds its
expert weights in the 256 MB last-level cache.  Each layer's bf16 resident set
is what the budget rule selects from a warm-up window of router traces.

Prints one JSON line: MoE-layer tokens/s, the roofline record of the dominant
kernel (gate/up + SwiGLU, timed with HIP events on the compute stream in a
second pass over the same steps), and the CPU oracle timed on one layer call.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="C2", choices=["C2", "C3", "C4", "C5"],
                    help="C2: decode T=32 (the headline metric); C3: the same layer in prefill, T=4096; "
                         "C4: decode T=32 on the 512-expert, top-10 layer shape with a shared expert; "
                         "C5: a decode stack whose hot set drifts, with live promotions and demotions")
    ap.add_argument("--layers", type=int, default=None, help="independent weight sets to rotate over")
    ap.add_argument("--window", type=int, default=None, help="routing-only warm-up steps per layer for hotness")
    ap.add_argument("--pair", default="bf16-int4", choices=["bf16-int4", "int4-int2"],
                    help="precision pair of the C2/C3 layer: high tier for the resident experts, low tier for the rest")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="time the C2/C3 layer shape at T = 1, 2, 4, ... 8192 tokens per step (one JSON line)")
    ap.add_argument("--seed", type=int, default=0)
    # C5 schedule (defaults: the configuration as stated -- 48 layers, 256-step window, the Zipf permutation
    # re-drawn every 256 steps, 2048 steps, windowed counts (alpha = 0) and plain top-n)
    ap.add_argument("--redraw", type=int, default=256, help="C5: steps between re-draws of the Zipf permutation")
    ap.add_argument("--alpha", type=float, default=0.0, help="C5: EMA factor of the hotness score, 0 <= alpha < 1")
    ap.add_argument("--margin", type=float, default=0.0, help="C5: hysteresis margin in counts (0: plain top-n)")
    ap.add_argument("--issue-per-step", type=int, default=32, help="C5: transitions issued per step at most")
    ap.add_argument("--max-inflight", type=int, default=64, help="C5: transitions between issue and publication at most")
    ap.add_argument("--spare", type=int, default=64, help="C5: spare blocks per pool (the transient room of in-flight transitions)")
    ap.add_argument("--banks", type=int, default=8, help="C5: pinned host master banks, shared by layer mod banks")
    ap.add_argument("--budget-gib", type=float, default=40.0, help="C4: expert-weight budget of the whole stack")
    return ap.parse_args()


def run_c5(args):
    """Decode stack under hot-set drift, as the configuration states it: 48 30B-shaped layers, the Zipf
    permutation re-drawn every 256 steps, a 256-step hotness window, 2048 steps, windowed counts and
    plain top-n (flags change each of these).  Every step runs route + forward of all layers and then one
    worker step of the transition queue; at each window end the scores pick the next resident sets.
    Reports stack tokens/s over all steps, per-step time percentiles against a run without drift, the
    migration traffic, and how long each re-draw took to be fully published.  The CPU leg replays
    sampled (step, layer) calls with the format map the library reported for them."""
    import numpy as np
    import torch

    from paper_2511_15015_amd import binding as B
    from paper_2511_15015_amd import layer as LY
    from paper_2511_15015_amd import stack as ST
    from paper_2511_15015_amd import workloads as W

    torch.cuda.set_device(0)
    wl = W.WORKLOADS["C5"]
    L, T, E, k, d, f, n = args.layers, wl.T, wl.E, wl.k, wl.d, wl.f, wl.n_hi
    window, steps, redraw = args.window, args.steps, args.redraw
    alpha_q16 = int(round(args.alpha * 65536))
    margin_q16 = int(round(args.margin * 65536))
    n_epochs = (steps + redraw - 1) // redraw if redraw else 1
    say = lambda m: print(f"bench C5: {m}", file=sys.stderr, flush=True)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        stk = ST.DriftStack(wl, L, args.seed, window, alpha_q16=alpha_q16, banks=args.banks, spare=args.spare,
                            max_inflight=args.max_inflight,
                            n_epochs=n_epochs, stream=stream, progress=say)
        kw = dict(margin_q16=margin_q16, issue_per_step=args.issue_per_step)
        say("warm-up run (no drift): reaches the resident sets of the first permutation")
        stk.run(2 * window, 0, time_steps=False, **kw)
        say("steady run (no drift)")
        steady, _ = stk.run(min(steps, 2 * window), 0, **kw)
        # sampled calls for the replay: layers {0, L/2 - 1, L - 1} at the first step, around every window
        # boundary and at the last step
        sl = sorted({0, max(L // 2 - 1, 0), L - 1})
        ss = sorted({0, steps - 1} | {w * window + o for w in range(1, steps // window + 1) for o in (-1, 0, 1)
                                      if 0 <= w * window + o < steps})
        say(f"drift run: {steps} steps, re-draw every {redraw}")
        drift, kept = stk.run(steps, redraw, samples={(s_, l_) for s_ in ss for l_ in sl}, **kw)
        budget_ok = drift["peak_reserved_bytes"] <= stk.budget_cap()
    out = {
        "metric": "MoE-stack tokens/s (decode B=32) under hot-set drift with live promotion/demotion",
        "value": T * drift["steps"] / drift["wall_s"], "unit": "tokens/s", "n_gpus": 1, "steps": drift["steps"],
        "warmup": 2 * window, "ms_per_step": drift["wall_s"] * 1e3 / drift["steps"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"C5: {L} 30B-A3B-shaped MoE layers per step, decode T={T}, Zipf(s={wl.zipf_s}) permutation "
                               f"re-drawn every {redraw} steps, {window}-step hotness window, EMA alpha {args.alpha:g}, "
                               f"margin {args.margin:g} counts, {n} bf16 experts per layer, at most {args.max_inflight} "
                               f"transitions in flight, {args.issue_per_step} issued per step, {args.spare} spare blocks per pool; pinned bf16 masters as "
                               f"{stk.banks} banks shared by layer mod {stk.banks}",
                   "step": "route + forward of every layer (one dx_route_forward each), stream synchronize, then one "
                           "dx_transitions_pump; dx_window_end + dx_select_resident + queueing at every window end"},
        "drift": drift, "steady": steady, "budget_respected": bool(budget_ok),
        "layer_us": drift["wall_s"] * 1e6 / drift["steps"] / L,
    }
    if not args.no_cpu_baseline:
        # the oracle replays the kept calls with the format map each of them ran under
        from oracle import dxo
        t0 = time.perf_counter()
        worst, n_checked = 0.0, 0
        cache = {}
        for smp in kept:
            if time.perf_counter() - t0 > 40.0:
                break
            layer, b, ep = smp["layer"], smp["batch"], smp["epoch"]
            x, lg = stk.x_bits[layer][b], stk.logits_host[ep][layer][b]
            ids, w, counts, offsets, perm = dxo.route(lg, k)
            assert np.array_equal(smp["ids"].cpu().numpy(), ids) and np.array_equal(smp["perm"].cpu().numpy(), perm)
            versions, filler = [None] * E, None
            for e in np.flatnonzero(counts > 0):
                e = int(e)
                key = (layer % stk.banks, e, int(smp["formats"][e]))
                if key not in cache:
                    m = stk.master_bits(layer, e)
                    cache[key] = (dxo.ExpertVersion.bf16(*m) if smp["formats"][e] == B.DX_FMT_BF16
                                  else dxo.ExpertVersion.int4_from_master(*m, wl.group))
                versions[e] = filler = cache[key]
            versions = [v if v is not None else filler for v in versions]
            y_ref = dxo.moe_forward(versions, d, f, wl.group, x, ids, w)
            yg = W.bf16_bits_to_f32(LY.device_to_bits(smp["y"])).astype(np.float64)
            worst = max(worst, float(np.linalg.norm(yg - y_ref) / np.linalg.norm(y_ref)))
            n_checked += 1
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n_checked * T / dt / L, "unit": "tokens/s", "cores": dxo.threads(), "kind": "oracle",
                               "sample": f"{n_checked} sampled layer calls of the drift run (layers {sl}, first step, every "
                                         f"window boundary -1/0/+1, last step) replayed with the reported format maps in "
                                         f"{dt:.1f} s, incl. quantizing the int4 versions; per-layer rate divided by {L} layers"}
        out["parity_max_rel_l2_sampled_calls"] = worst
        out["parity_sampled_calls"] = n_checked
    stk.close()
    print(json.dumps(out))


def run_sweep(args):
    """Tokens per step from 1 to 8192 on the 30B-shaped layer (the style of a prompt-length sweep): the
    same route + forward step as the headline benchmark, rotating over 8 layers' weights."""
    import dataclasses

    import numpy as np
    import torch

    from paper_2511_15015_amd import binding as B
    from paper_2511_15015_amd import layer as LY
    from paper_2511_15015_amd import workloads as W

    torch.cuda.set_device(0)
    base = W.WORKLOADS["C2"]
    L, E, k, d, f, t_max = 8, base.E, base.k, base.d, base.f, 8192
    stream = torch.cuda.Stream()
    rows = []
    with torch.cuda.stream(stream):
        ctx = B.Context(L=L, E=E, d=d, f=f, top_k=k, group=base.group, max_tokens=t_max, route_updates_hotness=True,
                        stream=stream.cuda_stream)
        rb = LY.RoutingBuffers(t_max, E, k)
        layers = []
        for layer in range(L):
            # resident set: the hottest experts of the layer's Zipf permutation (ranks 1..n_hi)
            bias = W.zipf_bias(E, base.zipf_s, args.seed, base.config_id, layer)
            resident = np.argsort(-bias, kind="stable")[:base.n_hi]
            wg, wu, wd = W.device_masters(base, args.seed, layer)
            layers.append(LY.LayerWeights(ctx, layer, wg, wu, wd, resident, base.group, keep_masters=False))
            del wg, wu, wd
        y = torch.empty((t_max, d), dtype=torch.bfloat16, device="cuda")
        lib, h = ctx.lib, ctx.h
        p_ids, p_w, p_counts, p_off, p_perm = (t.data_ptr() for t in (rb.ids, rb.w, rb.counts, rb.offsets, rb.perm))
        T = 1
        while T <= t_max:
            wl = dataclasses.replace(base, T=T)
            xs, lgs = [], []
            for layer in range(L):
                x, lg = W.layer_inputs(wl, args.seed, layer, step=0)
                xs.append(LY.bits_to_device(x))
                lgs.append(torch.from_numpy(lg).cuda())

            def step_fn(i):
                layer = i % L
                if lib.dx_route_forward(h, layer, None, lgs[layer].data_ptr(), xs[layer].data_ptr(), T,
                                        p_ids, p_w, p_counts, p_off, p_perm, y.data_ptr()):
                    raise RuntimeError(lib.dx_last_error(h).decode())

            steps = 240 if T <= 256 else 48
            for i in range(L):
                step_fn(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                step_fn(i)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            row = {"T": T, "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3)}
            if T <= 256:
                # the same L calls recorded once into a HIP graph and replayed: the device's own time per
                # call, where the host's three launches per call are the longer part (the smallest batches)
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for i in range(L):
                        step_fn(i)
                g.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps // L):
                    g.replay()
                torch.cuda.synchronize()
                row["ms_per_step_graph"] = (time.perf_counter() - t0) * 1e3 / (steps // L * L)
                del g
            rows.append(row)
            T *= 2
    ctx.close()
    at32 = next(r for r in rows if r["T"] == 32)
    print(json.dumps({
        "metric": "MoE-layer tokens/s against tokens per step", "value": at32["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": 240, "warmup": L, "ms_per_step": at32["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"30B-A3B-shaped MoE layer (d={d}, f={f}, E={E}, top-{k}, Zipf(s={base.zipf_s}) routing, "
                               f"{base.n_hi} bf16 + {E - base.n_hi} int4-g{base.group} experts), T from 1 to {t_max}, "
                               f"rotating over {L} layers' weights; value and ms_per_step are the T=32 row",
                   "step": "dx_route_forward (route + forward) of one layer"},
        "sweep": rows}))


def main():
    args = parse()
    if args.sweep:
        if args.gpus != 1:
            print("bench.py: this build runs on one GPU only; --gpus must be 1", file=sys.stderr)
            sys.exit(2)
        return run_sweep(args)
    defaults = {"C2": dict(steps=960, warmup=96, layers=48, window=64),
                "C3": dict(steps=48, warmup=8, layers=4, window=2),
                "C4": dict(steps=40, warmup=4, layers=48, window=16),
                "C5": dict(steps=2048, warmup=0, layers=48, window=256)}[args.workload]
    for key, val in defaults.items():
        if getattr(args, key) is None:
            setattr(args, key, val)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one process, one MI355X); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2511_15015_amd import binding as B
    from paper_2511_15015_amd import layer as LY
    from paper_2511_15015_amd import stack as ST
    from paper_2511_15015_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    if args.workload == "C5":
        return run_c5(args)
    torch.cuda.set_device(0)
    wl = W.WORKLOADS[args.workload]
    L, T, E, k, d, f = args.layers, wl.T, wl.E, wl.k, wl.d, wl.f
    seed = args.seed
    stacked = args.workload == "C4"          # a step is the whole stack: T / time of all L layers
    quant_pair = args.pair == "int4-int2"
    hi_fmt = B.DX_FMT_INT4G if quant_pair else B.DX_FMT_BF16
    b_hi = B.dx_expert_bytes(d, f, wl.group, hi_fmt)
    b_lo = B.dx_expert_bytes(d, f, wl.group, hi_fmt + 1)
    layer_budget = wl.n_hi * b_hi + (E - wl.n_hi) * b_lo       # 535560192 B for the bf16 / int4 pair
    b_sh = B.dx_expert_bytes(d, wl.shared_f, wl.group, B.DX_FMT_BF16) if wl.shared_f else 0
    checked_layers = sorted({0, max(L // 2 - 1, 0), L - 1}) if stacked else [0]
    say = lambda m: print(f"bench {args.workload}: {m}", file=sys.stderr, flush=True)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        if stacked:
            # one context for the whole stack, the byte budget of the configuration, the budget rule and
            # dx_select_resident per layer
            stack_budget = int(args.budget_gib * 2 ** 30)
            stk = ST.StaticStack(wl, L, seed, stack_budget, args.window, stream=stream,
                                 keep_masters_of=() if args.no_cpu_baseline else checked_layers, progress=say)
            ctx, rb, y, xs, lgs, layers, resident, shared = stk.ctx, stk.rb, stk.y, stk.xs, stk.lgs, stk.layers, \
                stk.resident, stk.shared
            n_per_layer = sorted({len(r) for r in resident})
            assert stk.bytes_held() <= stack_budget
            masters_of = lambda layer: stk.masters[layer]
        else:
            ctx = B.Context(L=L, E=E, d=d, f=f, top_k=k, group=wl.group, max_tokens=T,
                            window_steps=args.window, budget_bytes=L * (layer_budget + b_sh), shared_f=wl.shared_f,
                            route_updates_hotness=True, stream=stream.cuda_stream, hi_fmt=hi_fmt)
            rb = LY.RoutingBuffers(T, E, k)
            # inputs of every layer: the measured batch plus the warm-up window's router traces
            xs, lgs = [], []
            for layer in range(L):
                x, lg = W.layer_inputs(wl, seed, layer, step=0)
                xs.append(LY.bits_to_device(x))
                lgs.append(torch.from_numpy(lg).cuda())
            wr = [W.router_matrix(wl, seed, layer) for layer in range(L)]
            for step in range(1, args.window + 1):
                for layer in range(L):
                    xw = W.activations(wl, seed, layer, step)
                    lg = torch.from_numpy(W.router_logits(wl, xw, wr[layer], seed, layer)).cuda()
                    rb.route(ctx, layer, lg)          # also counts the selections (route_updates_hotness)
            ctx.dx_window_end()
            resident = [ctx.dx_select_resident(layer, layer_budget) for layer in range(L)]
            assert all(len(r) == wl.n_hi for r in resident), [len(r) for r in resident]
            n_per_layer = [wl.n_hi]
            # weights: draw each layer's masters on the device, keep bf16 for the resident set, int4 for the rest
            layers, shared = [], []
            for layer in range(L):
                if wl.shared_f:   # the always-resident bf16 shared expert of the layer
                    shared.append(ST.shared_expert_weights(wl, layer))
                    ctx.dx_swap_handle(layer, E, B.make_handle(B.DX_FMT_BF16, *shared[layer]))
                wg, wu, wd = W.device_masters(wl, seed, layer)
                if quant_pair:
                    layers.append(LY.QuantPairLayerWeights(ctx, layer, wg, wu, wd, resident[layer], wl.group))
                else:
                    layers.append(LY.LayerWeights(ctx, layer, wg, wu, wd, resident[layer], wl.group, keep_masters=False))
                del wg, wu, wd
            y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
            masters_of = lambda layer: W.device_masters(wl, seed, layer)
        stream.synchronize()

        # argument tuples resolved once: the timed loop is one C call per layer
        lib, h = ctx.lib, ctx.h
        p_ids, p_w, p_counts, p_off, p_perm = (t.data_ptr() for t in (rb.ids, rb.w, rb.counts, rb.offsets, rb.perm))
        route_args = [(h, layer, lgs[layer].data_ptr(), T, p_ids, p_w, p_counts, p_off, p_perm) for layer in range(L)]
        fwd_args = [(h, layer, None, xs[layer].data_ptr(), T, p_ids, p_w, p_off, p_perm, y.data_ptr())
                    for layer in range(L)]
        step_args = [(h, layer, None, lgs[layer].data_ptr(), xs[layer].data_ptr(), T, p_ids, p_w, p_counts, p_off,
                      p_perm, y.data_ptr()) for layer in range(L)]
        separate = os.environ.get("DX_BENCH_SEPARATE_CALLS") == "1"

        def layer_call(layer):
            if separate:
                rc = lib.dx_route(*route_args[layer]) or lib.dx_moe_forward(*fwd_args[layer])
            else:   # the same two steps as one call (decode batches route inside the gate/up kernel)
                rc = lib.dx_route_forward(*step_args[layer])
            if rc:
                raise RuntimeError(lib.dx_last_error(h).decode())

        def step_fn(i):
            if stacked:
                for layer in range(L):
                    layer_call(layer)
            else:
                layer_call(i % L)

        calls_per_step = L if stacked else 1
        for i in range(args.warmup):
            step_fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_fn(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps

        # algorithmic work per layer call, from the routing each layer's batch produces
        alg_bytes = alg_flops = step_bytes = 0.0
        for layer in range(L):
            layer_call(layer)
            counts = rb.counts.cpu().numpy()
            act = counts > 0
            hi = layers[layer].is_hi
            n_hi_act, n_lo_act = float((act & hi).sum()), float((act & ~hi).sum())
            # decode, gate/up launch: activated experts' gate+up bytes in their stored format + the token rows
            alg_bytes += n_hi_act * (2 * b_hi // 3) + n_lo_act * (2 * b_lo // 3) + T * d * 2 + 2 * b_sh // 3
            # decode, whole layer call: all three matrices of every activated expert (+ the shared expert) once,
            # x and the logits in, y and the routing arrays out
            step_bytes += n_hi_act * b_hi + n_lo_act * b_lo + b_sh + 2 * T * d * 2 + T * E * 4 + T * k * 12 + E * 8
            # prefill: the 256-row tile kernel multiplies the leading multiple of 256 rows of every bf16 and
            # every int4 segment (not of int2 segments): 2 * rows * d * 2f each
            big = hi if quant_pair else np.ones_like(hi)
            rows = (counts[big] // 256 * 256).sum()
            alg_flops += float(rows) * 2.0 * d * 2 * f
        alg_per_launch, flops_per_launch, step_bytes_per_call = alg_bytes / L, alg_flops / L, step_bytes / L

        # second pass over the same steps with HIP events around each forward kernel
        ctx.dx_set_profiling(True)
        for i in range(args.steps):
            step_fn(i)
        prof = ctx.dx_get_profile()
        ctx.dx_set_profiling(False)
        gate_up_us = prof["gate_up_ms"] * 1e3 / prof["calls"]

        # third pass: an event after every step, for the spread of the step times (each event adds a
        # little to the step it closes; the mean above is the wall clock without them)
        n_spread = min(args.steps, 480)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_spread + 1)]
        marks[0].record(stream)
        for i in range(n_spread):
            step_fn(i)
            marks[i + 1].record(stream)
        stream.synchronize()
        spread = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(n_spread)]) * 1e3

        # what a read-only kernel of the same launch shape and load policy reaches on this device: regions of the size
        # of the gate/up launch's bytes, rotating over 2.25 GiB so that nothing comes from the last-level cache
        probe_mib = 192
        probe_buf = torch.ones(12 * probe_mib << 20, dtype=torch.uint8, device="cuda")
        regions = [probe_buf.data_ptr() + (i * probe_mib << 20) for i in range(12)]
        for i in range(12):
            ctx.dx_probe_read(regions[i], probe_mib << 20)
        pe0, pe1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pe0.record(stream)
        for i in range(48):
            ctx.dx_probe_read(regions[i % 12], probe_mib << 20)
        pe1.record(stream)
        stream.synchronize()
        probe_gbs = 48 * (probe_mib << 20) / (pe0.elapsed_time(pe1) * 1e-3) / 1e9
        del probe_buf

    decode = args.workload in ("C2", "C4")
    shape_name = {"C2": "30B-A3B", "C3": "30B-A3B", "C4": "80B-A3B"}[args.workload]
    call_us = ms_per_step * 1e3 / calls_per_step
    if decode:
        achieved = alg_per_launch / (gate_up_us * 1e-6) / 1e9
        routed = not separate and T <= 64 and E <= 512 and k <= 16    # what dx_route_forward does with these shapes
        whole = step_bytes_per_call / (call_us * 1e-6) / 1e9
        roofline = {"bound": "hbm", "kernel": "k_stream_routed (routing prologue + gate/up)" if routed else "k_stream<gate/up>",
                    "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                    "algorithmic_bytes_per_launch": alg_per_launch, "avg_launch_us": gate_up_us,
                    "whole_step": {"algorithmic_bytes_per_layer_call": step_bytes_per_call, "us_per_layer_call": call_us,
                                   "achieved": whole, "frac": whole / HBM_PEAK_GBS,
                                   "note": "every activated expert's three matrices once in their stored format, the "
                                           "shared expert, x, logits, y and the routing arrays, over the wall-clock "
                                           "time of a layer call (all kernels and the gaps between them)"},
                    "read_probe_GBps": probe_gbs, "frac_of_read_probe": achieved / probe_gbs,
                    "read_probe": "dx_probe_read: 192 MiB per launch, read-only, same launch shape and load policy (whole lines, non-temporal), cold regions"}
    else:
        routed = False
        achieved = flops_per_launch / (gate_up_us * 1e-6) / 1e12
        step_flops = float(T * k) * 2.0 * d * 3 * f      # all routed pairs through gate, up and down
        roofline = {"bound": "mfma", "kernel": "k_big<gate/up>", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                    "algorithmic_flops_per_launch": flops_per_launch, "avg_launch_us": gate_up_us,
                    "note": "timed while the 128-row tile and streaming kernels of the same pass run beside it "
                            "on the side streams, as in the timed steps",
                    "whole_step_tflops": step_flops / (ms_per_step * 1e-3) / 1e12}
    # HBM traffic of the dominant kernel from the committed counter summary; the summary names the commit
    # whose kernels it was taken on, printed next to it (this tree may have moved on since)
    tpath = os.path.join(ROOT, "profiles", "k_stream_gate_up_C2_decode_pmc.txt" if decode
                         else "k_big_gate_up_C3_prefill_pmc.txt")
    if os.path.exists(tpath) and not quant_pair and args.workload != "C4":
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                roofline["traffic"] = float(line.split(":")[1])
            if line.startswith("kernels_at_commit:"):
                roofline["traffic_taken_at_commit"] = line.split(":")[1].strip()

    out = {
        "metric": ("MoE-stack tokens/s (decode B=32, all layers per step) + achieved HBM GB/s" if stacked else
                   "MoE-layer tokens/s (decode B=32) + achieved HBM GB/s") if decode
                  else "MoE-layer tokens/s (prefill T=4096) + MFMA utilisation",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {shape_name}-shaped MoE layer, {'decode' if decode else 'prefill'} T={T}, d={d}, f={f}, E={E}, top-{k}, "
                               + (f"one bf16 shared expert (f={wl.shared_f}), " if wl.shared_f else "") +
                               f"Zipf(s={wl.zipf_s}) routing, {'/'.join(str(n) for n in n_per_layer)} {'int4' if quant_pair else 'bf16'} + the rest "
                               f"{'int2' if quant_pair else 'int4'}-g{wl.group} experts per layer, "
                               + (f"stack of {L} layers in one context under a {args.budget_gib:g} GiB expert budget "
                                  f"({stk.bytes_held() / 2**30:.2f} GiB held), a step = all {L} layers"
                                  if stacked else f"rotating over {L} layers' weights"),
                   "step": "dx_route (top-k, permutation, hotness counters) + dx_moe_forward of one layer"
                           + (" as two calls" if separate else ", as one dx_route_forward call")
                           + ("" if separate or routed or not decode else
                              " (these shapes run the routing kernel and the forward kernels one after the other)")
                           + (f", for each of the {L} layers" if stacked else "")},
        "kernel_us": {"gate_up": gate_up_us, "down": prof["down_ms"] * 1e3 / prof["calls"],
                      "combine": prof["combine_ms"] * 1e3 / prof["calls"],
                      "empty_event_pair": prof["empty_ms"] * 1e3 / prof["calls"]},
        "step_us_with_an_event_per_step": {"p50": float(np.percentile(spread, 50)), "p99": float(np.percentile(spread, 99)),
                                           "mean": float(spread.mean()), "steps": int(n_spread)},
        "launches_per_step": ((3 if routed else 4) * calls_per_step) if decode else None,
        "roofline": roofline,
    }
    if stacked:
        out["us_per_layer"] = call_us

    if not args.no_cpu_baseline:
        # the oracle, as it stands, on full layer calls (layer 0's weights, all T tokens, route + forward,
        # a fresh seeded batch per call) on the host cores, for about 10 s; before that, the batches the GPU
        # was timed on, for the layers in `checked_layers`, against the output of the timed call
        # (dx_route_forward, or the two calls when they were timed)
        from oracle import dxo

        def oracle_versions(layer):
            wg, wu, wd = (LY.device_to_bits(m) for m in masters_of(layer))
            res = set(int(e) for e in resident[layer])
            sh = dxo.ExpertVersion.bf16(*(LY.device_to_bits(t) for t in shared[layer])) if wl.shared_f else None
            if quant_pair:
                return [dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) if e in res
                        else dxo.ExpertVersion.int2_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(E)], sh
            return [dxo.ExpertVersion.bf16(wg[e], wu[e], wd[e]) if e in res
                    else dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(E)], sh

        tokens0 = None if decode else np.arange(0, T, 2, dtype=np.int32)     # prefill: every second token
        worst, ids_ok, dt_prefill = 0.0, True, None
        versions0 = None
        for layer in checked_layers:
            versions, sh = oracle_versions(layer)
            if layer == 0:
                versions0, sh0 = versions, sh
            xb, lgb = W.layer_inputs(wl, seed, layer, step=0)
            with torch.cuda.stream(stream):
                layer_call(layer)
                stream.synchronize()
            t0 = time.perf_counter()
            ids, w, counts, offsets, perm = dxo.route(lgb, k)
            y_ref = dxo.moe_forward(versions, d, f, wl.group, xb, ids, w, tokens=tokens0, shared=sh, shared_f=wl.shared_f)
            dt_prefill = time.perf_counter() - t0
            yg = W.bf16_bits_to_f32(LY.device_to_bits(y)).astype(np.float64)
            if tokens0 is not None:
                yg = yg[tokens0]
            worst = max(worst, float(np.linalg.norm(yg - y_ref) / np.linalg.norm(y_ref)))
            ids_ok = ids_ok and bool(np.array_equal(rb.ids.cpu().numpy(), ids)) and \
                bool(np.array_equal(rb.perm.cpu().numpy(), perm))
            del versions
        if decode:
            batches = [W.layer_inputs(wl, seed, 0, step=i) for i in range(400)]
            calls = 0
            t0 = time.perf_counter()
            while calls < len(batches) and time.perf_counter() - t0 < 10.0:
                xb, lgb = batches[calls]
                ids, w, counts, offsets, perm = dxo.route(lgb, k)
                dxo.moe_forward(versions0, d, f, wl.group, xb, ids, w, shared=sh0, shared_f=wl.shared_f)
                calls += 1
            dt = time.perf_counter() - t0
            out["cpu_baseline"] = {"value": calls * T / dt / calls_per_step, "unit": "tokens/s", "cores": dxo.threads(),
                                   "kind": "oracle",
                                   "sample": f"{calls} full layer calls (layer 0's experts, all {T} tokens each, "
                                             f"route + forward) in {dt:.1f} s"
                                             + (f"; the stack rate is that per-layer rate divided by {L} layers "
                                                f"(extrapolated)" if stacked else "")}
        else:
            out["cpu_baseline"] = {"value": len(tokens0) / dt_prefill, "unit": "tokens/s", "cores": dxo.threads(), "kind": "oracle",
                                   "sample": f"routing of all {T} tokens + the layer output of {len(tokens0)} evenly "
                                             f"spaced tokens of one batch (layer 0's experts) in {dt_prefill:.1f} s"}
        out["parity_max_rel_l2"] = worst
        out["parity_ids_and_perm_exact"] = ids_ok
        out["parity_checked"] = {"layers": checked_layers, "path": "the timed call: " +
                                 ("dx_route + dx_moe_forward" if separate else "dx_route_forward")}
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
