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
    return ap.parse_args()


def run_c5(args):
    """Decode stack under hot-set drift (30B-shaped layers, Zipf permutation re-drawn every four
    windows, so that the transitions of one re-draw are through before the next): every step runs route + forward of all layers and then one worker step of the transition
    queue; at each window end the EMA scores pick the next resident sets.  Reports stack tokens/s over
    all steps, per-step time percentiles against a run of the same length without drift, and the
    migration traffic."""
    import numpy as np
    import torch

    from paper_2511_15015_amd import binding as B
    from paper_2511_15015_amd import layer as LY
    from paper_2511_15015_amd import workloads as W

    torch.cuda.set_device(0)
    wl = W.WORKLOADS["C5"]
    L, T, E, k, d, f, n = args.layers, wl.T, wl.E, wl.k, wl.d, wl.f, wl.n_hi
    window, n_windows, redraw, n_batches = args.window, args.steps // args.window, 4, 16
    b_hi = B.dx_expert_bytes(d, f, wl.group, B.DX_FMT_BF16)
    b_lo = B.dx_expert_bytes(d, f, wl.group, B.DX_FMT_INT4G)
    layer_budget, spare = n * b_hi + (E - n) * b_lo, 16
    stream = torch.cuda.Stream()
    results = {}
    with torch.cuda.stream(stream):
        ctx = B.Context(L=L, E=E, d=d, f=f, top_k=k, group=wl.group, max_tokens=T, window_steps=window,
                        alpha_q16=32768, budget_bytes=L * layer_budget, transient_bytes=spare * (b_hi + b_lo),
                        route_updates_hotness=True, stream=stream.cuda_stream)
        ctx.dx_pools_create(L * n + spare, L * (E - n) + spare)
        ctx.dx_transitions_limits(8)
        pinned = []
        for layer in range(L):
            dev = W.device_masters(wl, args.seed, layer)
            host = [torch.empty(m.shape, dtype=m.dtype).pin_memory() for m in dev]
            for h, m in zip(host, dev):
                h.copy_(m)
            pinned.append(host)
            for e in range(E):
                ctx.dx_expert_install(layer, e, B.DX_FMT_BF16 if e < n else B.DX_FMT_INT4G, *(m[e] for m in dev),
                                      src_on_device=True)
                ctx.dx_register_host_master(layer, e, *(h[e] for h in host))
            del dev
        rb = LY.RoutingBuffers(T, E, k)
        y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        n_epochs = (n_windows + redraw - 1) // redraw
        xs = [[None] * n_batches for _ in range(L)]
        lgs = [[[None] * n_batches for _ in range(L)] for _ in range(n_epochs)]
        for layer in range(L):
            for b in range(n_batches):
                xb = W.activations(wl, args.seed, layer, b)
                xs[layer][b] = LY.bits_to_device(xb)
                wr = W.router_matrix(wl, args.seed, layer)
                for ep in range(n_epochs):
                    lgs[ep][layer][b] = torch.from_numpy(W.router_logits(wl, xb, wr, args.seed, layer, ep)).cuda()
        lib, h = ctx.lib, ctx.h
        p_ids, p_w, p_counts, p_off, p_perm = (t.data_ptr() for t in (rb.ids, rb.w, rb.counts, rb.offsets, rb.perm))

        def run(drift):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n_windows * window + 1)]
            st0 = ctx.dx_get_stats()
            settle = []                      # steps from a re-draw until the queue and the migration stream are empty
            since_redraw, armed = None, False
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev[0].record(stream)
            step = 0
            for wdw in range(n_windows):
                ep = wdw // redraw if drift else 0
                if drift and wdw % redraw == 0 and wdw > 0:
                    since_redraw, armed = 0, False
                for s_ in range(window):
                    b = step % n_batches
                    for layer in range(L):
                        if lib.dx_route_forward(h, layer, None, lgs[ep][layer][b].data_ptr(), xs[layer][b].data_ptr(), T,
                                                p_ids, p_w, p_counts, p_off, p_perm, y.data_ptr()):
                            raise RuntimeError(lib.dx_last_error(h).decode())
                    step += 1
                    ev[step].record(stream)
                    stream.synchronize()       # a decode loop reads its tokens here; keeps host and GPU in step
                    issued, published, queued = ctx.dx_transitions_pump(4)
                    if since_redraw is not None:
                        since_redraw += 1
                        if armed and queued == 0 and ctx.dx_get_stats()["in_flight"] == 0:
                            settle.append(since_redraw)
                            since_redraw = None
                ctx.dx_window_end()
                for layer in range(L):
                    target = ctx.dx_select_resident_stable(layer, layer_budget, margin_q16=2 << 16)
                    pro, dem = ctx.dx_plan_transitions(layer, target)
                    ctx.dx_transitions_enqueue(layer, pro, dem)
                armed = True
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            ctx.dx_migrate_poll(wait=True)
            ms = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(len(ev) - 1)])
            st1 = ctx.dx_get_stats()
            return dict(wall_s=wall, steps=len(ms), p50_ms=float(np.percentile(ms, 50)), p99_ms=float(np.percentile(ms, 99)),
                        max_ms=float(ms.max()), mean_ms=float(ms.mean()),
                        promotions=st1["promotions_published"] - st0["promotions_published"],
                        demotions=st1["demotions_published"] - st0["demotions_published"],
                        h2d_bytes_per_step=(st1["h2d_bytes"] - st0["h2d_bytes"]) / len(ms),
                        quantize_bytes_per_step=(st1["quantize_read_bytes"] + st1["quantize_write_bytes"]
                                                 - st0["quantize_read_bytes"] - st0["quantize_write_bytes"]) / len(ms),
                        steps_to_settle_after_redraw=settle, peak_in_flight=st1["peak_in_flight"],
                        peak_reserved_bytes=st1["peak_reserved_bytes"])

        run(False)                                                    # warm-up: reaches the epoch-0 resident sets
        results["steady"] = run(False)
        results["drift"] = run(True)
        budget_ok = results["drift"]["peak_reserved_bytes"] <= L * layer_budget + spare * (b_hi + b_lo)
    ctx.close()
    dr = results["drift"]
    out = {
        "metric": "MoE-stack tokens/s (decode B=32) under hot-set drift with live promotion/demotion",
        "value": T * dr["steps"] / dr["wall_s"], "unit": "tokens/s", "n_gpus": 1, "steps": dr["steps"], "warmup": dr["steps"],
        "ms_per_step": dr["wall_s"] * 1e3 / dr["steps"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"C5: {L} 30B-A3B-shaped MoE layers per step (of the model's 48; pinned host masters "
                               f"for all of them are {48 * E * b_hi / 2**30:.0f} GiB), decode T={T}, Zipf(s={wl.zipf_s}) permutation "
                               f"re-drawn every {redraw} windows of {window} steps, EMA alpha 0.5, margin 2 counts, "
                               f"{n} bf16 experts per layer, at most 8 transitions in flight, 4 issued per step",
                   "step": "route + forward of every layer, stream synchronize, then one dx_transitions_pump"},
        "drift": dr, "steady": results["steady"], "budget_respected": bool(budget_ok),
    }
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
            rows.append({"T": T, "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3)})
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
                "C4": dict(steps=480, warmup=48, layers=16, window=16),
                "C5": dict(steps=512, warmup=0, layers=8, window=32)}[args.workload]
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
    quant_pair = args.pair == "int4-int2"
    hi_fmt = B.DX_FMT_INT4G if quant_pair else B.DX_FMT_BF16
    b_hi = B.dx_expert_bytes(d, f, wl.group, hi_fmt)
    b_lo = B.dx_expert_bytes(d, f, wl.group, hi_fmt + 1)
    layer_budget = wl.n_hi * b_hi + (E - wl.n_hi) * b_lo       # 535560192 B for the bf16 / int4 pair
    b_sh = B.dx_expert_bytes(d, wl.shared_f, wl.group, B.DX_FMT_BF16) if wl.shared_f else 0

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
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
        # weights: draw each layer's masters on the device, keep bf16 for the resident set, int4 for the rest
        layers, shared = [], []
        for layer in range(L):
            if wl.shared_f:   # the always-resident bf16 shared expert of the layer
                g = torch.Generator(device="cuda")
                g.manual_seed(1000 + layer)
                shared.append([(0.02 * torch.randn(s, generator=g, device="cuda")).to(torch.bfloat16)
                               for s in ((wl.shared_f, d), (wl.shared_f, d), (d, wl.shared_f))])
                ctx.dx_swap_handle(layer, E, B.make_handle(B.DX_FMT_BF16, *shared[layer]))
            wg, wu, wd = W.device_masters(wl, seed, layer)
            if quant_pair:
                layers.append(LY.QuantPairLayerWeights(ctx, layer, wg, wu, wd, resident[layer], wl.group))
            else:
                layers.append(LY.LayerWeights(ctx, layer, wg, wu, wd, resident[layer], wl.group, keep_masters=False))
            del wg, wu, wd
        y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        stream.synchronize()

        # argument tuples resolved once: the timed loop is two C calls per step
        lib, h = ctx.lib, ctx.h
        p_ids, p_w, p_counts, p_off, p_perm = (t.data_ptr() for t in (rb.ids, rb.w, rb.counts, rb.offsets, rb.perm))
        route_args = [(h, layer, lgs[layer].data_ptr(), T, p_ids, p_w, p_counts, p_off, p_perm) for layer in range(L)]
        fwd_args = [(h, layer, None, xs[layer].data_ptr(), T, p_ids, p_w, p_off, p_perm, y.data_ptr())
                    for layer in range(L)]

        step_args = [(h, layer, None, lgs[layer].data_ptr(), xs[layer].data_ptr(), T, p_ids, p_w, p_counts, p_off,
                      p_perm, y.data_ptr()) for layer in range(L)]
        separate = os.environ.get("DX_BENCH_SEPARATE_CALLS") == "1"

        def step_fn(i):
            layer = i % L
            if separate:
                rc = lib.dx_route(*route_args[layer]) or lib.dx_moe_forward(*fwd_args[layer])
            else:   # the same two steps as one call (decode batches route inside the gate/up kernel)
                rc = lib.dx_route_forward(*step_args[layer])
            if rc:
                raise RuntimeError(lib.dx_last_error(h).decode())

        for i in range(args.warmup):
            step_fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step_fn(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms_per_step = (t1 - t0) * 1e3 / args.steps

        # second pass over the same steps with HIP events around each forward kernel
        ctx.dx_set_profiling(True)
        alg_bytes = alg_flops = 0.0
        for i in range(args.steps):
            step_fn(i)
            if i < L:   # algorithmic work of the dominant (gate/up) launch for this layer's batch
                counts = rb.counts.cpu().numpy()
                act = counts > 0
                hi = layers[i % L].is_hi
                # decode: activated experts' gate+up bytes in their stored format + the token rows
                alg_bytes += float((act & hi).sum() * (2 * b_hi // 3) + (act & ~hi).sum() * (2 * b_lo // 3) + T * d * 2
                                   + 2 * b_sh // 3)
                # prefill: the 256-row tile kernel multiplies the leading multiple of 256 rows of every bf16
                # segment: 2 * rows * d * 2f each
                # (no bf16 experts in the int4 / int2 pair: there the 128-row tile kernel takes every segment above 32)
                rows = (counts[hi] // 256 * 256).sum() if not quant_pair else counts[counts > 32].sum()
                alg_flops += float(rows) * 2.0 * d * 2 * f
        prof = ctx.dx_get_profile()
        ctx.dx_set_profiling(False)
        n_alg = min(args.steps, L)
        alg_per_launch = alg_bytes / n_alg
        flops_per_launch = alg_flops / n_alg
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

        # what a plain read-only kernel of the same launch shape reaches on this device: regions of the size
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
    if decode:
        achieved = alg_per_launch / (gate_up_us * 1e-6) / 1e9
        routed = not separate and T <= 64 and E <= 128 and k <= 16    # what dx_route_forward does with these shapes
        roofline = {"bound": "hbm", "kernel": "k_stream_routed (routing prologue + gate/up)" if routed else "k_stream<gate/up>",
                    "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                    "algorithmic_bytes_per_launch": alg_per_launch, "avg_launch_us": gate_up_us,
                    "read_probe_GBps": probe_gbs, "frac_of_read_probe": achieved / probe_gbs,
                    "read_probe": "dx_probe_read: 192 MiB per launch, read-only, same launch shape, cold regions"}
    else:
        achieved = flops_per_launch / (gate_up_us * 1e-6) / 1e12
        step_flops = float(T * k) * 2.0 * d * 3 * f      # all routed pairs through gate, up and down
        roofline = {"bound": "mfma", "kernel": "k_tiled<gate/up>" if quant_pair else "k_big<gate/up>", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                    "algorithmic_flops_per_launch": flops_per_launch, "avg_launch_us": gate_up_us,
                    "note": "timed while the 128-row tile and streaming kernels of the same pass run beside it "
                            "on the side streams, as in the timed steps",
                    "whole_step_tflops": step_flops / (ms_per_step * 1e-3) / 1e12}
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "k_stream_gate_up_C2_decode_pmc.txt" if decode
                         else "k_big_gate_up_C3_prefill_pmc.txt")
    if os.path.exists(tpath) and not quant_pair and args.workload != "C4":
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
    roofline["traffic"] = traffic

    out = {
        "metric": "MoE-layer tokens/s (decode B=32) + achieved HBM GB/s" if decode
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
                               f"Zipf(s={wl.zipf_s}) routing, {wl.n_hi} {'int4' if quant_pair else 'bf16'} + {E - wl.n_hi} "
                               f"{'int2' if quant_pair else 'int4'}-g{wl.group} experts "
                               f"per layer, rotating over {L} layers' weights",
                   "step": "dx_route (top-k, permutation, hotness counters) + dx_moe_forward of one layer"
                           + (" as two calls" if separate else ", as one dx_route_forward call")
                           + ("" if separate or (T <= 64 and E <= 128 and k <= 16) else
                              " (these shapes run the routing kernel and the forward kernels one after the other)")},
        "kernel_us": {"gate_up": gate_up_us, "down": prof["down_ms"] * 1e3 / prof["calls"],
                      "combine": prof["combine_ms"] * 1e3 / prof["calls"],
                      "empty_event_pair": prof["empty_ms"] * 1e3 / prof["calls"]},
        "step_us_with_an_event_per_step": {"p50": float(np.percentile(spread, 50)), "p99": float(np.percentile(spread, 99)),
                                           "mean": float(spread.mean()), "steps": int(n_spread)},
        "launches_per_step": (3 if routed else 4) if decode else None,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        # the oracle, as it stands, on full layer calls (layer 0's weights, all T tokens, route + forward,
        # a fresh seeded batch per call) on the host cores, for about 10 s
        from oracle import dxo
        wg, wu, wd = (LY.device_to_bits(m) for m in W.device_masters(wl, seed, 0))
        res0 = set(int(e) for e in resident[0])
        sh0 = dxo.ExpertVersion.bf16(*(LY.device_to_bits(t) for t in shared[0])) if wl.shared_f else None
        if quant_pair:
            versions = [dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) if e in res0
                        else dxo.ExpertVersion.int2_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(E)]
        else:
            versions = [dxo.ExpertVersion.bf16(wg[e], wu[e], wd[e]) if e in res0
                        else dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(E)]
        if decode:
            batches = [W.layer_inputs(wl, seed, 0, step=i) for i in range(400)]
            calls, y_ref0, ids0 = 0, None, None
            t0 = time.perf_counter()
            while calls < len(batches) and time.perf_counter() - t0 < 10.0:
                xb, lgb = batches[calls]
                ids, w, counts, offsets, perm = dxo.route(lgb, k)
                y_ref = dxo.moe_forward(versions, d, f, wl.group, xb, ids, w, shared=sh0, shared_f=wl.shared_f)
                if calls == 0:
                    y_ref0, ids0 = y_ref, ids
                calls += 1
            dt = time.perf_counter() - t0
            tokens0 = None
            out["cpu_baseline"] = {"value": calls * T / dt, "unit": "tokens/s", "cores": dxo.threads(), "kind": "oracle",
                                   "sample": f"{calls} full layer calls (layer 0's experts, all {T} tokens each, "
                                             f"route + forward) in {dt:.1f} s"}
        else:
            xb, lgb = W.layer_inputs(wl, seed, 0, step=0)
            tokens0 = np.arange(0, T, 2, dtype=np.int32)                 # every second token of the batch
            t0 = time.perf_counter()
            ids0, w, counts, offsets, perm = dxo.route(lgb, k)
            y_ref0 = dxo.moe_forward(versions, d, f, wl.group, xb, ids0, w, tokens=tokens0, shared=sh0,
                                     shared_f=wl.shared_f)
            dt = time.perf_counter() - t0
            out["cpu_baseline"] = {"value": len(tokens0) / dt, "unit": "tokens/s", "cores": dxo.threads(), "kind": "oracle",
                                   "sample": f"routing of all {T} tokens + the layer output of {len(tokens0)} evenly "
                                             f"spaced tokens of one batch (layer 0's experts) in {dt:.1f} s"}
        # the first of those calls on the GPU, as a sanity check of the benchmarked path
        with torch.cuda.stream(stream):
            rb.route(ctx, 0, lgs[0])
            rb.forward(ctx, 0, xs[0], y)
            stream.synchronize()
        yg = W.bf16_bits_to_f32(LY.device_to_bits(y)).astype(np.float64)
        if tokens0 is not None:
            yg = yg[tokens0]
        out["parity_rel_l2_layer0"] = float(np.linalg.norm(yg - y_ref0) / np.linalg.norm(y_ref0))
        out["parity_ids_exact_layer0"] = bool(np.array_equal(rb.ids.cpu().numpy(), ids0))
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
