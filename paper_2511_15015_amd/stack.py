"""Caller-side set-up and driving loops of the two stack workloads.

Allocation, input staging and call sequencing only (PyTorch owns the memory,
the library's kernels do every step of the path); shared by ``bench.py`` and
the GPU tests so that both run the same schedule.

``StaticStack``: the 80B-shaped 48-layer decode stack under a byte budget for
the whole stack: one context, a warm-up window of router traces, the budget
rule and ``dx_select_resident`` per layer, then one ``dx_route_forward`` per
layer and step.

``DriftStack``: the 30B-shaped decode stack whose Zipf permutation is re-drawn
every ``redraw_steps`` steps: every expert lives in the context's pools, bf16
masters sit in pinned host memory, and between steps the transition queue
issues promotions (copies on the migration stream) and demotions (on-device
quantizer) and publishes what has completed.  The pinned masters are kept as
``banks`` banks shared by ``layer mod banks`` (48 layers of private masters
would be 54 GiB of pinned memory): every layer still has its own router, hot
set, pool blocks and transitions, and the bytes moved are unchanged.
"""
from __future__ import annotations

import time

import numpy as np
import torch

from . import binding as B
from . import layer as LY
from . import workloads as W


def shared_expert_weights(wl, layer: int, device="cuda"):
    """bf16 weights of the layer's always-resident shared expert, drawn on the device."""
    g = torch.Generator(device=device)
    g.manual_seed(1000 + layer)
    return [(0.02 * torch.randn(s, generator=g, device=device)).to(torch.bfloat16)
            for s in ((wl.shared_f, wl.d), (wl.shared_f, wl.d), (wl.d, wl.shared_f))]


class StaticStack:
    """L layers of one workload shape in one context, resident sets chosen per layer by the budget
    rule from a warm-up window of router traces.  ``keep_masters_of``: layers whose bf16 masters stay
    on the device (for a check against the CPU reference)."""

    def __init__(self, wl, L: int, seed: int, stack_budget: int, window: int, stream=None,
                 keep_masters_of=(), progress=None):
        self.wl, self.L, self.seed = wl, L, seed
        T, E, k, d, f = wl.T, wl.E, wl.k, wl.d, wl.f
        self.b_hi = B.dx_expert_bytes(d, f, wl.group, B.DX_FMT_BF16)
        self.b_lo = B.dx_expert_bytes(d, f, wl.group, B.DX_FMT_INT4G)
        self.b_sh = B.dx_expert_bytes(d, wl.shared_f, wl.group, B.DX_FMT_BF16) if wl.shared_f else 0
        self.stack_budget = stack_budget
        self.layer_budget = (stack_budget - L * self.b_sh) // L
        self.ctx = B.Context(L=L, E=E, d=d, f=f, top_k=k, group=wl.group, max_tokens=T, window_steps=window,
                             budget_bytes=stack_budget, shared_f=wl.shared_f, route_updates_hotness=True,
                             stream=stream.cuda_stream if stream is not None else None)
        self.rb = LY.RoutingBuffers(T, E, k)
        self.y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        self.x_bits, self.logits_host, self.xs, self.lgs = [], [], [], []
        for layer in range(L):
            x, lg = W.layer_inputs(wl, seed, layer, step=0)
            self.x_bits.append(x)
            self.logits_host.append(lg)
            self.xs.append(LY.bits_to_device(x))
            self.lgs.append(torch.from_numpy(lg).cuda())
        # warm-up window: routing only, the routing kernel counts the selections
        for layer in range(L):
            wr = W.router_matrix(wl, seed, layer)
            for step in range(1, window + 1):
                xw = W.activations(wl, seed, layer, step)
                lg = torch.from_numpy(W.router_logits(wl, xw, wr, seed, layer)).cuda()
                self.rb.route(self.ctx, layer, lg)
        self.scores = self.ctx.dx_window_end()
        self.resident = [self.ctx.dx_select_resident(layer, self.layer_budget) for layer in range(L)]
        self.layers, self.shared, self.masters = [], [], {}
        for layer in range(L):
            if progress and layer % 8 == 0:
                progress(f"materialising layer {layer} of {L}")
            if wl.shared_f:
                self.shared.append(shared_expert_weights(wl, layer))
                self.ctx.dx_swap_handle(layer, E, B.make_handle(B.DX_FMT_BF16, *self.shared[layer]))
            wg, wu, wd = W.device_masters(wl, seed, layer)
            keep = layer in keep_masters_of
            self.layers.append(LY.LayerWeights(self.ctx, layer, wg, wu, wd, self.resident[layer], wl.group,
                                               keep_masters=keep))
            if keep:
                self.masters[layer] = (wg, wu, wd)
            del wg, wu, wd
        lib, h = self.ctx.lib, self.ctx.h
        p = [t.data_ptr() for t in (self.rb.ids, self.rb.w, self.rb.counts, self.rb.offsets, self.rb.perm)]
        self._args = [(h, layer, None, self.lgs[layer].data_ptr(), self.xs[layer].data_ptr(), T, *p, self.y.data_ptr())
                      for layer in range(L)]
        self._lib = lib

    def layer_call(self, layer: int):
        if self._lib.dx_route_forward(*self._args[layer]):
            raise RuntimeError(self._lib.dx_last_error(self.ctx.h).decode())

    def step(self):
        for layer in range(self.L):
            self.layer_call(layer)

    def bytes_held(self) -> int:
        """Expert bytes the stack holds under the budget rule (routed experts + shared experts)."""
        return sum(len(r) * self.b_hi + (self.wl.E - len(r)) * self.b_lo + self.b_sh for r in self.resident)

    def close(self):
        self.ctx.close()


class DriftStack:
    """The drifting decode stack (see the module text).  ``run`` drives ``steps`` steps; ``samples`` is a
    set of (step, layer) at which the format map, the routing arrays and the layer output are kept for a
    replay by the CPU reference."""

    def __init__(self, wl, L: int, seed: int, window: int, alpha_q16: int = 0, banks: int = 8, spare: int = 16,
                 max_inflight: int = 32, n_batches: int = 16, n_epochs: int = 1, stream=None, progress=None):
        self.wl, self.L, self.seed, self.window = wl, L, seed, window
        T, E, k, d, f, n = wl.T, wl.E, wl.k, wl.d, wl.f, wl.n_hi
        self.banks = min(banks, L)
        self.b_hi = B.dx_expert_bytes(d, f, wl.group, B.DX_FMT_BF16)
        self.b_lo = B.dx_expert_bytes(d, f, wl.group, B.DX_FMT_INT4G)
        self.layer_budget = n * self.b_hi + (E - n) * self.b_lo
        self.spare = spare
        self.stream = stream
        self.ctx = B.Context(L=L, E=E, d=d, f=f, top_k=k, group=wl.group, max_tokens=T, window_steps=window,
                             alpha_q16=alpha_q16, budget_bytes=L * self.layer_budget,
                             transient_bytes=spare * (self.b_hi + self.b_lo), route_updates_hotness=True,
                             stream=stream.cuda_stream if stream is not None else None)
        self.ctx.dx_pools_create(L * n + spare, L * (E - n) + spare)
        self.ctx.dx_transitions_limits(max_inflight)
        # master banks: drawn on the device, copied once into pinned host memory
        self.pinned = []
        dev_banks = []
        for b in range(self.banks):
            if progress:
                progress(f"master bank {b} of {self.banks}")
            dev = W.device_masters(wl, seed, b)
            host = [torch.empty(m.shape, dtype=m.dtype).pin_memory() for m in dev]
            for hm, m in zip(host, dev):
                hm.copy_(m)
            self.pinned.append(host)
            dev_banks.append(dev)
        # initial state: experts 0 .. n-1 bf16 (the selection on all-zero scores), the others int4
        for layer in range(L):
            if progress and layer % 8 == 0:
                progress(f"installing layer {layer} of {L}")
            dev, host = dev_banks[layer % self.banks], self.pinned[layer % self.banks]
            for e in range(E):
                self.ctx.dx_expert_install(layer, e, B.DX_FMT_BF16 if e < n else B.DX_FMT_INT4G, *(m[e] for m in dev),
                                           src_on_device=True)
                self.ctx.dx_register_host_master(layer, e, *(hm[e] for hm in host))
        del dev_banks
        self.rb = LY.RoutingBuffers(T, E, k)
        self.y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        self.n_batches, self.n_epochs = n_batches, n_epochs
        self.x_bits = [[None] * n_batches for _ in range(L)]
        self.xs = [[None] * n_batches for _ in range(L)]
        self.logits_host = [[[None] * n_batches for _ in range(L)] for _ in range(n_epochs)]
        self.lgs = [[[None] * n_batches for _ in range(L)] for _ in range(n_epochs)]
        for layer in range(L):
            wr = W.router_matrix(wl, seed, layer)
            for b in range(n_batches):
                xb = W.activations(wl, seed, layer, b)
                self.x_bits[layer][b] = xb
                self.xs[layer][b] = LY.bits_to_device(xb)
                for ep in range(n_epochs):
                    lg = W.router_logits(wl, xb, wr, seed, layer, ep)
                    self.logits_host[ep][layer][b] = lg
                    self.lgs[ep][layer][b] = torch.from_numpy(lg).cuda()

    def master_bits(self, layer: int, e: int):
        """bf16 bit patterns of expert e's masters (gate, up, down) of `layer`, from the pinned bank."""
        return tuple(hm[e].view(torch.int16).numpy().view(np.uint16) for hm in self.pinned[layer % self.banks])

    def run(self, steps: int, redraw_steps: int = 0, margin_q16: int = 0, rank_slack: int = 0, issue_per_step: int = 16,
            samples=(), time_steps: bool = True, epoch0: int = 0):
        """Drives `steps` steps: per step one dx_route_forward per layer, a stream synchronisation (a decode
        loop reads its tokens there), one dx_transitions_pump; at every window end dx_window_end, the selection
        per layer and the candidates into the queue.  Epoch (which Zipf permutation the logits carry) =
        epoch0 + step // redraw_steps.  Returns the measurements and the kept samples."""
        ctx, lib, h, L, T = self.ctx, self.ctx.lib, self.ctx.h, self.L, self.wl.T
        rb, y = self.rb, self.y
        p = [t.data_ptr() for t in (rb.ids, rb.w, rb.counts, rb.offsets, rb.perm)]
        yp = y.data_ptr()
        stream = self.stream if self.stream is not None else torch.cuda.current_stream()
        samples = set(samples)
        kept = []
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)] if time_steps else None
        st0 = ctx.dx_get_stats()
        drain, since_enqueue = [], None  # steps from a window end until its transitions are all published
        hi_pairs = total_pairs = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if ev:
            ev[0].record(stream)
        for step in range(steps):
            ep = epoch0 + (step // redraw_steps if redraw_steps else 0)
            assert ep < self.n_epochs
            b = step % self.n_batches
            for layer in range(L):
                if lib.dx_route_forward(h, layer, None, self.lgs[ep][layer][b].data_ptr(), self.xs[layer][b].data_ptr(), T,
                                        *p, yp):
                    raise RuntimeError(lib.dx_last_error(h).decode())
                if (step, layer) in samples:
                    # the map the kernels of this call read: publications happen in the pump, between steps
                    kept.append(dict(step=step, layer=layer, epoch=ep, batch=b, formats=ctx.dx_get_formats()[layer].copy(),
                                     y=y.clone(), ids=rb.ids.clone(), perm=rb.perm.clone(), counts=rb.counts.clone()))
            if ev:
                ev[step + 1].record(stream)
            stream.synchronize()
            issued, published, queued = ctx.dx_transitions_pump(issue_per_step)
            if since_enqueue is not None:
                since_enqueue += 1
                if queued == 0 and ctx.dx_get_stats()["in_flight"] == 0:
                    drain.append(since_enqueue)
                    since_enqueue = None
            if (step + 1) % self.window == 0 and step + 1 < steps:  # no step follows the last one to carry it out
                wanted = 0
                ctx.dx_window_end()
                for layer in range(L):
                    if margin_q16 or rank_slack:
                        target = ctx.dx_select_resident_stable(layer, self.layer_budget, margin_q16=margin_q16,
                                                               rank_slack=rank_slack)
                    else:
                        target = ctx.dx_select_resident(layer, self.layer_budget)
                    pro, dem = ctx.dx_plan_transitions(layer, target)
                    ctx.dx_transitions_enqueue(layer, pro, dem)
                    wanted += len(pro) + len(dem)
                if wanted and since_enqueue is None:
                    since_enqueue = 0
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        st1 = ctx.dx_get_stats()
        out = dict(wall_s=wall, steps=steps,
                   promotions=st1["promotions_published"] - st0["promotions_published"],
                   demotions=st1["demotions_published"] - st0["demotions_published"],
                   h2d_bytes_per_step=(st1["h2d_bytes"] - st0["h2d_bytes"]) / steps,
                   quantize_bytes_per_step=(st1["quantize_read_bytes"] + st1["quantize_write_bytes"]
                                            - st0["quantize_read_bytes"] - st0["quantize_write_bytes"]) / steps,
                   steps_to_drain_after_window_end=drain, still_draining_at_end=since_enqueue is not None,
                   queued_at_end=st1["queued"], in_flight_at_end=st1["in_flight"],
                   peak_in_flight=st1["peak_in_flight"], peak_reserved_bytes=st1["peak_reserved_bytes"],
                   deferred=st1["deferred"] - st0["deferred"])
        if ev:
            ms = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])
            out.update(p50_ms=float(np.percentile(ms, 50)), p99_ms=float(np.percentile(ms, 99)), max_ms=float(ms.max()),
                       mean_ms=float(ms.mean()))
        return out, kept

    def budget_cap(self) -> int:
        return self.L * self.layer_budget + self.spare * (self.b_hi + self.b_lo)

    def close(self):
        self.ctx.dx_migrate_poll(wait=True)
        self.ctx.close()
