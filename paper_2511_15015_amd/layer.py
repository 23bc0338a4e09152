"""Caller-side set-up of one MoE layer's expert versions in device memory.

Allocation and bookkeeping only (PyTorch owns the memory): the bf16 versions
are slices of the master tensors, the int4 versions are produced by the
library's quantize kernel, and every expert is published through
``dx_swap_handle``.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


class LayerWeights:
    """Expert versions of one layer in caller-owned memory.

    wg, wu: bf16 device tensors [E, f, d]; wd: [E, d, f].  Experts listed in
    ``resident_ids`` are published as bf16, all others as int4 with group size
    ``group``.  With ``keep_masters=False`` only the resident experts' bf16
    weights stay referenced."""

    def __init__(self, ctx: B.Context, layer: int, wg, wu, wd, resident_ids, group: int,
                 keep_masters: bool = True, publish: bool = True):
        E, f, d = wg.shape
        assert wu.shape == (E, f, d) and wd.shape == (E, d, f)
        assert wg.dtype == torch.bfloat16 and wg.is_cuda
        self.ctx, self.layer, self.E, self.f, self.d, self.group = ctx, layer, E, f, d, group
        dev = wg.device
        res = np.asarray(sorted(int(e) for e in resident_ids), np.int64)
        is_hi = np.zeros(E, bool)
        is_hi[res] = True
        lo = np.flatnonzero(~is_hi)
        self.is_hi = is_hi
        self.hi_ids, self.lo_ids = res, lo
        self.hi_slot = {int(e): i for i, e in enumerate(res)}
        self.lo_slot = {int(e): i for i, e in enumerate(lo)}
        # int4 versions of the non-resident experts: one quantize launch per matrix kind
        nlo = len(lo)
        self.q = [torch.empty((nlo, f, d // 2), dtype=torch.uint8, device=dev),
                  torch.empty((nlo, f, d // 2), dtype=torch.uint8, device=dev),
                  torch.empty((nlo, d, f // 2), dtype=torch.uint8, device=dev)]
        self.s = [torch.empty((nlo, f, d // group), dtype=torch.bfloat16, device=dev),
                  torch.empty((nlo, f, d // group), dtype=torch.bfloat16, device=dev),
                  torch.empty((nlo, d, f // group), dtype=torch.bfloat16, device=dev)]
        if nlo:
            lo_t = torch.from_numpy(lo).to(dev)
            for i, m in enumerate((wg, wu, wd)):
                src = m.index_select(0, lo_t).contiguous()
                rows, K = src.shape[0] * src.shape[1], src.shape[2]
                ctx.dx_quantize_expert(src, rows, K, group, self.q[i], self.s[i])
                torch.cuda.current_stream().synchronize()
                del src
        if keep_masters:
            self.hi = [wg, wu, wd]
            self._hi_index = lambda e: e
        else:
            res_t = torch.from_numpy(res).to(dev)
            self.hi = [m.index_select(0, res_t).contiguous() for m in (wg, wu, wd)]
            self._hi_index = lambda e: self.hi_slot[e]
        if publish:
            for e in range(E):
                ctx.dx_swap_handle(layer, e, self.handle(e))

    def handle(self, e: int, fmt: int | None = None) -> B.DxHandle:
        """Handle of expert e in its configured format (or ``fmt`` if that version exists)."""
        e = int(e)
        want_hi = self.is_hi[e] if fmt is None else fmt == B.DX_FMT_BF16
        if want_hi:
            i = self._hi_index(e)
            return B.make_handle(B.DX_FMT_BF16, self.hi[0][i], self.hi[1][i], self.hi[2][i])
        i = self.lo_slot[e]
        return B.make_handle(B.DX_FMT_INT4G, self.q[0][i], self.q[1][i], self.q[2][i],
                             self.s[0][i], self.s[1][i], self.s[2][i])


class QuantPairLayerWeights:
    """Expert versions of one layer for the int4 (high tier) / int2 (low tier) pair, in caller-owned
    memory: experts in ``hi_ids`` are published as int4, all others as int2, both produced by the
    library's quantize kernels from the bf16 masters wg, wu [E,f,d], wd [E,d,f]."""

    def __init__(self, ctx: B.Context, layer: int, wg, wu, wd, hi_ids, group: int):
        E, f, d = wg.shape
        assert wu.shape == (E, f, d) and wd.shape == (E, d, f) and wg.dtype == torch.bfloat16 and wg.is_cuda
        dev = wg.device
        self.is_hi = np.zeros(E, bool)
        self.is_hi[np.asarray(sorted(int(e) for e in hi_ids), np.int64)] = True
        self.sets = {}
        for fmt, ids, div, quant in ((B.DX_FMT_INT4G, np.flatnonzero(self.is_hi), 2, ctx.dx_quantize_expert),
                                     (B.DX_FMT_INT2G, np.flatnonzero(~self.is_hi), 4, ctx.dx_quantize_expert_int2)):
            n = len(ids)
            q = [torch.empty((n, f, d // div), dtype=torch.uint8, device=dev),
                 torch.empty((n, f, d // div), dtype=torch.uint8, device=dev),
                 torch.empty((n, d, f // div), dtype=torch.uint8, device=dev)]
            sc = [torch.empty((n, f, d // group), dtype=torch.bfloat16, device=dev),
                  torch.empty((n, f, d // group), dtype=torch.bfloat16, device=dev),
                  torch.empty((n, d, f // group), dtype=torch.bfloat16, device=dev)]
            if n:
                idx = torch.from_numpy(ids).to(dev)
                for i, m in enumerate((wg, wu, wd)):
                    src = m.index_select(0, idx).contiguous()
                    quant(src, src.shape[0] * src.shape[1], src.shape[2], group, q[i], sc[i])
                    torch.cuda.current_stream().synchronize()
                    del src
            self.sets[fmt] = (q, sc, {int(e): i for i, e in enumerate(ids)})
        for e in range(E):
            fmt = B.DX_FMT_INT4G if self.is_hi[e] else B.DX_FMT_INT2G
            q, sc, slot = self.sets[fmt]
            i = slot[e]
            ctx.dx_swap_handle(layer, e, B.make_handle(fmt, q[0][i], q[1][i], q[2][i], sc[0][i], sc[1][i], sc[2][i]))


class RoutingBuffers:
    """Device buffers written by dx_route and read by dx_moe_forward."""

    def __init__(self, T: int, E: int, k: int, device="cuda"):
        self.T, self.E, self.k = T, E, k
        self.ids = torch.empty((T, k), dtype=torch.int32, device=device)
        self.w = torch.empty((T, k), dtype=torch.float32, device=device)
        self.counts = torch.empty(E, dtype=torch.int32, device=device)
        self.offsets = torch.empty(E + 1, dtype=torch.int32, device=device)
        self.perm = torch.empty(T * k, dtype=torch.int32, device=device)

    def route(self, ctx: B.Context, layer: int, logits, T=None):
        T = self.T if T is None else T
        ctx.dx_route(layer, logits, T, self.ids, self.w, self.counts, self.offsets, self.perm)

    def route_forward(self, ctx: B.Context, layer: int, logits, x, y, table=None, T=None):
        T = self.T if T is None else T
        ctx.dx_route_forward(layer, table, logits, x, T, self.ids, self.w, self.counts, self.offsets, self.perm, y)

    def forward(self, ctx: B.Context, layer: int, x, y, table=None, T=None):
        T = self.T if T is None else T
        ctx.dx_moe_forward(layer, table, x, T, self.ids, self.w, self.offsets, self.perm, y)


def bits_to_device(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """numpy uint16 bf16 bit patterns -> bf16 device tensor (a reinterpretation, no rounding)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def device_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
