"""Seeded synthetic inputs for the mixed-precision MoE layer.

This module only *draws data*: activations, router matrices, expert master
weights and the Zipf-skewed router bias, all rounded to bf16 where the layer
consumes bf16.  It holds none of the method's arithmetic (no top-k, no
quantizer, no expert math, no selection rule), so both the CPU oracle and the
HIP path can be fed from the same arrays without sharing any code.

Shapes follow the model table of the paper's evaluation setup (Table
"Configuration of evaluated MoE models": 48 layers, 128 experts top-8 for the
30B model; 48 layers, 512 experts + 1 shared, top-10 for the 80B model).  The
heavy-tailed routing stands in for the skew described in the paper's
Observation 2; no item of any public benchmark is used or reproduced.

bf16 tensors are carried as ``numpy.uint16`` bit patterns on the host.
"""
from __future__ import annotations

import dataclasses
import numpy as np


# --------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (input formatting only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bits."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    T: int            # tokens per layer call
    d: int            # hidden size
    f: int            # expert SwiGLU intermediate size
    E: int            # routed experts per layer
    k: int            # top-k
    group: int        # int4 group size along K
    n_hi: int         # bf16-resident experts per layer the budget should yield
    L: int = 1        # layers
    zipf_s: float | None = None   # exponent of the Zipf router bias (None: no bias)
    shared_f: int = 0             # intermediate size of the always-bf16 shared expert (0: none)
    window_steps: int = 256
    redraw_every: int = 0         # steps between re-draws of the Zipf permutation (0: never)
    steps: int = 1


WORKLOADS = {
    # tiny layer the CPU oracle finishes in well under a second
    "C1": Workload("C1", 1, T=16, d=256, f=128, E=8, k=2, group=64, n_hi=2),
    # Qwen3-30B-A3B-shaped layer, decode
    "C2": Workload("C2", 2, T=32, d=2048, f=768, E=128, k=8, group=128, n_hi=32, zipf_s=1.1),
    # same layer, prefill
    "C3": Workload("C3", 3, T=4096, d=2048, f=768, E=128, k=8, group=128, n_hi=32, zipf_s=1.1),
    # Qwen3-Next-80B-A3B-shaped 48-layer stack, decode, one shared expert per layer
    "C4": Workload("C4", 4, T=32, d=2048, f=512, E=512, k=10, group=128, n_hi=12, L=48,
                   zipf_s=1.0, shared_f=512),
    # 30B-shaped 48-layer stack with the hot set re-drawn every 256 steps
    "C5": Workload("C5", 5, T=32, d=2048, f=768, E=128, k=8, group=128, n_hi=32, L=48,
                   zipf_s=1.1, redraw_every=256, steps=2048),
    # Phi-3.5-MoE-shaped layer: few, very large experts, top-2 (a different tiling regime; not one of
    # the baseline configurations, used by the shape tests and the token-count sweep)
    "X1": Workload("X1", 6, T=32, d=4096, f=6400, E=16, k=2, group=128, n_hi=4, zipf_s=1.0),
}

# tensor ids for the seed sequence
_TID_X, _TID_WR, _TID_PERM, _TID_WG, _TID_WU, _TID_WD, _TID_SHARED = range(7)


def _rng(seed: int, config_id: int, layer: int, tensor_id: int, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, config_id, layer, tensor_id, extra]))


def zipf_bias(E: int, s: float, seed: int, config_id: int, layer: int, epoch: int = 0) -> np.ndarray:
    """Per-expert router bias ln(z_rank) under a seeded random permutation.

    z_r = r^-s / sum_r r^-s for rank r = 1..E.  ``epoch`` re-draws the
    permutation (hot-set drift)."""
    r = np.arange(1, E + 1, dtype=np.float64)
    z = r ** (-float(s))
    z /= z.sum()
    pi = _rng(seed, config_id, layer, _TID_PERM, epoch).permutation(E)
    return np.log(z[pi]).astype(np.float32)


def activations(wl: Workload, seed: int = 0, layer: int = 0, step: int = 0) -> np.ndarray:
    """x [T, d] ~ N(0, 1), bf16 bits."""
    g = _rng(seed, wl.config_id, layer, _TID_X, step)
    return f32_to_bf16_bits(g.standard_normal((wl.T, wl.d), dtype=np.float32))


def router_matrix(wl: Workload, seed: int = 0, layer: int = 0) -> np.ndarray:
    """W_r [E, d] ~ N(0, std 0.02), bf16 bits."""
    g = _rng(seed, wl.config_id, layer, _TID_WR)
    return f32_to_bf16_bits(0.02 * g.standard_normal((wl.E, wl.d), dtype=np.float32))


def router_logits(wl: Workload, x_bits: np.ndarray, wr_bits: np.ndarray,
                  seed: int = 0, layer: int = 0, epoch: int = 0) -> np.ndarray:
    """fp32 logits [T, E] = x . W_r^T (+ Zipf bias).  Computed once here and
    handed, as one array, to every consumer."""
    x = bf16_bits_to_f32(x_bits)
    wr = bf16_bits_to_f32(wr_bits)
    logits = (x @ wr.T).astype(np.float32)
    if wl.zipf_s is not None:
        logits = logits + zipf_bias(wl.E, wl.zipf_s, seed, wl.config_id, layer, epoch)[None, :]
    return np.ascontiguousarray(logits, dtype=np.float32)


def expert_master(wl: Workload, seed: int, layer: int, expert: int):
    """bf16 master weights of one routed expert: (W_gate [f,d], W_up [f,d], W_down [d,f])."""
    out = []
    for tid, shape in ((_TID_WG, (wl.f, wl.d)), (_TID_WU, (wl.f, wl.d)), (_TID_WD, (wl.d, wl.f))):
        g = _rng(seed, wl.config_id, layer, tid, expert)
        out.append(f32_to_bf16_bits(0.02 * g.standard_normal(shape, dtype=np.float32)))
    return tuple(out)


def shared_master(wl: Workload, seed: int, layer: int):
    """bf16 weights of the layer's shared expert (80B-shaped workload)."""
    assert wl.shared_f > 0
    f = wl.shared_f
    out = []
    for i, shape in enumerate(((f, wl.d), (f, wl.d), (wl.d, f))):
        g = _rng(seed, wl.config_id, layer, _TID_SHARED, i)
        out.append(f32_to_bf16_bits(0.02 * g.standard_normal(shape, dtype=np.float32)))
    return tuple(out)


def layer_masters(wl: Workload, seed: int = 0, layer: int = 0):
    """All routed experts of one layer as stacked arrays [E,f,d], [E,f,d], [E,d,f] (bf16 bits)."""
    wg = np.empty((wl.E, wl.f, wl.d), np.uint16)
    wu = np.empty((wl.E, wl.f, wl.d), np.uint16)
    wd = np.empty((wl.E, wl.d, wl.f), np.uint16)
    for e in range(wl.E):
        wg[e], wu[e], wd[e] = expert_master(wl, seed, layer, e)
    return wg, wu, wd


def layer_inputs(wl: Workload, seed: int = 0, layer: int = 0, step: int = 0, epoch: int = 0):
    """(x bits [T,d], logits fp32 [T,E]) for one layer call."""
    x = activations(wl, seed, layer, step)
    wr = router_matrix(wl, seed, layer)
    return x, router_logits(wl, x, wr, seed, layer, epoch)


# --------------------------------------------------------------------------
# device-side draws for the full-size stacks (torch is the memory provider)
# --------------------------------------------------------------------------
def device_masters(wl: Workload, seed: int, layer: int, device="cuda"):
    """Stacked bf16 master weights of one layer drawn on the device:
    W_gate [E,f,d], W_up [E,f,d], W_down [E,d,f].  The same tensors (copied
    back to the host where needed) feed both consumers, so the draw need not
    match the host generator bit for bit."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + wl.config_id * 10007 + layer) & 0x7FFFFFFF)
    mk = lambda *shape: (0.02 * torch.randn(*shape, generator=g, device=device,
                                            dtype=torch.float32)).to(torch.bfloat16)
    return mk(wl.E, wl.f, wl.d), mk(wl.E, wl.f, wl.d), mk(wl.E, wl.d, wl.f)
