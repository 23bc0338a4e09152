"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle
on the same seeded inputs.  Integer stages bit-exact; layer outputs within
rel-L2 1e-2 (the bar the build's target states); routing weights within 1e-5."""
import numpy as np
import pytest
import torch

from paper_2511_15015_amd import workloads as W
from paper_2511_15015_amd.workloads import WORKLOADS, bf16_bits_to_f32, f32_to_bf16_bits
from tests.bounds import assert_elementwise

pytestmark = pytest.mark.gpu

REL_L2_TOL = 1e-2
W_TOL = 1e-5


@pytest.fixture(scope="module")
def B():
    from paper_2511_15015_amd import binding
    binding.load()
    assert torch.cuda.is_available()
    return binding


@pytest.fixture(scope="module")
def LY():
    from paper_2511_15015_amd import layer
    return layer


def rel_l2(y_gpu_bits, y_ref):
    y = bf16_bits_to_f32(y_gpu_bits).astype(np.float64)
    return float(np.linalg.norm(y - y_ref) / max(np.linalg.norm(y_ref), 1e-300))


def sync():
    torch.cuda.synchronize()


# ------------------------------------------------------------------ quantizer
@pytest.mark.parametrize("rows,K,group", [(128, 256, 64), (768, 2048, 128), (2048, 768, 128), (37, 96, 32),
                                          (1, 128, 128), (5, 64, 64)])
def test_quantize_bit_exact(B, LY, dxo, rows, K, group):
    print(f"quantize rows={rows} K={K} group={group}", flush=True)
    g = np.random.default_rng(rows * 7 + K)
    w = 0.02 * g.standard_normal((rows, K)).astype(np.float32)
    w[0, :group] = 0.0                       # an all-zero group
    if rows > 2:
        w[1] *= 1e3
        w[2] *= 1e-4
    # exact .5 ties: scale 1 (absmax 7), values k + 0.5
    w[-1, :group] = 0.0
    w[-1, 0] = 7.0
    w[-1, 1:9] = [0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, -6.5]
    bits = f32_to_bf16_bits(w)
    q_ref, s_ref = dxo.quantize(bits, group)
    ctx = B.Context(L=1, E=4, d=128, f=128, top_k=2, group=group, max_tokens=4)
    wd = LY.bits_to_device(bits)
    q = torch.empty((rows, K // 2), dtype=torch.uint8, device="cuda")
    s = torch.empty((rows, K // group), dtype=torch.bfloat16, device="cuda")
    ctx.dx_quantize_expert(wd, rows, K, group, q, s)
    sync()
    assert np.array_equal(LY.device_to_bits(s), s_ref)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    ctx.close()


@pytest.mark.parametrize("bits", [4, 2])
def test_quantize_exact_ties_and_extreme_scales(B, LY, dxo, bits):
    """Rows built to sit on the quantizer's rounding ties: the group scale is a power of two (absmax = q_max *
    2^k) and the other values are multiples of half a step, so about half of them are exact ties that must go
    to the even code; scales with other mantissas mixed in; groups with tiny and huge scales (the kernel's
    divide shortcut does not cover those) and an all-zero group.  Codes and scales bit for bit."""
    group, rows, K = 128, 96, 1024
    g = np.random.default_rng(1234 + bits)
    q_max = 7 if bits == 4 else 1
    w = np.zeros((rows, K), np.float32)
    for r in range(rows):
        for c0 in range(0, K, group):
            kind = (r + c0 // group) % 6
            if kind == 0:                                   # step 2^k: every multiple of step/2 in range
                step = 2.0 ** int(g.integers(-12, 3))
                vals = g.integers(-2 * q_max, 2 * q_max + 1, group) * (step / 2)
            elif kind == 1:                                 # step 1.5 * 2^k: ties at odd multiples of 0.75 * 2^k
                step = 1.5 * 2.0 ** int(g.integers(-10, 2))
                vals = g.integers(-2 * q_max, 2 * q_max + 1, group) * (step / 2)
            elif kind == 2:                                 # tiny scale (below the shortcut's range)
                step = 2.0 ** -110
                vals = g.integers(-2 * q_max, 2 * q_max + 1, group) * (step / 2)
            elif kind == 3:                                 # huge scale
                step = 2.0 ** 105
                vals = g.integers(-2 * q_max, 2 * q_max + 1, group) * (step / 2)
            elif kind == 4:                                 # ordinary weights
                step = None
                vals = 0.02 * g.standard_normal(group)
            else:
                step = None
                vals = np.zeros(group)
            vals = np.asarray(vals, np.float64)
            if step is not None:
                vals[0] = q_max * step                      # pins absmax, hence the scale
            w[r, c0:c0 + group] = vals
    bits_in = f32_to_bf16_bits(w)
    quant = dxo.quantize if bits == 4 else dxo.quantize2
    q_ref, s_ref = quant(bits_in, group)
    # the rows really are full of ties: the oracle's codes differ from rounding half away from zero
    wf = bf16_bits_to_f32(bits_in).astype(np.float64)
    sf = np.repeat(bf16_bits_to_f32(s_ref).astype(np.float64), group, axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        frac = np.where(sf > 0, np.abs(wf / sf) % 1.0, 0.0)
    assert np.count_nonzero(frac == 0.5) > rows * K // 8
    ctx = B.Context(L=1, E=4, d=128, f=128, top_k=2, group=group, max_tokens=4)
    q = torch.empty((rows, K // (8 // bits)), dtype=torch.uint8, device="cuda")
    s = torch.empty((rows, K // group), dtype=torch.bfloat16, device="cuda")
    (ctx.dx_quantize_expert if bits == 4 else ctx.dx_quantize_expert_int2)(LY.bits_to_device(bits_in), rows, K, group, q, s)
    sync()
    assert np.array_equal(LY.device_to_bits(s), s_ref)
    bad = np.argwhere(q.cpu().numpy() != q_ref)
    assert len(bad) == 0, bad[:5]
    ctx.close()


def test_quantize_rejects_bad_arguments(B):
    ctx = B.Context(L=1, E=4, d=128, f=128, top_k=2, group=64, max_tokens=4)
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.DxError) as ei:
        ctx.dx_quantize_expert(buf, 2, 96, 64, buf, buf)          # K % group != 0
    assert ei.value.status == B.DX_ERR_INVALID
    with pytest.raises(B.DxError):
        ctx.dx_quantize_expert(buf, 2, 128, 48, buf, buf)         # unsupported group
    with pytest.raises(B.DxError):
        ctx.dx_quantize_expert(None, 2, 128, 64, buf, buf)        # null pointer
    ctx.dx_quantize_expert(buf, 0, 128, 64, buf, buf)             # empty is fine
    ctx.close()


# -------------------------------------------------------------------- routing
def _check_route(B, LY, dxo, logits, k, max_tokens=None):
    T, E = logits.shape
    ctx = B.Context(L=1, E=E, d=64, f=64, top_k=k, group=32, max_tokens=max(max_tokens or T, 1))
    rb = LY.RoutingBuffers(max(T, 1), E, k)
    dl = torch.from_numpy(logits).cuda() if T else torch.empty((1, E), dtype=torch.float32, device="cuda")
    rb.route(ctx, 0, dl, T)
    sync()
    ids_r, w_r, counts_r, offsets_r, perm_r = dxo.route(logits, k)
    assert np.array_equal(rb.counts.cpu().numpy(), counts_r)
    assert np.array_equal(rb.offsets.cpu().numpy(), offsets_r)
    if T:
        assert np.array_equal(rb.ids.cpu().numpy()[:T], ids_r)
        assert np.array_equal(rb.perm.cpu().numpy()[:T * k], perm_r)
        wg = rb.w.cpu().numpy()[:T].astype(np.float64)
        assert np.max(np.abs(wg - w_r) / np.maximum(w_r, 1e-30)) < W_TOL or np.max(np.abs(wg - w_r)) < 1e-7
    ctx.close()


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_route_workloads_bit_exact(B, LY, dxo, name):
    wl = WORKLOADS[name]
    print(f"route {name} T={wl.T} E={wl.E} k={wl.k}", flush=True)
    _, logits = W.layer_inputs(wl, seed=0)
    _check_route(B, LY, dxo, logits, wl.k)


@pytest.mark.parametrize("T,E,k", [(0, 8, 2), (1, 8, 2), (63, 16, 4), (64, 16, 4), (65, 16, 4), (130, 200, 6),
                                   (1000, 1024, 3), (5, 8, 8), (3, 1, 1), (257, 64, 64)])
def test_route_edge_shapes_and_ties(B, LY, dxo, T, E, k):
    print(f"route T={T} E={E} k={k}", flush=True)
    g = np.random.default_rng(T * 31 + E)
    # logits on a coarse grid: many exact ties, both signs of zero
    logits = np.round(g.standard_normal((T, E)) * 2).astype(np.float32) / 2
    logits[logits == 0] *= np.where(g.random(np.count_nonzero(logits == 0)) < 0.5, -1.0, 1.0).astype(np.float32)
    _check_route(B, LY, dxo, logits, k)


def test_route_rejects_bad_arguments(B, LY):
    ctx = B.Context(L=2, E=8, d=64, f=64, top_k=2, group=32, max_tokens=16)
    rb = LY.RoutingBuffers(16, 8, 2)
    lg = torch.zeros((16, 8), dtype=torch.float32, device="cuda")
    for layer, T in [(2, 4), (-1, 4), (0, 17), (0, -1)]:
        with pytest.raises(B.DxError) as ei:
            ctx.dx_route(layer, lg, T, rb.ids, rb.w, rb.counts, rb.offsets, rb.perm)
        assert ei.value.status == B.DX_ERR_INVALID
    with pytest.raises(B.DxError):
        ctx.dx_route(0, None, 4, rb.ids, rb.w, rb.counts, rb.offsets, rb.perm)
    for bad in [dict(E=0), dict(top_k=9), dict(group=48), dict(d=100), dict(max_tokens=0), dict(alpha_q16=65536)]:
        kw = dict(L=1, E=8, d=64, f=64, top_k=2, group=32, max_tokens=4)
        kw.update(bad)
        with pytest.raises(B.DxError):
            B.Context(**kw)
    ctx.close()


@pytest.mark.parametrize("T,E,d,with_bias", [(32, 128, 2048, True), (1, 8, 64, False), (33, 40, 96, True),
                                             (4096, 128, 2048, True), (70, 512, 2048, False)])
def test_router_logits_match_oracle(B, LY, dxo, T, E, d, with_bias):
    """The router gate on the matrix cores against the fp64 oracle: fp32 accumulation of exact bf16
    products, so the difference stays near d * 2^-24 of the largest partial sum."""
    g = np.random.default_rng(T + E)
    x = W.f32_to_bf16_bits(g.standard_normal((T, d)).astype(np.float32))
    wr = W.f32_to_bf16_bits((0.02 * g.standard_normal((E, d))).astype(np.float32))
    bias = (g.standard_normal(E) * 3).astype(np.float32) if with_bias else None
    ctx = B.Context(L=1, E=E, d=d, f=64, top_k=2, group=32, max_tokens=T)
    out = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda")
    ctx.dx_router_logits(LY.bits_to_device(x), LY.bits_to_device(wr),
                         torch.from_numpy(bias).cuda() if with_bias else None, T, out)
    sync()
    ref = dxo.router_logits(x, wr, bias)
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    scale = float(np.abs(ref).max())
    assert np.abs(got - ref).max() <= 2e-5 * max(scale, 1.0), np.abs(got - ref).max()
    with pytest.raises(B.DxError):
        ctx.dx_router_logits(LY.bits_to_device(x), LY.bits_to_device(wr), None, T + 1, out)
    ctx.close()


# ------------------------------------------------------------------ the layer
class Layer:
    """One layer set up on both sides from the same master bits."""

    def __init__(self, B, LY, dxo, wl, resident, seed=0, layer=0, masters=None, T=None, shared=None):
        self.wl, self.B = wl, B
        T = wl.T if T is None else T
        self.T = T
        self.masters = masters if masters is not None else W.layer_masters(wl, seed, layer)
        wg, wu, wd = self.masters
        self.ctx = B.Context(L=1, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=max(T, 1),
                             shared_f=wl.shared_f if shared is not None else 0)
        self.dev = [LY.bits_to_device(m) for m in self.masters]
        self.lw = LY.LayerWeights(self.ctx, 0, *self.dev, resident, wl.group)
        self.rb = LY.RoutingBuffers(max(T, 1), wl.E, wl.k)
        self.resident = set(int(e) for e in resident)
        self.versions = [dxo.ExpertVersion.bf16(wg[e], wu[e], wd[e]) if e in self.resident
                         else dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group)
                         for e in range(wl.E)]
        self.shared = None
        if shared is not None:
            self.shared_dev = [LY.bits_to_device(m) for m in shared]
            self.ctx.dx_swap_handle(0, wl.E, B.make_handle(B.DX_FMT_BF16, *self.shared_dev))
            self.shared = dxo.ExpertVersion.bf16(*shared)
        self.LY, self.dxo = LY, dxo

    def run(self, x_bits, logits, tokens=None):
        T = x_bits.shape[0]
        xd = self.LY.bits_to_device(x_bits)
        ld = torch.from_numpy(logits).cuda()
        y = torch.empty((T, self.wl.d), dtype=torch.bfloat16, device="cuda")
        self.rb.route(self.ctx, 0, ld, T)
        self.rb.forward(self.ctx, 0, xd, y, None, T)
        sync()
        ids, w, counts, offsets, perm = self.dxo.route(logits, self.wl.k)
        assert np.array_equal(self.rb.ids.cpu().numpy()[:T], ids)
        y_ref = self.dxo.moe_forward(self.versions, self.wl.d, self.wl.f, self.wl.group, x_bits, ids, w,
                                     shared=self.shared, shared_f=self.wl.shared_f if self.shared else 0,
                                     tokens=tokens)
        y_gpu = self.LY.device_to_bits(y)
        if tokens is not None:
            y_gpu = y_gpu[np.asarray(tokens)]
        # next to the norm the caller checks: every element within the bound the bf16 roundings of H, O and y allow
        used = assert_elementwise(self.dxo, y_gpu, y_ref, self.versions, self.wl.group, x_bits, ids, w, shared=self.shared,
                                  tokens=tokens, T_call=T)
        print(f"  element-wise: largest error = {used:.2f} of its bound", flush=True)
        return y_gpu, y_ref


def test_forward_c1_mixed_all_hi_all_lo(B, LY, dxo):
    wl = WORKLOADS["C1"]
    x, logits = W.layer_inputs(wl, seed=0)
    masters = W.layer_masters(wl, 0, 0)
    for resident in ([1, 6], list(range(wl.E)), []):
        print(f"forward C1 resident={resident}", flush=True)
        ly = Layer(B, LY, dxo, wl, resident, masters=masters)
        y_gpu, y_ref = ly.run(x, logits)
        err = rel_l2(y_gpu, y_ref)
        print("  rel-L2", err, flush=True)
        assert err <= REL_L2_TOL
        ly.ctx.close()


@pytest.mark.parametrize("shift", [16, 80, 112])
def test_forward_weights_that_start_inside_a_line(B, LY, dxo, shift):
    """The boundary promises 16-byte alignment only.  The decode kernels fetch weights in pieces that are whole
    128-byte lines when a matrix starts on a line; here every matrix and scale array of every expert starts
    `shift` bytes into one (bf16 and int4 versions, d = 2048 so that the line-shaped loads are the ones that
    run): same bits as with the aligned copies, and the oracle's values."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=24, E=8, k=3, d=2048, f=128, group=128)
    print(f"weights shifted by {shift} bytes", flush=True)
    x, logits = W.layer_inputs(wl, seed=41)
    ly = Layer(B, LY, dxo, wl, [1, 4, 6], seed=41)
    y_gpu, y_ref = ly.run(x, logits)
    assert rel_l2(y_gpu, y_ref) <= REL_L2_TOL
    keep = []

    def moved(t):
        n = t.numel() * t.element_size()
        raw = torch.zeros(n + 256, dtype=torch.uint8, device=t.device)
        base = (-raw.data_ptr()) % 128 + shift                      # `shift` bytes past a line boundary
        v = raw[base:base + n].view(t.dtype).view(t.shape)
        v.copy_(t)
        assert v.data_ptr() % 128 == shift % 128 and v.data_ptr() % 16 == 0
        keep.append(raw)
        return v

    lw = ly.lw
    for e in range(wl.E):
        if lw.is_hi[e]:
            h = B.make_handle(B.DX_FMT_BF16, *(moved(m[e]) for m in lw.hi))
        else:
            i = lw.lo_slot[e]
            h = B.make_handle(B.DX_FMT_INT4G, *(moved(q[i]) for q in lw.q), *(moved(sc[i]) for sc in lw.s))
        ly.ctx.dx_swap_handle(0, e, h)
    y_moved, _ = ly.run(x, logits)
    assert np.array_equal(y_moved, y_gpu)
    ly.ctx.close()


@pytest.mark.parametrize("T", [1, 7, 16, 17, 33, 40])
def test_forward_ragged_token_counts(B, LY, dxo, T):
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=4, k=2)   # few experts: segments longer than one 16-row tile
    print(f"forward ragged T={T}", flush=True)
    x, logits = W.layer_inputs(wl, seed=3)
    ly = Layer(B, LY, dxo, wl, [0, 2], seed=3)
    y_gpu, y_ref = ly.run(x, logits)
    assert rel_l2(y_gpu, y_ref) <= REL_L2_TOL
    # per-token check as well: no token may be far off
    yg = bf16_bits_to_f32(y_gpu).astype(np.float64)
    tok = np.linalg.norm(yg - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    assert tok.max() <= 2 * REL_L2_TOL
    ly.ctx.close()


def test_forward_group32(B, LY, dxo):
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], group=32, T=9)
    x, logits = W.layer_inputs(wl, seed=4)
    ly = Layer(B, LY, dxo, wl, [3], seed=4)
    y_gpu, y_ref = ly.run(x, logits)
    assert rel_l2(y_gpu, y_ref) <= REL_L2_TOL
    ly.ctx.close()


def test_forward_c2_decode_full(B, LY, dxo):
    """The 30B-shaped decode layer at full size; resident set = top-32 by the oracle's window counts."""
    wl = WORKLOADS["C2"]
    print("forward C2: drawing masters", flush=True)
    masters = W.layer_masters(wl, 0, 0)
    x, logits = W.layer_inputs(wl, seed=0)
    # hotness from a warm-up window of routing only (oracle side decides the set for both)
    c = np.zeros(wl.E, np.int64)
    for step in range(1, 9):
        _, lg = W.layer_inputs(wl, seed=0, step=step)
        _, _, counts, _, _ = dxo.route(lg, wl.k)
        dxo.hotness_update(c, counts)
    S = np.zeros(wl.E, np.uint64)
    dxo.window_end(S, c, 0)
    resident = dxo.select_topn(S, wl.n_hi)
    print("forward C2: running", flush=True)
    ly = Layer(B, LY, dxo, wl, resident, masters=masters)
    y_gpu, y_ref = ly.run(x, logits)
    err = rel_l2(y_gpu, y_ref)
    print("  C2 rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    ly.ctx.close()


def test_forward_with_shared_expert(B, LY, dxo):
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C4"], L=1, E=16, k=4, T=19, d=256, f=128, shared_f=256, group=128)
    x, logits = W.layer_inputs(wl, seed=5)
    shared = W.shared_master(wl, 5, 0)
    ly = Layer(B, LY, dxo, wl, [0, 5, 9], seed=5, shared=shared)
    y_gpu, y_ref = ly.run(x, logits)
    err = rel_l2(y_gpu, y_ref)
    print("  shared rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    ly.ctx.close()


def test_forward_empty_batch_and_bad_arguments(B, LY, dxo):
    wl = WORKLOADS["C1"]
    ly = Layer(B, LY, dxo, wl, [0])
    y = torch.zeros((wl.T, wl.d), dtype=torch.bfloat16, device="cuda")
    x = torch.zeros((wl.T, wl.d), dtype=torch.bfloat16, device="cuda")
    ly.rb.forward(ly.ctx, 0, x, y, None, 0)                      # T = 0: nothing to do
    with pytest.raises(B.DxError):
        ly.rb.forward(ly.ctx, 0, None, y, None, 4)
    with pytest.raises(B.DxError):
        ly.rb.forward(ly.ctx, 1, x, y, None, 4)
    with pytest.raises(B.DxError):
        ly.rb.forward(ly.ctx, 0, x, y, None, wl.T + 1)
    ly.ctx.close()
    # a context whose experts were never published refuses to run
    ctx = B.Context(L=1, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T)
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    with pytest.raises(B.DxError):
        rb.forward(ctx, 0, x, y, None, 4)
    ctx.close()


# ---------------------------------------------------------- swap / publication
def test_swap_handle_takes_effect_between_forward_passes(B, LY, dxo):
    wl = WORKLOADS["C1"]
    x, logits = W.layer_inputs(wl, seed=0)
    masters = W.layer_masters(wl, 0, 0)
    ly = Layer(B, LY, dxo, wl, [], masters=masters)              # all int4
    y_gpu0, y_ref0 = ly.run(x, logits)
    assert rel_l2(y_gpu0, y_ref0) <= REL_L2_TOL
    fm = ly.ctx.dx_get_formats()
    assert np.all(fm == B.DX_FMT_INT4G)
    # publish bf16 versions of every expert, straight from the master tensors
    v0 = ly.ctx.dx_get_handle(0, 3).version
    for e in range(wl.E):
        ly.ctx.dx_swap_handle(0, e, B.make_handle(B.DX_FMT_BF16, ly.dev[0][e], ly.dev[1][e], ly.dev[2][e]))
    assert ly.ctx.dx_get_handle(0, 3).version == v0 + 1
    assert np.all(ly.ctx.dx_get_formats() == B.DX_FMT_BF16)
    ly.versions = [dxo.ExpertVersion.bf16(masters[0][e], masters[1][e], masters[2][e]) for e in range(wl.E)]
    y_gpu1, y_ref1 = ly.run(x, logits)
    assert rel_l2(y_gpu1, y_ref1) <= REL_L2_TOL
    assert rel_l2(y_gpu1, y_ref0) > rel_l2(y_gpu1, y_ref1)       # it really switched versions
    # a version whose producer has not finished is refused
    ev = torch.cuda.Event()
    side = torch.cuda.Stream()
    big = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    with torch.cuda.stream(side):
        for _ in range(20):
            big.add_(1.0)
        ev.record(side)
    with pytest.raises(B.DxError) as ei:
        ly.ctx.dx_swap_handle(0, 0, ly.lw.handle(0, B.DX_FMT_INT4G), producer_event=ev.cuda_event)
    assert ei.value.status == B.DX_ERR_BUSY
    ev.synchronize()
    ly.ctx.dx_swap_handle(0, 0, ly.lw.handle(0, B.DX_FMT_INT4G), producer_event=ev.cuda_event)
    assert ly.ctx.dx_get_formats()[0, 0] == B.DX_FMT_INT4G
    with pytest.raises(B.DxError):
        ly.ctx.dx_swap_handle(0, wl.E, ly.lw.handle(0, B.DX_FMT_INT4G))   # no shared expert configured
    ly.ctx.close()


# ------------------------------------------------------- hotness and selection
def test_hotness_window_and_selection_match_oracle(B, LY, dxo):
    wl = WORKLOADS["C2"]
    L = 3
    b_hi, b_lo = dxo.expert_bytes(wl.d, wl.f, wl.group, 0), dxo.expert_bytes(wl.d, wl.f, wl.group, 1)
    ctx = B.Context(L=L, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T, alpha_q16=16384)
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    c = np.zeros((L, wl.E), np.int64)
    S = np.zeros((L, wl.E), np.uint64)
    for window in range(3):
        for step in range(6):
            for layer in range(L):
                _, lg = W.layer_inputs(wl, seed=1, layer=layer, step=window * 6 + step)
                rb.route(ctx, layer, torch.from_numpy(lg).cuda())
                ctx.dx_hotness_update(layer, rb.counts)
                _, _, counts, _, _ = dxo.route(lg, wl.k)
                dxo.hotness_update(c[layer], counts)
        assert np.array_equal(ctx.dx_get_counters(), c)
        S_gpu = ctx.dx_window_end()
        for layer in range(L):
            dxo.window_end(S[layer], c[layer], 16384)
        assert np.array_equal(S_gpu, S)
        assert not ctx.dx_get_counters().any()
        for layer in range(L):
            budget = 535560192
            ids = ctx.dx_select_resident(layer, budget)
            n = dxo.budget_capacity(budget, wl.E, b_hi, b_lo)
            assert n == 32 and np.array_equal(ids, dxo.select_topn(S[layer], n))
            assert len(ids) * b_hi + (wl.E - len(ids)) * b_lo <= budget
    with pytest.raises(B.DxError) as ei:
        ctx.dx_select_resident(0, wl.E * b_lo - 1)
    assert ei.value.status == B.DX_ERR_BUDGET
    ctx.close()


def test_route_can_update_hotness_itself(B, LY, dxo):
    wl = WORKLOADS["C2"]
    for T in (wl.T, 200):                       # single-chunk and multi-chunk routing paths
        ctx = B.Context(L=2, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=T,
                        route_updates_hotness=True)
        rb = LY.RoutingBuffers(T, wl.E, wl.k)
        c = np.zeros((2, wl.E), np.int64)
        g = np.random.default_rng(T)
        for step in range(5):
            for layer in range(2):
                lg = g.standard_normal((T, wl.E)).astype(np.float32)
                rb.route(ctx, layer, torch.from_numpy(lg).cuda())
                _, _, counts, _, _ = dxo.route(lg, wl.k)
                dxo.hotness_update(c[layer], counts)
        assert np.array_equal(ctx.dx_get_counters(), c)
        ctx.close()


# ------------------------------------------------------- prefill-sized batches
@pytest.mark.parametrize("T,E,k,resident", [(65, 4, 2, [0, 2]), (128, 4, 2, [0, 2]), (200, 4, 2, [1]), (300, 8, 3, [0, 5, 6]),
                                            (129, 2, 2, [0]), (400, 4, 1, []),
                                            # bf16 segments of 256 rows and more: 256 x 256 tiles plus a remainder
                                            (700, 4, 2, [0, 2]), (1100, 2, 2, [0, 1]), (512, 2, 2, [1]),
                                            (256, 1, 1, [0]),
                                            # one bf16 expert with 200, 385 = 256 + 129, 384 = 256 + 128 rows; two with 641
                                            (200, 1, 1, [0]), (385, 1, 1, [0]), (384, 1, 1, [0]), (641, 2, 2, [0, 1])])
def test_forward_prefill_tiles_small_shapes(B, LY, dxo, T, E, k, resident):
    """Up to 128 tokens per call the streaming kernels walk each segment in blocks of 32 tokens; above,
    segments of more than 32 tokens take the tiled MFMA kernels (bf16 and int4), the others the
    streaming ones; ragged row tiles; every token checked."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k)
    print(f"prefill tiles T={T} E={E} k={k} resident={resident}", flush=True)
    x, logits = W.layer_inputs(wl, seed=6)
    ly = Layer(B, LY, dxo, wl, resident, seed=6)
    y_gpu, y_ref = ly.run(x, logits)
    err = rel_l2(y_gpu, y_ref)
    print("  rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    yg = bf16_bits_to_f32(y_gpu).astype(np.float64)
    tok = np.linalg.norm(yg - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    assert tok.max() <= 2 * REL_L2_TOL
    ly.ctx.close()


@pytest.mark.parametrize("T,E,k,d,f,group,resident", [
    (600, 2, 2, 256, 128, 32, []),          # both experts int4 with 600 rows: two 256-row tiles and a remainder each
    (1100, 2, 2, 256, 128, 64, []),         # four tiles each; the down contraction is four steps (one trip of the loop)
    (520, 2, 1, 512, 256, 128, []),         # about 260 rows each: one tile and a few rows
    (700, 4, 2, 512, 256, 128, [0]),        # bf16 and int4 tiles in one launch
    (768, 1, 1, 256, 384, 128, []),         # three groups per row of W_down: the int4 experts stay with the 128-row tiles
    (300, 1, 1, 2048, 768, 128, []),        # the 30B layer's K extents: 64 and 24 steps
])
def test_forward_prefill_int4_segments_of_256_rows_and_more(B, LY, dxo, T, E, k, d, f, group, resident):
    """int4 experts with 256 rows and more: the leading multiple of 256 rows takes the 256 x 256 tile kernel, which
    expands the codes into its LDS ring (when the number of groups per row is even); every token, and the same
    bits on a second run."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k, d=d, f=f, group=group)
    print(f"prefill int4 tiles T={T} E={E} k={k} d={d} f={f} g={group} resident={resident}", flush=True)
    x, logits = W.layer_inputs(wl, seed=31)
    ly = Layer(B, LY, dxo, wl, resident, seed=31)
    y_gpu, y_ref = ly.run(x, logits)
    err = rel_l2(y_gpu, y_ref)
    print("  rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    yg = bf16_bits_to_f32(y_gpu).astype(np.float64)
    tok = np.linalg.norm(yg - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    assert tok.max() <= 2 * REL_L2_TOL
    again, _ = ly.run(x, logits)
    assert np.array_equal(again, y_gpu)
    ly.ctx.close()


@pytest.mark.parametrize("T,E,group,resident", [(150, 16, 128, [0, 5, 9]), (600, 16, 128, [0, 5, 9]),
                                               # 256-row tiles of the shared expert, of a bf16 and of int4 experts in one launch
                                               (1100, 4, 64, [1])])
def test_forward_prefill_with_shared_expert(B, LY, dxo, T, E, group, resident):
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C4"], L=1, E=E, k=min(4, E), T=T, d=256, f=128, shared_f=256, group=group)
    x, logits = W.layer_inputs(wl, seed=8)
    shared = W.shared_master(wl, 8, 0)
    ly = Layer(B, LY, dxo, wl, resident, seed=8, shared=shared)
    y_gpu, y_ref = ly.run(x, logits)
    err = rel_l2(y_gpu, y_ref)
    print("  prefill shared rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    ly.ctx.close()


@pytest.mark.parametrize("T,n_hi", [(4096, None), (8192, None), (4096, 0)])
def test_forward_c3_prefill_sampled_tokens(B, LY, dxo, T, n_hi):
    """The 30B-shaped prefill layer at full size (T=4096) and at twice that (the largest batch the
    benchmarks use), and with no resident expert (every expert int4, the large segments in 256-row tiles):
    routing bit-exact on all tokens, layer output checked on sampled tokens the oracle computes one by one."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C3"], T=T)
    if n_hi is not None:
        wl = dataclasses.replace(wl, n_hi=n_hi)
    print("forward C3: drawing masters", flush=True)
    masters = W.layer_masters(wl, 0, 0)
    x, logits = W.layer_inputs(wl, seed=0)
    ids, w, counts, offsets, perm = dxo.route(logits, wl.k)
    S = counts.astype(np.uint64) << np.uint64(16)
    resident = set(int(e) for e in dxo.select_topn(S, wl.n_hi)) if wl.n_hi else set()
    ctx = B.Context(L=1, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T)
    dev = [LY.bits_to_device(m) for m in masters]
    lw = LY.LayerWeights(ctx, 0, *dev, resident, wl.group)
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    y = torch.empty((wl.T, wl.d), dtype=torch.bfloat16, device="cuda")
    print("forward C3: running", flush=True)
    rb.route(ctx, 0, torch.from_numpy(logits).cuda())
    rb.forward(ctx, 0, LY.bits_to_device(x), y)
    sync()
    assert np.array_equal(rb.ids.cpu().numpy(), ids)
    assert np.array_equal(rb.perm.cpu().numpy(), perm)
    g = np.random.default_rng(0)
    # sampled tokens: random ones plus tokens routed to the largest and to the smallest segments
    big, small = int(np.argmax(counts)), int(np.argmin(np.where(counts > 0, counts, 1 << 30)))
    forced = [int(perm[offsets[big]] // wl.k), int(perm[offsets[big + 1] - 1] // wl.k), int(perm[offsets[small]] // wl.k)]
    tokens = np.unique(np.concatenate([g.choice(wl.T, 40, replace=False), forced])).astype(np.int32)
    wg, wu, wd = masters
    needed = set(int(e) for e in ids[tokens].ravel())
    filler = None
    versions = [None] * wl.E
    for e in needed:
        versions[e] = (dxo.ExpertVersion.bf16(wg[e], wu[e], wd[e]) if e in resident
                       else dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group))
        filler = versions[e]
    versions = [v if v is not None else filler for v in versions]
    y_ref = dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w, tokens=tokens)
    y_gpu = LY.device_to_bits(y)[tokens]
    err = rel_l2(y_gpu, y_ref)
    print("  C3 sampled rel-L2", err, "segments max/min", counts.max(), counts[counts > 0].min(), flush=True)
    assert err <= REL_L2_TOL
    yg = bf16_bits_to_f32(y_gpu).astype(np.float64)
    tok = np.linalg.norm(yg - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    assert tok.max() <= 2 * REL_L2_TOL
    used = assert_elementwise(dxo, y_gpu, y_ref, versions, wl.group, x, ids, w, tokens=tokens, T_call=wl.T)
    print(f"  element-wise: largest error = {used:.2f} of its bound", flush=True)
    del lw
    ctx.close()


@pytest.mark.parametrize("T,one_call", [(32, False), (300, False), (32, True)])
def test_route_and_forward_replay_from_a_captured_graph(B, LY, dxo, T, one_call):
    """dx_route + dx_moe_forward (or the two as one dx_route_forward call) recorded into a HIP graph (the
    decode pass, and the prefill pass with its fork/join over the side streams), replayed several times
    with eager work and synchronisations in between: every replay reproduces the eager result bit for bit."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=4 if T > 64 else 8)
    x, logits = W.layer_inputs(wl, seed=9)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ly = Layer(B, LY, dxo, wl, [0, 2], seed=9)
        ctx, rb = ly.ctx, ly.rb
        xd, ld = LY.bits_to_device(x), torch.from_numpy(logits).cuda()
        y = torch.empty((T, wl.d), dtype=torch.bfloat16, device="cuda")
        rb.route(ctx, 0, ld, T)
        rb.forward(ctx, 0, xd, y, None, T)
        stream.synchronize()
        eager = y.clone()
        ids, w, *_ = dxo.route(logits, wl.k)
        y_ref = dxo.moe_forward(ly.versions, wl.d, wl.f, wl.group, x, ids, w)
        assert rel_l2(LY.device_to_bits(eager), y_ref) <= REL_L2_TOL
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            if one_call:
                rb.route_forward(ctx, 0, ld, xd, y, None, T)
            else:
                rb.route(ctx, 0, ld, T)
                rb.forward(ctx, 0, xd, y, None, T)
        for rep in range(4):
            y.zero_()                                  # eager work between the replays
            rb.perm.zero_()
            stream.synchronize()
            g.replay()
            stream.synchronize()
            assert torch.equal(y, eager), rep
        # new inputs in the same buffers: the replay follows them
        x2, logits2 = W.layer_inputs(wl, seed=10)
        xd.copy_(LY.bits_to_device(x2))
        ld.copy_(torch.from_numpy(logits2).cuda())
        stream.synchronize()
        g.replay()
        stream.synchronize()
        ids2, w2, *_ = dxo.route(logits2, wl.k)
        assert np.array_equal(rb.ids.cpu().numpy()[:T], ids2)
        y_ref2 = dxo.moe_forward(ly.versions, wl.d, wl.f, wl.group, x2, ids2, w2)
        assert rel_l2(LY.device_to_bits(y), y_ref2) <= REL_L2_TOL
        del g
    ly.ctx.close()


# ------------------------------------------- the int4 (high) / int2 (low) precision pair
@pytest.mark.parametrize("rows,K,group", [(128, 256, 64), (768, 2048, 128), (37, 128, 32), (2048, 768, 128)])
def test_int2_quantize_bit_exact(B, LY, dxo, rows, K, group):
    g = np.random.default_rng(rows + K)
    w = (0.02 * g.standard_normal((rows, K))).astype(np.float32)
    w[0, :group] = 0.0
    wb = W.f32_to_bf16_bits(w)
    ctx = B.Context(L=1, E=2, d=64, f=64, top_k=1, group=32, max_tokens=4)
    q = torch.zeros((rows, K // 4), dtype=torch.uint8, device="cuda")
    s = torch.zeros((rows, K // group), dtype=torch.bfloat16, device="cuda")
    ctx.dx_quantize_expert_int2(LY.bits_to_device(wb), rows, K, group, q, s)
    sync()
    q_ref, s_ref = dxo.quantize2(wb, group)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(LY.device_to_bits(s), s_ref)
    ctx.close()


def _quant_pair_layer(B, LY, dxo, wl, hi_ids, seed, T):
    masters = W.layer_masters(wl, seed, 0)
    ctx = B.Context(L=1, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=max(T, 1), hi_fmt=B.DX_FMT_INT4G)
    dev = [LY.bits_to_device(m) for m in masters]
    lw = LY.QuantPairLayerWeights(ctx, 0, *dev, hi_ids, wl.group)
    wg, wu, wd = masters
    versions = [dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) if e in set(hi_ids)
                else dxo.ExpertVersion.int2_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(wl.E)]
    return ctx, lw, versions


@pytest.mark.parametrize("T,E,k,d,f,group,hi_ids", [
    (16, 8, 2, 256, 128, 64, [1, 6]),          # decode, K-chunks of 64 (16 codes per lane and chunk)
    (40, 8, 2, 256, 128, 128, [0]),            # two token tiles, chunks of 128
    (7, 4, 2, 512, 256, 128, []),              # every expert int2
    (33, 16, 4, 2048, 768, 128, [2, 3, 5]),    # the 30B layer's K extents
    (300, 4, 2, 256, 128, 64, [0, 2]),         # prefill-sized: 128-row tiles expand int2 on the way to LDS
    (700, 4, 2, 256, 128, 128, [1]),
    (700, 4, 2, 512, 256, 128, [1, 2]),        # int4 segments of 256 rows and more: 256-row tiles
])
def test_forward_int4_int2_pair(B, LY, dxo, T, E, k, d, f, group, hi_ids):
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k, d=d, f=f, group=group)
    print(f"int4/int2 pair T={T} E={E} k={k} d={d} f={f} g={group} hi={hi_ids}", flush=True)
    x, logits = W.layer_inputs(wl, seed=13)
    ctx, lw, versions = _quant_pair_layer(B, LY, dxo, wl, hi_ids, 13, T)
    fm = ctx.dx_get_formats()[0]
    st = ctx.dx_get_states()[0]
    for e in range(E):
        assert fm[e] == (B.DX_FMT_INT4G if e in hi_ids else B.DX_FMT_INT2G)
        assert st[e] == (B.DX_STATE_RESIDENT_HI if e in hi_ids else B.DX_STATE_RESIDENT_LO)
    rb = LY.RoutingBuffers(T, E, k)
    y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    rb.route(ctx, 0, torch.from_numpy(logits).cuda())
    rb.forward(ctx, 0, LY.bits_to_device(x), y)
    sync()
    ids, w, *_ = dxo.route(logits, k)
    assert np.array_equal(rb.ids.cpu().numpy(), ids)
    y_ref = dxo.moe_forward(versions, d, f, group, x, ids, w)
    err = rel_l2(LY.device_to_bits(y), y_ref)
    print("  rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    ctx.close()


def test_int2_handles_need_a_group_of_64_or_more(B, LY):
    with pytest.raises(B.DxError):
        B.Context(L=1, E=4, d=64, f=64, top_k=2, group=32, max_tokens=4, hi_fmt=B.DX_FMT_INT4G)
    ctx = B.Context(L=1, E=4, d=64, f=64, top_k=2, group=32, max_tokens=4)
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    h = B.make_handle(B.DX_FMT_INT2G, buf, buf, buf, buf, buf, buf)
    with pytest.raises(B.DxError):
        ctx.dx_swap_handle(0, 0, h)
    ctx.close()


@pytest.mark.parametrize("T,E,k,d,f,shared_f,resident", [
    (1, 8, 2, 256, 128, 0, [0, 3]), (7, 8, 2, 256, 128, 0, []), (16, 8, 4, 512, 384, 0, list(range(8))),
    (17, 4, 2, 256, 256, 0, [1]), (32, 4, 3, 512, 384, 0, [0, 2]), (32, 2, 2, 256, 128, 0, [0]),
    (32, 16, 4, 256, 128, 256, [0, 5, 9]), (9, 16, 4, 512, 256, 128, []), (32, 128, 8, 256, 128, 0, list(range(0, 128, 3))),
])
def test_forward_decode_group128_small_shapes(B, LY, dxo, T, E, k, d, f, shared_f, resident):
    """Decode batches of up to 32 tokens with group 128 (K-chunks of 128): one and two token tiles per
    expert, one to three K-chunks, all-bf16 / all-int4 / mixed tables, the shared expert; every token,
    and the same bits on a second run (every sum has a fixed order)."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k, d=d, f=f, group=128, shared_f=shared_f)
    print(f"decode g128 T={T} E={E} k={k} d={d} f={f} shared_f={shared_f}", flush=True)
    x, logits = W.layer_inputs(wl, seed=21)
    shared = W.shared_master(wl, 21, 0) if shared_f else None
    ly = Layer(B, LY, dxo, wl, resident, seed=21, shared=shared)
    y_gpu, y_ref = ly.run(x, logits)
    err = rel_l2(y_gpu, y_ref)
    print("  rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    yg = bf16_bits_to_f32(y_gpu).astype(np.float64)
    tok = np.linalg.norm(yg - y_ref, axis=1) / np.linalg.norm(y_ref, axis=1)
    assert tok.max() <= 2 * REL_L2_TOL
    again, _ = ly.run(x, logits)
    assert np.array_equal(again, y_gpu)                              # a fixed summation order: bit-reproducible
    ly.ctx.close()


@pytest.mark.parametrize("T", [16, 200])
def test_forward_with_a_caller_owned_handle_table(B, LY, dxo, T):
    """dx_moe_forward(handle_table, ...): a table in caller memory (here with the opposite format of
    every expert) is used instead of the context's own; passing the context's table address is the
    same as passing none."""
    import ctypes as C
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T)
    x, logits = W.layer_inputs(wl, seed=17)
    ly = Layer(B, LY, dxo, wl, [0, 2], seed=17)
    ctx, rb = ly.ctx, ly.rb
    xd, ld = LY.bits_to_device(x), torch.from_numpy(logits).cuda()
    y0 = torch.empty((T, wl.d), dtype=torch.bfloat16, device="cuda")
    y1, y2 = torch.empty_like(y0), torch.empty_like(y0)
    rb.route(ctx, 0, ld, T)
    rb.forward(ctx, 0, xd, y0, None, T)
    rb.forward(ctx, 0, xd, y1, ctx.dx_handle_table(0), T)
    # a second set of versions, formats flipped, in a table the caller owns
    flipped = [e for e in range(wl.E) if e not in (0, 2)]
    lw2 = LY.LayerWeights(ctx, 0, *ly.dev, flipped, wl.group, publish=False)
    raw = b"".join(bytes(lw2.handle(e)) for e in range(wl.E))
    assert len(raw) == 64 * wl.E
    table = torch.frombuffer(bytearray(raw), dtype=torch.uint8).cuda()
    rb.forward(ctx, 0, xd, y2, table, T)
    sync()
    assert torch.equal(y0, y1)
    ids, w, *_ = dxo.route(logits, wl.k)
    wg, wu, wd = ly.masters
    v_flip = [dxo.ExpertVersion.bf16(wg[e], wu[e], wd[e]) if e in flipped
              else dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(wl.E)]
    assert rel_l2(LY.device_to_bits(y0), dxo.moe_forward(ly.versions, wl.d, wl.f, wl.group, x, ids, w)) <= REL_L2_TOL
    assert rel_l2(LY.device_to_bits(y2), dxo.moe_forward(v_flip, wl.d, wl.f, wl.group, x, ids, w)) <= REL_L2_TOL
    assert not torch.equal(y0, y2)
    assert np.array_equal(ctx.dx_get_formats()[0], [0 if e in (0, 2) else 1 for e in range(wl.E)])   # own table untouched
    del lw2
    ctx.close()


# --------------------------------------------- routing inside the forward call
def _route_forward_case(B, LY, dxo, wl, resident, seed, shared=None, logits=None, hotness=False):
    """dx_route_forward against the oracle (every routing array bit-exact, y within the bar) and against
    dx_route + dx_moe_forward on the same inputs (the same bits)."""
    x, lg = W.layer_inputs(wl, seed=seed)
    if logits is not None:
        lg = logits
    T = wl.T
    ly = Layer(B, LY, dxo, wl, resident, seed=seed, shared=shared)
    ctx, rb = ly.ctx, ly.rb
    xd, ld = LY.bits_to_device(x), torch.from_numpy(lg).cuda()
    y_sep = torch.empty((T, wl.d), dtype=torch.bfloat16, device="cuda")
    y_one = torch.full_like(y_sep, float("nan"))
    rb.route(ctx, 0, ld, T)
    rb.forward(ctx, 0, xd, y_sep, None, T)
    sync()
    for t in (rb.ids, rb.counts, rb.offsets, rb.perm):
        t.fill_(-1)
    rb.w.fill_(float("nan"))
    rb.route_forward(ctx, 0, ld, xd, y_one, None, T)
    sync()
    ids, w, counts, offsets, perm = dxo.route(lg, wl.k)
    assert np.array_equal(rb.ids.cpu().numpy()[:T], ids)
    assert np.array_equal(rb.counts.cpu().numpy(), counts)
    assert np.array_equal(rb.offsets.cpu().numpy(), offsets)
    assert np.array_equal(rb.perm.cpu().numpy()[:T * wl.k], perm)
    wg = rb.w.cpu().numpy()[:T].astype(np.float64)
    assert np.max(np.abs(wg - w) / np.maximum(w, 1e-30)) < W_TOL or np.max(np.abs(wg - w)) < 1e-7
    assert torch.equal(y_one, y_sep)
    y_ref = dxo.moe_forward(ly.versions, wl.d, wl.f, wl.group, x, ids, w, shared=ly.shared,
                            shared_f=wl.shared_f if ly.shared else 0)
    err = rel_l2(LY.device_to_bits(y_one), y_ref)
    print("  rel-L2", err, flush=True)
    assert err <= REL_L2_TOL
    assert_elementwise(dxo, LY.device_to_bits(y_one), y_ref, ly.versions, wl.group, x, ids, w, shared=ly.shared, T_call=T)
    ctx.close()


@pytest.mark.parametrize("T,E,k,d,f,group,shared_f,resident", [
    (16, 8, 2, 256, 128, 64, 0, [1, 6]),                 # the small configuration
    (1, 8, 2, 256, 128, 128, 0, [0, 3]), (7, 8, 8, 256, 128, 128, 0, []), (17, 4, 2, 256, 256, 128, 0, [1]),
    (32, 128, 8, 256, 128, 128, 0, list(range(0, 128, 3))), (32, 16, 4, 256, 128, 128, 256, [0, 5, 9]),
    (31, 100, 16, 512, 384, 128, 0, list(range(50))), (32, 1, 1, 256, 128, 32, 0, [0]),
    # more than 32 tokens: a second routing pass in the prologue, segments of more than 32 tokens
    (33, 8, 2, 256, 128, 64, 0, [1]), (64, 128, 8, 256, 128, 128, 0, list(range(0, 128, 5))),
    (50, 16, 4, 256, 128, 128, 256, [0, 5, 9]), (63, 4, 4, 256, 128, 128, 0, [2]),
    # more than 128 experts: 32 logits per lane in the routing prologue, two experts per thread in the scans
    (8, 200, 4, 256, 128, 64, 0, [7]), (32, 512, 10, 256, 128, 128, 0, list(range(3, 512, 43))),
    (32, 512, 10, 256, 128, 128, 128, list(range(0, 512, 50))), (64, 300, 16, 256, 128, 128, 0, [0, 299]),
    (33, 511, 10, 256, 128, 64, 128, list(range(100, 140))), (1, 129, 1, 256, 128, 128, 0, []),
    # shapes the self-routing kernel does not take: the call runs the two kernels one after the other
    (65, 8, 2, 256, 128, 64, 0, [1]), (8, 600, 4, 256, 128, 64, 0, [7]), (150, 4, 2, 256, 128, 64, 0, [0]),
    # full-width contractions (8 or 16 K-chunks) at small intermediate sizes, every chunk size, with and
    # without a shared expert, resident sets from none to all
    (32, 16, 4, 2048, 128, 128, 0, [0, 5, 9]), (32, 128, 8, 2048, 128, 128, 0, list(range(0, 128, 4))),
    (17, 12, 3, 2048, 128, 128, 0, []), (5, 8, 2, 2048, 128, 128, 0, list(range(8))), (1, 8, 2, 1024, 128, 128, 0, [2, 3]),
    (32, 16, 4, 2048, 128, 128, 256, [0, 5, 9]), (16, 6, 6, 1024, 128, 128, 128, [4]), (31, 40, 16, 1024, 128, 64, 0, [1, 2, 3, 30]),
    (32, 8, 2, 512, 64, 64, 0, [0, 1]), (9, 8, 3, 512, 64, 32, 64, [6]), (32, 4, 2, 256, 32, 32, 0, [3]),
    (32, 128, 8, 2048, 128, 128, 0, list(range(60, 124))), (3, 128, 8, 2048, 128, 128, 128, [0]),
])
def test_route_forward_matches_oracle_and_separate_calls(B, LY, dxo, T, E, k, d, f, group, shared_f, resident):
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k, d=d, f=f, group=group, shared_f=shared_f)
    print(f"route_forward T={T} E={E} k={k} d={d} f={f} g={group} shared_f={shared_f}", flush=True)
    shared = W.shared_master(wl, 23, 0) if shared_f else None
    _route_forward_case(B, LY, dxo, wl, resident, 23, shared=shared)


def test_route_forward_with_tied_logits(B, LY, dxo):
    """Logits on a coarse grid (many exact ties, both signs of zero): the ids must follow the tie rule."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["C1"], T=32, E=128, k=8, d=256, f=128, group=128)
    g = np.random.default_rng(77)
    logits = np.round(g.standard_normal((wl.T, wl.E)) * 2).astype(np.float32) / 2
    logits[logits == 0] *= np.where(g.random(np.count_nonzero(logits == 0)) < 0.5, -1.0, 1.0).astype(np.float32)
    _route_forward_case(B, LY, dxo, wl, [0, 1, 2, 64, 127], 29, logits=logits)


@pytest.mark.parametrize("case", ["coarse grid", "all equal", "favourites are neighbours", "one lane and ties",
                                  "favourites 64 apart", "few above a sea of equals", "second pass"])
def test_route_forward_wide_layer_threshold_and_its_fallback(B, LY, dxo, case):
    """Layers of more than 128 experts select through a threshold and a short list per lane, and fall back to
    the plain selection when a lane's list overflows: logits built so that both ways run (many exact ties;
    every favourite of a token among 32 neighbouring experts, or among the 32 experts 64 * g + 4 * c + j that
    one lane of the selection holds; a few distinct values above a constant), all of them against the oracle's
    ids, weights and permutation."""
    import dataclasses
    T = 40 if case == "second pass" else 32
    wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=512, k=10, d=256, f=128, group=128)
    g = np.random.default_rng(901)
    if case == "coarse grid":
        logits = np.round(g.standard_normal((T, wl.E)) * 2).astype(np.float32) / 2
        logits[logits == 0] *= np.where(g.random(np.count_nonzero(logits == 0)) < 0.5, -1.0, 1.0).astype(np.float32)
    elif case == "all equal":
        logits = np.full((T, wl.E), 0.25, np.float32)
        logits[1::2] = -3.0
    elif case == "favourites are neighbours":
        logits = g.standard_normal((T, wl.E)).astype(np.float32)
        for t in range(T):       # the ten largest inside one lane's 32 experts, a different lane per token
            lane = t % 16
            logits[t, 32 * lane + g.permutation(32)[:12]] += 8.0
    elif case == "one lane and ties":
        logits = g.standard_normal((T, wl.E)).astype(np.float32)
        for t in range(T):
            own = (64 * np.arange(8)[:, None] + 4 * (t % 16) + np.arange(4)[None, :]).ravel()
            logits[t, own[::2]] = 5.0                               # sixteen equal favourites in one lane's set
    elif case == "favourites 64 apart":
        logits = g.standard_normal((T, wl.E)).astype(np.float32)
        for t in range(T):
            own = (64 * np.arange(8)[:, None] + 4 * (t % 16) + np.arange(4)[None, :]).ravel()
            logits[t, own[g.permutation(32)[:12]]] += 8.0           # the ten largest inside one lane's set
    elif case == "few above a sea of equals":
        logits = np.zeros((T, wl.E), np.float32)
        for t in range(T):
            logits[t, g.permutation(wl.E)[:4]] = g.random(4).astype(np.float32) + 1.0   # 4 < k distinct leaders
    else:
        logits = (g.standard_normal((T, wl.E)) * 1.5).astype(np.float32)
    _route_forward_case(B, LY, dxo, wl, list(range(5, 512, 61)), 31, logits=logits)


def test_route_forward_c2_full_size_and_hotness(B, LY, dxo):
    """The 30B-shaped decode layer through dx_route_forward, with the hotness update inside the call."""
    wl = WORKLOADS["C2"]
    masters = W.layer_masters(wl, 0, 0)
    wg, wu, wd = masters
    resident = list(range(0, wl.E, 4))
    ctx = B.Context(L=2, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T, route_updates_hotness=True)
    dev = [LY.bits_to_device(m) for m in masters]
    lws = [LY.LayerWeights(ctx, l, *dev, resident, wl.group) for l in range(2)]
    versions = [dxo.ExpertVersion.bf16(wg[e], wu[e], wd[e]) if e in set(resident)
                else dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(wl.E)]
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    c = np.zeros((2, wl.E), np.int64)
    y = torch.empty((wl.T, wl.d), dtype=torch.bfloat16, device="cuda")
    for step in range(3):
        for layer in range(2):
            x, lg = W.layer_inputs(wl, seed=0, layer=layer, step=step)
            print(f"route_forward C2 step {step} layer {layer}", flush=True)
            rb.route_forward(ctx, layer, torch.from_numpy(lg).cuda(), LY.bits_to_device(x), y)
            sync()
            ids, w, counts, offsets, perm = dxo.route(lg, wl.k)
            dxo.hotness_update(c[layer], counts)
            assert np.array_equal(rb.ids.cpu().numpy(), ids) and np.array_equal(rb.perm.cpu().numpy(), perm)
            assert np.array_equal(rb.offsets.cpu().numpy(), offsets)
            if step == 2:
                y_ref = dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w)
                err = rel_l2(LY.device_to_bits(y), y_ref)
                print("  rel-L2", err, flush=True)
                assert err <= REL_L2_TOL
                used = assert_elementwise(dxo, LY.device_to_bits(y), y_ref, versions, wl.group, x, ids, w)
                print(f"  element-wise: largest error = {used:.2f} of its bound", flush=True)
    assert np.array_equal(ctx.dx_get_counters(), c)
    del lws
    ctx.close()


def test_route_forward_rejects_bad_arguments(B, LY):
    ctx = B.Context(L=1, E=8, d=64, f=64, top_k=2, group=32, max_tokens=4)
    rb = LY.RoutingBuffers(4, 8, 2)
    buf = torch.zeros(4096, dtype=torch.float32, device="cuda")
    with pytest.raises(B.DxError):
        ctx.dx_route_forward(1, None, buf, buf, 4, rb.ids, rb.w, rb.counts, rb.offsets, rb.perm, buf)   # layer
    with pytest.raises(B.DxError):
        ctx.dx_route_forward(0, None, buf, buf, 5, rb.ids, rb.w, rb.counts, rb.offsets, rb.perm, buf)   # T > max
    with pytest.raises(B.DxError):
        ctx.dx_route_forward(0, None, None, buf, 4, rb.ids, rb.w, rb.counts, rb.offsets, rb.perm, buf)  # null logits
    with pytest.raises(B.DxError):
        ctx.dx_route_forward(0, None, buf, buf, 4, rb.ids, rb.w, rb.counts, rb.offsets, rb.perm, buf)   # no versions published
    ctx.close()


def test_profiling_reports_every_kernel_of_a_forward_call(B, LY, dxo):
    """dx_set_profiling / dx_get_profile: decode calls (separate and as one call) and a prefill call are
    counted, every kernel reports a positive, plausible duration, reading clears the record, and the
    results are the same as without profiling."""
    import dataclasses
    for T, one_call in ((32, False), (32, True), (300, False)):
        wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=8 if T <= 64 else 4)
        x, logits = W.layer_inputs(wl, seed=31)
        ly = Layer(B, LY, dxo, wl, [0, 2], seed=31)
        ctx, rb = ly.ctx, ly.rb
        xd, ld = LY.bits_to_device(x), torch.from_numpy(logits).cuda()
        y0 = torch.empty((T, wl.d), dtype=torch.bfloat16, device="cuda")
        y1 = torch.empty_like(y0)
        rb.route(ctx, 0, ld, T)
        rb.forward(ctx, 0, xd, y0, None, T)
        ctx.dx_set_profiling(True)
        for _ in range(3):
            if one_call:
                rb.route_forward(ctx, 0, ld, xd, y1, None, T)
            else:
                rb.route(ctx, 0, ld, T)
                rb.forward(ctx, 0, xd, y1, None, T)
        p = ctx.dx_get_profile()
        print(f"profile T={T} one_call={one_call}: {p}", flush=True)
        assert p["calls"] == 3
        for key in ("gate_up_ms", "down_ms", "combine_ms"):
            assert 0.0 < p[key] < 3 * 50.0, (key, p[key])          # three calls, far below 50 ms each
        assert p["empty_ms"] >= 0.0
        assert ctx.dx_get_profile()["calls"] == 0                   # reading clears
        ctx.dx_set_profiling(False)
        sync()
        assert torch.equal(y0, y1)
        ctx.close()


def test_route_forward_random_shapes_match_separate_calls(B, LY, dxo):
    """Seeded random decode shapes (tokens, experts, top-k, sizes, group, resident sets, with and without a
    shared expert): dx_route_forward gives the routing arrays of the oracle, bit for bit, and the same y
    bits as dx_route + dx_moe_forward.  (The layer output itself is checked against the oracle in the
    tests above; this one covers many shapes quickly.)"""
    import dataclasses
    g = np.random.default_rng(20251115)
    for case in range(36):
        group = int(g.choice([32, 64, 128]))
        d = group * int(g.integers(1, 9)) if group < 128 else 128 * int(g.choice([1, 2, 4, 8]))
        d = max(d, 64)
        f = group * int(g.integers(1, 5))
        if f % 16:
            f = (f // 16 + 1) * 16
        E = int(g.choice([1, 2, 5, 8, 16, 37, 64, 100, 128]))
        k = int(g.integers(1, min(E, 16) + 1))
        T = int(g.integers(1, 65))
        shared_f = int(g.choice([0, 0, f]))
        n_res = int(g.integers(0, E + 1))
        resident = sorted(g.choice(E, size=n_res, replace=False).tolist())
        wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k, d=d, f=f, group=group, shared_f=shared_f)
        print(f"case {case}: T={T} E={E} k={k} d={d} f={f} g={group} shared_f={shared_f} hi={n_res}", flush=True)
        x, logits = W.layer_inputs(wl, seed=100 + case)
        shared = W.shared_master(wl, 100 + case, 0) if shared_f else None
        ly = Layer(B, LY, dxo, wl, resident, seed=100 + case, shared=shared)
        ctx, rb = ly.ctx, ly.rb
        xd, ld = LY.bits_to_device(x), torch.from_numpy(logits).cuda()
        y_sep = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        y_one = torch.full_like(y_sep, float("nan"))
        rb.route(ctx, 0, ld, T)
        rb.forward(ctx, 0, xd, y_sep, None, T)
        sync()
        w_sep = rb.w.clone()
        for t in (rb.ids, rb.counts, rb.offsets, rb.perm):
            t.fill_(-1)
        rb.route_forward(ctx, 0, ld, xd, y_one, None, T)
        sync()
        ids, w, counts, offsets, perm = dxo.route(logits, k)
        assert np.array_equal(rb.ids.cpu().numpy()[:T], ids)
        assert np.array_equal(rb.counts.cpu().numpy(), counts)
        assert np.array_equal(rb.offsets.cpu().numpy(), offsets)
        assert np.array_equal(rb.perm.cpu().numpy()[:T * k], perm)
        assert torch.equal(rb.w[:T], w_sep[:T])
        assert torch.equal(y_one, y_sep)
        ctx.close()


def test_forward_random_shapes_match_oracle(B, LY, dxo):
    """Seeded random layers in both regimes (1 to 400 tokens; streaming kernels, 128-row and 256-row tiles,
    shapes that fit the tiles and shapes that do not): every layer output within the bar of the oracle's,
    token by token within twice the bar."""
    import dataclasses
    g = np.random.default_rng(20251116)
    for case in range(24):
        group = int(g.choice([32, 64, 128]))
        d = int(g.choice([128, 256, 384, 512])) if group <= 64 else int(g.choice([128, 256, 512]))
        f = int(g.choice([64, 128, 192, 256, 384])) if group <= 64 else int(g.choice([128, 256, 384]))
        if d % group or f % group:
            d, f = 2 * group, 2 * group
        E = int(g.choice([1, 2, 3, 4, 8, 16, 32]))
        k = int(g.integers(1, min(E, 6) + 1))
        T = int(g.choice([1, 5, 31, 32, 33, 64, 100, 128, 129, 200, 257, 400]))
        shared_f = int(g.choice([0, 0, f]))
        n_res = int(g.integers(0, E + 1))
        resident = sorted(g.choice(E, size=n_res, replace=False).tolist())
        wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k, d=d, f=f, group=group, shared_f=shared_f)
        print(f"case {case}: T={T} E={E} k={k} d={d} f={f} g={group} shared_f={shared_f} hi={resident}", flush=True)
        x, logits = W.layer_inputs(wl, seed=200 + case)
        shared = W.shared_master(wl, 200 + case, 0) if shared_f else None
        ly = Layer(B, LY, dxo, wl, resident, seed=200 + case, shared=shared)
        y_gpu, y_ref = ly.run(x, logits)
        err = rel_l2(y_gpu, y_ref)
        print("  rel-L2", err, flush=True)
        assert err <= REL_L2_TOL
        yg = bf16_bits_to_f32(y_gpu).astype(np.float64)
        tok = np.linalg.norm(yg - y_ref, axis=1) / np.maximum(np.linalg.norm(y_ref, axis=1), 1e-30)
        assert tok.max() <= 2 * REL_L2_TOL
        ly.ctx.close()


def test_forward_random_shapes_int4_int2_pair(B, LY, dxo):
    """Seeded random layers of the int4 (high) / int2 (low) pair in both regimes, through dx_route_forward:
    routing bit-exact, layer output within the bar of the oracle's."""
    import dataclasses
    g = np.random.default_rng(20251117)
    for case in range(16):
        group = int(g.choice([64, 128]))
        d = int(g.choice([128, 256, 512]))
        f = int(g.choice([128, 256, 384]))
        E = int(g.choice([2, 4, 8, 16, 32]))
        k = int(g.integers(1, min(E, 6) + 1))
        T = int(g.choice([1, 7, 32, 33, 64, 100, 200, 300]))
        n_hi = int(g.integers(0, E + 1))
        hi_ids = sorted(g.choice(E, size=n_hi, replace=False).tolist())
        wl = dataclasses.replace(WORKLOADS["C1"], T=T, E=E, k=k, d=d, f=f, group=group)
        print(f"case {case}: T={T} E={E} k={k} d={d} f={f} g={group} int4={hi_ids}", flush=True)
        x, logits = W.layer_inputs(wl, seed=300 + case)
        ctx, lw, versions = _quant_pair_layer(B, LY, dxo, wl, hi_ids, 300 + case, T)
        rb = LY.RoutingBuffers(T, E, k)
        y = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        rb.route_forward(ctx, 0, torch.from_numpy(logits).cuda(), LY.bits_to_device(x), y)
        sync()
        ids, w, counts, offsets, perm = dxo.route(logits, k)
        assert np.array_equal(rb.ids.cpu().numpy(), ids) and np.array_equal(rb.perm.cpu().numpy(), perm)
        y_ref = dxo.moe_forward(versions, d, f, group, x, ids, w)
        err = rel_l2(LY.device_to_bits(y), y_ref)
        print("  rel-L2", err, flush=True)
        assert err <= REL_L2_TOL
        del lw
        ctx.close()


def test_probe_read_runs_and_checks_its_arguments(B):
    ctx = B.Context(L=1, E=8, d=64, f=64, top_k=2, group=32, max_tokens=4)
    buf = torch.zeros(8 << 20, dtype=torch.uint8, device="cuda")
    ctx.dx_probe_read(buf, 8 << 20)
    ctx.dx_probe_read(buf, 0)                                   # nothing to read
    sync()
    with pytest.raises(B.DxError):
        ctx.dx_probe_read(buf, (8 << 20) - 1)                   # not whole MiB
    with pytest.raises(B.DxError):
        ctx.dx_probe_read(None, 1 << 20)
    with pytest.raises(B.DxError):
        ctx.dx_probe_read(buf.data_ptr() + 4, 1 << 20)          # misaligned
    ctx.close()
