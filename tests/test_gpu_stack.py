"""GPU parity at the full shapes of the stack workloads: the 80B-shaped layer
(512 experts, top-10, one shared expert, budget rule giving 12 bf16 experts)
and the 30B-shaped stack with hot-set drift, live promotion/demotion and
publication between steps.  Layer outputs are checked against the CPU oracle
with the format map the library reports; integer stages bit for bit."""
import numpy as np
import pytest
import torch

from paper_2511_15015_amd import workloads as W
from paper_2511_15015_amd.workloads import WORKLOADS, bf16_bits_to_f32

pytestmark = pytest.mark.gpu
REL_L2_TOL = 1e-2


@pytest.fixture(scope="module")
def B():
    from paper_2511_15015_amd import binding
    binding.load()
    return binding


@pytest.fixture(scope="module")
def LY():
    from paper_2511_15015_amd import layer
    return layer


def rel_l2(y_bits, y_ref):
    y = bf16_bits_to_f32(y_bits).astype(np.float64)
    return float(np.linalg.norm(y - y_ref) / np.linalg.norm(y_ref))


def test_c4_layer_full_shape_with_budget_rule(B, LY, dxo):
    """One 80B-shaped layer at full size: the 40 GiB stack budget gives 12 bf16 experts per layer,
    chosen from a warm-up window; 500 int4 experts; the shared expert is added with weight 1."""
    wl = WORKLOADS["C4"]
    b_hi, b_lo = dxo.expert_bytes(wl.d, wl.f, wl.group, 0), dxo.expert_bytes(wl.d, wl.f, wl.group, 1)
    b_sh = dxo.expert_bytes(wl.d, wl.shared_f, wl.group, 0)
    stack_budget = 40 * 2 ** 30
    layer_budget = (stack_budget - wl.L * b_sh) // wl.L
    L = 2                                                           # two of the 48 layers are materialised
    ctx = B.Context(L=L, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T, shared_f=wl.shared_f,
                    route_updates_hotness=True)
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    # warm-up window of router traces -> scores -> resident set (GPU and oracle side by side)
    c = np.zeros((L, wl.E), np.int64)
    for step in range(1, 17):
        for layer in range(L):
            _, lg = W.layer_inputs(wl, 0, layer, step)
            rb.route(ctx, layer, torch.from_numpy(lg).cuda())
            _, _, counts, _, _ = dxo.route(lg, wl.k)
            dxo.hotness_update(c[layer], counts)
    S_gpu = ctx.dx_window_end()
    S = np.zeros((L, wl.E), np.uint64)
    for layer in range(L):
        dxo.window_end(S[layer], c[layer], 0)
    assert np.array_equal(S_gpu, S)
    for layer in range(L):
        print(f"C4 layer {layer}: selecting and materialising", flush=True)
        resident = ctx.dx_select_resident(layer, layer_budget)
        n = dxo.budget_capacity(layer_budget, wl.E, b_hi, b_lo)
        assert n == 12 and np.array_equal(resident, dxo.select_topn(S[layer], n))
        assert wl.L * (n * b_hi + (wl.E - n) * b_lo + b_sh) <= stack_budget        # the whole stack fits
        wg, wu, wd = W.device_masters(wl, 0, layer)
        lw = LY.LayerWeights(ctx, layer, wg, wu, wd, resident, wl.group, keep_masters=False)
        g = torch.Generator(device="cuda"); g.manual_seed(1000 + layer)
        shared = [(0.02 * torch.randn(s, generator=g, device="cuda")).to(torch.bfloat16)
                  for s in ((wl.shared_f, wl.d), (wl.shared_f, wl.d), (wl.d, wl.shared_f))]
        ctx.dx_swap_handle(layer, wl.E, B.make_handle(B.DX_FMT_BF16, *shared))
        x, lg = W.layer_inputs(wl, 0, layer, 0)
        y = torch.empty((wl.T, wl.d), dtype=torch.bfloat16, device="cuda")
        rb.route(ctx, layer, torch.from_numpy(lg).cuda())
        rb.forward(ctx, layer, LY.bits_to_device(x), y)
        torch.cuda.synchronize()
        ids, w, counts, offsets, perm = dxo.route(lg, wl.k)
        assert np.array_equal(rb.ids.cpu().numpy(), ids) and np.array_equal(rb.perm.cpu().numpy(), perm)
        res = set(int(e) for e in resident)
        mh = [LY.device_to_bits(m) for m in (wg, wu, wd)]
        versions, filler = [None] * wl.E, None
        for e in np.flatnonzero(counts > 0):
            e = int(e)
            versions[e] = (dxo.ExpertVersion.bf16(*(m[e] for m in mh)) if e in res
                           else dxo.ExpertVersion.int4_from_master(*(m[e] for m in mh), wl.group))
            filler = versions[e]
        versions = [v if v is not None else filler for v in versions]
        sh = dxo.ExpertVersion.bf16(*(LY.device_to_bits(t) for t in shared))
        y_ref = dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w, shared=sh, shared_f=wl.shared_f)
        err = rel_l2(LY.device_to_bits(y), y_ref)
        print(f"  C4 layer {layer}: active {int((counts > 0).sum())} experts, "
              f"{int(sum(counts[e] for e in res))}/{wl.T * wl.k} pairs on bf16 experts, rel-L2 {err:.2e}", flush=True)
        assert err <= REL_L2_TOL
        del lw, wg, wu, wd
    ctx.close()


def test_c5_drift_full_shape_few_layers(B, LY, dxo):
    """30B-shaped layers through the pools with the Zipf permutation re-drawn every window: promotions
    from pinned host masters and on-device demotions on the migration stream, polled between steps
    (no waiting), every checked step replayed by the oracle with the reported format map."""
    wl = WORKLOADS["C5"]
    L, window, n_windows = 2, 6, 3
    b_hi, b_lo = dxo.expert_bytes(wl.d, wl.f, wl.group, 0), dxo.expert_bytes(wl.d, wl.f, wl.group, 1)
    layer_budget = wl.n_hi * b_hi + (wl.E - wl.n_hi) * b_lo
    spare = 8
    ctx = B.Context(L=L, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T,
                    budget_bytes=L * layer_budget, transient_bytes=spare * (b_hi + b_lo), route_updates_hotness=True,
                    window_steps=window)
    ctx.dx_pools_create(L * wl.n_hi + spare, L * (wl.E - wl.n_hi) + spare)
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    y = torch.empty((wl.T, wl.d), dtype=torch.bfloat16, device="cuda")
    masters, pinned, lo_versions, hi_versions = [], [], [], []
    for layer in range(L):
        print(f"C5 layer {layer}: masters, pinned copies, oracle versions", flush=True)
        dev = W.device_masters(wl, 0, layer)
        host = [LY.device_to_bits(m) for m in dev]
        masters.append(host)
        pinned.append([torch.from_numpy(h.view(np.int16)).pin_memory() for h in host])
        hi_versions.append([dxo.ExpertVersion.bf16(*(h[e] for h in host)) for e in range(wl.E)])
        lo_versions.append([None] * wl.E)                        # quantised by the oracle on first use
        # initial state: experts 0..31 bf16 (the all-zero-score selection), the rest int4
        for e in range(wl.E):
            fmt = B.DX_FMT_BF16 if e < wl.n_hi else B.DX_FMT_INT4G
            ctx.dx_expert_install(layer, e, fmt, *(m[e] for m in dev), src_on_device=True)
        del dev
    assert ctx.dx_get_stats()["reserved_bytes"] == L * layer_budget

    def lo_version(layer, e):
        if lo_versions[layer][e] is None:
            lo_versions[layer][e] = dxo.ExpertVersion.int4_from_master(*(h[e] for h in masters[layer]), wl.group)
        return lo_versions[layer][e]

    def check(layer, step, epoch):
        fm = ctx.dx_get_formats()[layer]
        x, lg = W.layer_inputs(wl, 0, layer, step, epoch)
        rb.route(ctx, layer, torch.from_numpy(lg).cuda())
        rb.forward(ctx, layer, LY.bits_to_device(x), y)
        torch.cuda.synchronize()
        ids, w, counts, *_ = dxo.route(lg, wl.k)
        assert np.array_equal(rb.ids.cpu().numpy(), ids)
        versions, filler = [None] * wl.E, None
        for e in np.flatnonzero(counts > 0):
            e = int(e)
            versions[e] = hi_versions[layer][e] if fm[e] == B.DX_FMT_BF16 else lo_version(layer, e)
            filler = versions[e]
        versions = [v if v is not None else filler for v in versions]
        err = rel_l2(LY.device_to_bits(y), dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w))
        assert err <= REL_L2_TOL, (layer, step, err)
        return int(sum(counts[e] for e in np.flatnonzero(fm == B.DX_FMT_BF16)))

    pending = {layer: [] for layer in range(L)}                  # promotions waiting for capacity
    step = 0
    for wdw in range(n_windows):
        epoch = wdw                                              # the hot set is re-drawn every window
        for s in range(window):
            for layer in range(L):
                hot_pairs = check(layer, step, epoch)
                if s in (0, window - 1):
                    print(f"  window {wdw} step {step} layer {layer}: {hot_pairs}/{wl.T * wl.k} pairs on bf16 experts",
                          flush=True)
            # between steps: publish what has completed, then admit waiting promotions
            ctx.dx_migrate_poll()
            for layer in range(L):
                still = []
                for e in pending[layer]:
                    try:
                        ctx.dx_promote_async(layer, e, *(p[e] for p in pinned[layer]))
                    except B.DxError as err:
                        assert err.status in (B.DX_ERR_BUDGET, B.DX_ERR_NOMEM)
                        still.append(e)
                pending[layer] = still
            step += 1
        S = ctx.dx_window_end()
        for layer in range(L):
            target = ctx.dx_select_resident(layer, layer_budget)
            assert np.array_equal(target, dxo.select_topn(S[layer], wl.n_hi))
            pro, dem = ctx.dx_plan_transitions(layer, target)
            for e in dem:
                try:
                    ctx.dx_demote_async(layer, int(e))
                except B.DxError as err:                          # out of transient room: retried next window
                    assert err.status in (B.DX_ERR_BUDGET, B.DX_ERR_NOMEM)
            pending[layer] = [int(e) for e in pro]
        st = ctx.dx_get_stats()
        assert st["peak_reserved_bytes"] <= L * layer_budget + spare * (b_hi + b_lo)
    ctx.dx_migrate_poll(wait=True)
    st = ctx.dx_get_stats()
    print("  C5 stats:", st, flush=True)
    assert st["promotions_published"] > 0 and st["demotions_published"] > 0
    assert st["h2d_bytes"] == st["promotions_issued"] * b_hi
    assert st["quantize_read_bytes"] == st["demotions_issued"] * b_hi
    for layer in range(L):
        check(layer, step, n_windows - 1)
    ctx.close()


def test_c5_churn_with_ema_and_hysteresis(B, LY, dxo):
    """Policy over the drifting 30B-shaped router traces (routing and counting on the GPU, no expert
    weights needed): EMA scores and the selections with hysteresis are bit-exact against the oracle
    in every window; promotions per policy are counted, and the share of the next window's routed
    pairs that lands on the selected set shows what the steadier sets cost."""
    wl = WORKLOADS["C5"]
    L, window, n_windows, redraw = 4, 16, 12, 4
    n = wl.n_hi
    policies = {                                                     # name: (alpha_q16, margin in counts, rank slack)
        "alpha0": (0, 0, 0), "ema": (32768, 0, 0), "ema+margin2": (32768, 2, 0), "ema+margin8": (32768, 8, 0),
        "ema+slack4": (32768, 0, 4), "ema+slack8": (32768, 0, 8),
    }
    ctxs = {a: B.Context(L=L, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T,
                         alpha_q16=a, route_updates_hotness=True, window_steps=window)
            for a in sorted({p[0] for p in policies.values()})}
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    S_ref = {a: np.zeros((L, wl.E), np.uint64) for a in ctxs}
    cur = {name: np.zeros((L, wl.E), np.uint8) for name in policies}
    for name in policies:
        cur[name][:, :n] = 1                                         # the all-zero-score selection
    promotions = {name: 0 for name in policies}
    covered = {name: 0 for name in policies}
    total_pairs = 0
    step = 0
    for wdw in range(n_windows):
        epoch = wdw // redraw
        c = np.zeros((L, wl.E), np.int64)
        for s in range(window):
            for layer in range(L):
                _, lg = W.layer_inputs(wl, 0, layer, step, epoch)
                lgd = torch.from_numpy(lg).cuda()
                for ctx in ctxs.values():
                    rb.route(ctx, layer, lgd)
                _, _, counts, _, _ = dxo.route(lg, wl.k)
                dxo.hotness_update(c[layer], counts)
            step += 1
        if wdw > 0:                                                  # what the sets chosen a window ago caught
            total_pairs += int(c.sum())
            for name in policies:
                covered[name] += int((c * cur[name]).sum())
        for a, ctx in ctxs.items():
            S_gpu = ctx.dx_window_end()
            for layer in range(L):
                cl = c[layer].copy()
                dxo.window_end(S_ref[a][layer], cl, a)
            assert np.array_equal(S_gpu, S_ref[a]), (wdw, a)
        for name, (a, margin, slack) in policies.items():
            for layer in range(L):
                S = S_ref[a][layer]
                if slack:
                    got = B.dx_select_rank_slack(S, cur[name][layer], n, slack)
                    ref = dxo.select_rank_slack(S, cur[name][layer], n, slack)
                else:
                    got = B.dx_select_hysteresis(S, cur[name][layer], n, margin << 16)
                    ref = dxo.select_hysteresis(S, cur[name][layer], n, margin << 16)
                assert np.array_equal(got, ref), (wdw, name, layer)
                new = np.zeros(wl.E, np.uint8)
                new[got] = 1
                pro, dem = dxo.transition_sets(cur[name][layer], new)
                assert len(pro) == len(dem)
                promotions[name] += len(pro)
                cur[name][layer] = new
    for name in policies:
        print(f"  C5 policy {name:12s}: {promotions[name]:5d} promotions over {n_windows} windows x {L} layers, "
              f"{100.0 * covered[name] / total_pairs:5.1f} % of routed pairs on the selected set", flush=True)
    assert promotions["ema+margin2"] <= promotions["ema"] and promotions["ema+margin8"] <= promotions["ema+margin2"]
    assert promotions["ema+slack8"] <= promotions["ema+slack4"] <= promotions["ema"]
    for ctx in ctxs.values():
        ctx.close()


@pytest.mark.parametrize("T", [32, 1536])
def test_phi35_shaped_layer(B, LY, dxo, T):
    """16 experts of 4096 x 6400, top-2, 4 of them bf16: the decode batch runs the streaming kernels on
    K = 4096 and 6400 (more K-chunks than wavefronts), the prefill batch the 256-row and 128-row tile
    kernels with 50 column tiles; sampled tokens against the oracle, routing bit-exact."""
    import dataclasses
    wl = dataclasses.replace(WORKLOADS["X1"], T=T)
    print(f"X1 T={T}: drawing masters", flush=True)
    dev = W.device_masters(wl, 0, 0)
    x, lg = W.layer_inputs(wl, 0, 0, 0)
    ids, w, counts, offsets, perm = dxo.route(lg, wl.k)
    resident = set(int(e) for e in dxo.select_topn(counts.astype(np.uint64) << np.uint64(16), wl.n_hi))
    ctx = B.Context(L=1, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=T)
    lw = LY.LayerWeights(ctx, 0, *dev, resident, wl.group)
    rb = LY.RoutingBuffers(T, wl.E, wl.k)
    y = torch.empty((T, wl.d), dtype=torch.bfloat16, device="cuda")
    print(f"X1 T={T}: running, segments {counts.tolist()}", flush=True)
    rb.route(ctx, 0, torch.from_numpy(lg).cuda())
    rb.forward(ctx, 0, LY.bits_to_device(x), y)
    torch.cuda.synchronize()
    assert np.array_equal(rb.ids.cpu().numpy(), ids) and np.array_equal(rb.perm.cpu().numpy(), perm)
    g = np.random.default_rng(1)
    tokens = np.sort(g.choice(T, 6, replace=False)).astype(np.int32)
    needed = sorted(set(int(e) for e in ids[tokens].ravel()))
    versions, filler = [None] * wl.E, None
    for e in needed:
        host = [LY.device_to_bits(m[e]) for m in dev]
        versions[e] = (dxo.ExpertVersion.bf16(*host) if e in resident
                       else dxo.ExpertVersion.int4_from_master(*host, wl.group))
        filler = versions[e]
    versions = [v if v is not None else filler for v in versions]
    y_ref = dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w, tokens=tokens)
    err = rel_l2(LY.device_to_bits(y)[tokens], y_ref)
    print(f"  X1 T={T} rel-L2 {err:.3e} over tokens {tokens.tolist()}", flush=True)
    assert err <= REL_L2_TOL
    del lw
    ctx.close()


def test_c4_layer_with_the_int4_int2_pair_under_a_budget(B, LY, dxo):
    """The 80B-shaped layer with int4 as the high tier and int2 as the low one: a 24 GiB stack budget
    leaves room for a three-digit number of int4 experts per layer next to the int2 rest; the shared
    expert stays bf16.  Budget rule, selection and the layer output against the oracle."""
    wl = WORKLOADS["C4"]
    b_hi, b_lo = dxo.expert_bytes(wl.d, wl.f, wl.group, dxo.FMT_INT4), dxo.expert_bytes(wl.d, wl.f, wl.group, dxo.FMT_INT2)
    b_sh = dxo.expert_bytes(wl.d, wl.shared_f, wl.group, 0)
    assert b_hi == B.dx_expert_bytes(wl.d, wl.f, wl.group, B.DX_FMT_INT4G)
    assert b_lo == B.dx_expert_bytes(wl.d, wl.f, wl.group, B.DX_FMT_INT2G)
    stack_budget = 24 * 2 ** 30
    layer_budget = (stack_budget - wl.L * b_sh) // wl.L
    ctx = B.Context(L=1, E=wl.E, d=wl.d, f=wl.f, top_k=wl.k, group=wl.group, max_tokens=wl.T, shared_f=wl.shared_f,
                    route_updates_hotness=True, hi_fmt=B.DX_FMT_INT4G)
    rb = LY.RoutingBuffers(wl.T, wl.E, wl.k)
    c = np.zeros(wl.E, np.int64)
    for step in range(1, 17):
        _, lg = W.layer_inputs(wl, 0, 0, step)
        rb.route(ctx, 0, torch.from_numpy(lg).cuda())
        dxo.hotness_update(c, dxo.route(lg, wl.k)[2])
    S_gpu = ctx.dx_window_end()[0]
    S = np.zeros(wl.E, np.uint64)
    dxo.window_end(S, c, 0)
    assert np.array_equal(S_gpu, S)
    resident = ctx.dx_select_resident(0, layer_budget)              # uses the pair's b_hi / b_lo
    n = dxo.budget_capacity(layer_budget, wl.E, b_hi, b_lo)
    assert 100 < n < wl.E and np.array_equal(resident, dxo.select_topn(S, n))
    assert wl.L * (n * b_hi + (wl.E - n) * b_lo + b_sh) <= stack_budget
    assert wl.L * ((n + 1) * b_hi + (wl.E - n - 1) * b_lo + b_sh) > stack_budget
    print(f"C4 int4/int2: n = {n} int4 experts per layer", flush=True)
    wg, wu, wd = W.device_masters(wl, 0, 0)
    lw = LY.QuantPairLayerWeights(ctx, 0, wg, wu, wd, resident, wl.group)
    g = torch.Generator(device="cuda"); g.manual_seed(77)
    shared = [(0.02 * torch.randn(s, generator=g, device="cuda")).to(torch.bfloat16)
              for s in ((wl.shared_f, wl.d), (wl.shared_f, wl.d), (wl.d, wl.shared_f))]
    ctx.dx_swap_handle(0, wl.E, B.make_handle(B.DX_FMT_BF16, *shared))
    x, lg = W.layer_inputs(wl, 0, 0, 0)
    y = torch.empty((wl.T, wl.d), dtype=torch.bfloat16, device="cuda")
    rb.route(ctx, 0, torch.from_numpy(lg).cuda())
    rb.forward(ctx, 0, LY.bits_to_device(x), y)
    torch.cuda.synchronize()
    ids, w, counts, offsets, perm = dxo.route(lg, wl.k)
    assert np.array_equal(rb.ids.cpu().numpy(), ids)
    res = set(int(e) for e in resident)
    mh = [LY.device_to_bits(m) for m in (wg, wu, wd)]
    versions, filler = [None] * wl.E, None
    for e in np.flatnonzero(counts > 0):
        e = int(e)
        make = dxo.ExpertVersion.int4_from_master if e in res else dxo.ExpertVersion.int2_from_master
        versions[e] = make(*(m[e] for m in mh), wl.group)
        filler = versions[e]
    versions = [v if v is not None else filler for v in versions]
    sh = dxo.ExpertVersion.bf16(*(LY.device_to_bits(t) for t in shared))
    y_ref = dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w, shared=sh, shared_f=wl.shared_f)
    err = rel_l2(LY.device_to_bits(y), y_ref)
    on_hi = int(sum(counts[e] for e in res))
    print(f"  C4 int4/int2: {on_hi}/{wl.T * wl.k} pairs on int4 experts, rel-L2 {err:.2e}", flush=True)
    assert err <= REL_L2_TOL
    del lw
    ctx.close()


def _oracle_versions(dxo, B, LY, master_bits, formats, counts, group):
    """Oracle-side versions of the activated experts under a format map (others: any placeholder)."""
    versions, filler = [None] * len(formats), None
    for e in np.flatnonzero(counts > 0):
        e = int(e)
        m = master_bits(e)
        versions[e] = (dxo.ExpertVersion.bf16(*m) if formats[e] == B.DX_FMT_BF16
                       else dxo.ExpertVersion.int4_from_master(*m, group))
        filler = versions[e]
    return [v if v is not None else filler for v in versions]


def test_c4_stack_48_layers_under_40_gib(B, LY, dxo):
    """The 80B-shaped stack as the configuration states it: 48 layers in one context, a 40 GiB expert
    budget for the whole stack, the budget rule and dx_select_resident per layer (12 bf16 experts each),
    a step = one dx_route_forward per layer.  Selections of every layer against the oracle; the layer
    output of layers 0, 23 and 47 against the oracle (norm and element-wise), routing bit for bit."""
    from paper_2511_15015_amd import stack as ST
    from tests.bounds import assert_elementwise
    wl = WORKLOADS["C4"]
    L, window, budget = wl.L, 8, 40 * 2 ** 30
    checked = [0, 23, 47]
    stk = ST.StaticStack(wl, L, 0, budget, window, keep_masters_of=checked,
                         progress=lambda m: print("  C4 stack:", m, flush=True))
    b_hi, b_lo = dxo.expert_bytes(wl.d, wl.f, wl.group, 0), dxo.expert_bytes(wl.d, wl.f, wl.group, 1)
    b_sh = dxo.expert_bytes(wl.d, wl.shared_f, wl.group, 0)
    assert stk.layer_budget == (budget - L * b_sh) // L
    n = dxo.budget_capacity(stk.layer_budget, wl.E, b_hi, b_lo)
    assert n == 12
    # scores and selections of all 48 layers from the same warm-up traces on the oracle side
    for layer in range(L):
        c = np.zeros(wl.E, np.int64)
        wr = W.router_matrix(wl, 0, layer)
        for step in range(1, window + 1):
            lg = W.router_logits(wl, W.activations(wl, 0, layer, step), wr, 0, layer)
            dxo.hotness_update(c, dxo.route(lg, wl.k)[2])
        S = np.zeros(wl.E, np.uint64)
        dxo.window_end(S, c, 0)
        assert np.array_equal(stk.scores[layer], S), layer
        assert np.array_equal(stk.resident[layer], dxo.select_topn(S, n)), layer
    held = stk.bytes_held()
    assert held == L * (n * b_hi + (wl.E - n) * b_lo + b_sh) and held <= budget
    print(f"  C4 stack: {held / 2**30:.2f} GiB held of {budget / 2**30:.0f} GiB", flush=True)
    for _ in range(2):                                            # whole-stack steps
        stk.step()
    torch.cuda.synchronize()
    for layer in checked:
        stk.layer_call(layer)
        torch.cuda.synchronize()
        x, lg = stk.x_bits[layer], stk.logits_host[layer]
        ids, w, counts, offsets, perm = dxo.route(lg, wl.k)
        assert np.array_equal(stk.rb.ids.cpu().numpy(), ids) and np.array_equal(stk.rb.perm.cpu().numpy(), perm)
        mh = [LY.device_to_bits(m) for m in stk.masters[layer]]
        fm = stk.ctx.dx_get_formats()[layer]
        assert set(np.flatnonzero(fm == B.DX_FMT_BF16)) == set(int(e) for e in stk.resident[layer])
        versions = _oracle_versions(dxo, B, LY, lambda e: tuple(m[e] for m in mh), fm, counts, wl.group)
        sh = dxo.ExpertVersion.bf16(*(LY.device_to_bits(t) for t in stk.shared[layer]))
        y_ref = dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w, shared=sh, shared_f=wl.shared_f)
        yb = LY.device_to_bits(stk.y)
        err = rel_l2(yb, y_ref)
        used = assert_elementwise(dxo, yb, y_ref, versions, wl.group, x, ids, w, shared=sh)
        print(f"  C4 stack layer {layer}: rel-L2 {err:.2e}, element-wise {used:.2f} of the bound", flush=True)
        assert err <= REL_L2_TOL
    stk.close()


def test_c5_schedule_as_stated_on_48_layers(B, LY, dxo):
    """The drifting stack with the stated schedule (48 layers, 256-step hotness window, the Zipf
    permutation re-drawn every 256 steps, windowed counts, plain top-n) for three windows -- the stated
    run is eight; layers 0, 23 and 47 at the first step, around every window boundary and at the last
    step are replayed by the oracle with the format map the library reported for that call."""
    from paper_2511_15015_amd import stack as ST
    from tests.bounds import assert_elementwise
    wl = WORKLOADS["C5"]
    L, window, redraw, steps = wl.L, wl.window_steps, wl.redraw_every, 3 * wl.window_steps
    assert (L, window, redraw) == (48, 256, 256)
    stk = ST.DriftStack(wl, L, 0, window, n_epochs=steps // redraw, progress=lambda m: print("  C5:", m, flush=True))
    layers = [0, 23, 47]
    at = sorted({0, steps - 1} | {w * window + o for w in range(1, steps // window) for o in (-1, 0, 1)})
    print(f"  C5: running {steps} steps, sampling steps {at}", flush=True)
    res, kept = stk.run(steps, redraw, samples={(s, l) for s in at for l in layers}, time_steps=False)
    print("  C5:", {k: v for k, v in res.items() if k != "steps_to_drain_after_window_end"}, flush=True)
    assert len(kept) == len(at) * len(layers)
    assert res["promotions"] > 0 and res["demotions"] > 0
    assert res["peak_reserved_bytes"] <= stk.budget_cap()
    seen_mixed = 0
    for smp in kept:
        layer, b, ep = smp["layer"], smp["batch"], smp["epoch"]
        x, lg = stk.x_bits[layer][b], stk.logits_host[ep][layer][b]
        ids, w, counts, offsets, perm = dxo.route(lg, wl.k)
        assert np.array_equal(smp["ids"].cpu().numpy(), ids) and np.array_equal(smp["perm"].cpu().numpy(), perm)
        fm = smp["formats"]
        assert int((fm == B.DX_FMT_BF16).sum()) <= wl.n_hi
        seen_mixed += int(not np.array_equal(np.flatnonzero(fm == B.DX_FMT_BF16), np.arange(wl.n_hi)))
        versions = _oracle_versions(dxo, B, LY, lambda e: stk.master_bits(layer, e), fm, counts, wl.group)
        y_ref = dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w)
        yb = LY.device_to_bits(smp["y"])
        err = rel_l2(yb, y_ref)
        assert err <= REL_L2_TOL, (smp["step"], layer, err)
        assert_elementwise(dxo, yb, y_ref, versions, wl.group, x, ids, w)
    assert seen_mixed > 0                                         # the resident sets did move
    stk.close()
