"""Pins for the CPU oracle: it is checked against things other than itself --
library routines (numpy / scipy / torch CPU) on special cases, brute force in
pure Python on tiny inputs, closed forms, the sizes the paper prints in its
model table, and invariants the method must satisfy.  No GPU needed."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from paper_2511_15015_amd import workloads as wlmod
from paper_2511_15015_amd.workloads import WORKLOADS, bf16_bits_to_f32, f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits(a):
    return f32_to_bf16_bits(np.asarray(a, np.float32))


# ---------------------------------------------------------------- input format
def test_bf16_conversion_matches_torch():
    g = np.random.default_rng(1)
    a = np.concatenate([g.standard_normal(4096).astype(np.float32) * 10 ** g.uniform(-6, 6, 4096).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, -1e-40], np.float32)])
    ours = f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(bf16_bits_to_f32(ours), torch.from_numpy(a).to(torch.bfloat16).float().numpy())


# ---------------------------------------------------------------------- top-k
def _brute_topk(logits, k):
    T, E = logits.shape
    ids = np.empty((T, k), np.int32)
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-float(logits[t, e]), e))
        ids[t] = order[:k]
    return ids


@pytest.mark.parametrize("T,E,k", [(16, 8, 2), (7, 128, 8), (5, 512, 10), (3, 4, 4), (1, 1, 1)])
def test_topk_ids_brute_force(dxo, T, E, k):
    g = np.random.default_rng(T * 1000 + E)
    logits = g.standard_normal((T, E)).astype(np.float32)
    ids, w = dxo.topk(logits, k)
    assert np.array_equal(ids, _brute_topk(logits, k))
    # library routine: torch.topk values (ids may differ only under ties; none here)
    tv, ti = torch.topk(torch.from_numpy(logits), k, dim=1)
    assert np.array_equal(ids, ti.numpy().astype(np.int32))


def test_topk_ties_go_to_lower_index(dxo):
    logits = np.zeros((3, 8), np.float32)                 # all equal -> 0,1,2
    logits[1, [5, 2, 7]] = 1.0                            # three-way tie at the top
    logits[2] = [0.0, -0.0, 3.0, 3.0, -1.0, 0.0, 3.0, 2.0]   # -0.0 == +0.0
    ids, w = dxo.topk(logits, 4)
    assert ids[0].tolist() == [0, 1, 2, 3]
    assert ids[1].tolist() == [2, 5, 7, 0]
    assert ids[2].tolist() == [2, 3, 6, 7]
    assert np.allclose(w[0], 0.25)
    assert np.array_equal(ids, _brute_topk(logits, 4))


def test_topk_weights_softmax_identities(dxo):
    g = np.random.default_rng(7)
    logits = (3 * g.standard_normal((9, 32))).astype(np.float32)
    k = 5
    ids, w = dxo.topk(logits, k)
    assert np.allclose(w.sum(1), 1.0, atol=1e-14)
    # softmax over all experts, keep the top-k, renormalise: same numbers
    full = scipy.special.softmax(logits.astype(np.float64), axis=1)
    picked = np.take_along_axis(full, ids.astype(np.int64), 1)
    assert np.allclose(w, picked / picked.sum(1, keepdims=True), rtol=1e-12)
    # k = E: the weights are the full softmax, sorted by logit
    idsE, wE = dxo.topk(logits, 32)
    assert np.allclose(wE, np.take_along_axis(full, idsE.astype(np.int64), 1), rtol=1e-12)
    # descending order of the selected logits
    sel = np.take_along_axis(logits, ids.astype(np.int64), 1)
    assert np.all(sel[:, :-1] >= sel[:, 1:])


# ---------------------------------------------------------------- permutation
@pytest.mark.parametrize("T,E,k", [(16, 8, 2), (32, 128, 8), (200, 16, 4), (0, 8, 2)])
def test_permutation_is_stable_counting_sort(dxo, T, E, k):
    g = np.random.default_rng(E + T)
    ids = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32) if T else np.empty((0, k), np.int32)
    counts, offsets, perm = dxo.permute(ids, E)
    assert np.array_equal(counts, np.bincount(ids.ravel(), minlength=E))
    assert offsets[0] == 0 and offsets[E] == T * k
    assert np.array_equal(offsets[1:], np.cumsum(counts))
    assert np.array_equal(perm, np.argsort(ids.ravel(), kind="stable").astype(np.int32))
    assert sorted(perm.tolist()) == list(range(T * k))                       # bijection
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(ids.ravel()[seg] == e) and np.all(np.diff(seg) > 0)


def test_permute_rejects_bad_id(dxo):
    with pytest.raises(ValueError):
        dxo.permute(np.array([[0, 9]], np.int32), 8)


# ------------------------------------------------------------------ quantizer
def _signed_nibbles(q):
    lo = (q & 0xF).astype(np.int16)
    hi = (q >> 4).astype(np.int16)
    out = np.empty(q.shape[:-1] + (q.shape[-1] * 2,), np.int16)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return np.where(out >= 8, out - 16, out)


def test_quantizer_half_even_and_packing(dxo):
    # absmax 7 -> scale exactly 1; values with exact .5 fractions are bf16-representable
    row = np.zeros(64, np.float32)
    vals = [7.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, -3.5, -7.0, 6.5, -6.5, 0.25, -0.75, 4.5, 5.5]
    row[:len(vals)] = vals
    q, s = dxo.quantize(_bits(row)[None, :], 64)
    assert bf16_bits_to_f32(s)[0, 0] == 1.0
    codes = _signed_nibbles(q)[0]
    assert codes[:len(vals)].tolist() == [7, 0, 2, 2, 4, 0, -2, -2, -4, -7, 6, -6, 0, -1, 4, 6]
    # byte i = element 2i in the low nibble, element 2i+1 in the high nibble, two's complement
    assert q[0, 0] == (7 & 0xF) | ((0 & 0xF) << 4)
    assert q[0, 3] == ((-2) & 0xF) | (((-2) & 0xF) << 4)
    assert q[0, 4] == ((-4) & 0xF) | (((-7) & 0xF) << 4)


def test_quantizer_zero_group_and_grid_roundtrip(dxo):
    g = np.random.default_rng(3)
    rows, K, group = 6, 256, 64
    # weights already on the grid: w = q*s with max|q| = 7 and s a power of two times a bf16 value
    codes = g.integers(-7, 8, (rows, K)).astype(np.float32)
    codes[:, ::group] = 7.0                                    # make absmax/7 land on s exactly
    s_true = (2.0 ** g.integers(-9, -3, (rows, K // group))).astype(np.float32)
    w = codes * np.repeat(s_true, group, axis=1)
    w[2, 64:128] = 0.0                                         # an all-zero group
    wb = _bits(w)
    assert np.array_equal(bf16_bits_to_f32(wb), w)             # exactly representable
    q, s = dxo.quantize(wb, group)
    deq = dxo.dequantize(q, s, group)
    assert np.array_equal(deq, w)
    assert bf16_bits_to_f32(s)[2, 1] == 0.0 and np.all(q[2, 32:64] == 0)


@pytest.mark.parametrize("group", [64, 128])
def test_quantizer_half_step_bound_and_range(dxo, group):
    g = np.random.default_rng(group)
    w = (0.02 * g.standard_normal((48, 512))).astype(np.float32)
    w[5] *= 1e-3
    w[6] *= 1e3
    wb = _bits(w)
    wv = bf16_bits_to_f32(wb).astype(np.float64)
    q, s = dxo.quantize(wb, group)
    sv = np.repeat(bf16_bits_to_f32(s).astype(np.float64), group, axis=1)
    codes = _signed_nibbles(q).astype(np.float64)
    assert codes.min() >= -8 and codes.max() <= 7
    deq = dxo.dequantize(q, s, group).astype(np.float64)
    assert np.array_equal(deq, codes * sv)
    # |dequant(quant(w)) - w| <= s/2, with one fp32 ulp of the quotient allowed for the rounded divide
    slack = np.abs(wv) * 2.0 ** -23
    assert np.all(np.abs(deq - wv) <= sv / 2 + slack)
    # scale is bf16(absmax/7): within half a bf16 ulp of the exact quotient
    amax = np.abs(wv).reshape(48, -1, group).max(2)
    exact = amax / 7.0
    assert np.all(np.abs(bf16_bits_to_f32(s).astype(np.float64) - exact) <= exact * 2.0 ** -8)
    # the group's absmax element always maps to +-7
    assert np.all(np.abs(codes).reshape(48, -1, group).max(2) == 7)


def test_quantizer_numpy_fp32_cross_check(dxo):
    g = np.random.default_rng(11)
    group = 128
    wb = _bits(0.02 * g.standard_normal((32, 1024)))
    q, s = dxo.quantize(wb, group)
    w = bf16_bits_to_f32(wb).reshape(32, -1, group)
    sc = bf16_bits_to_f32(f32_to_bf16_bits(np.abs(w).max(2) / np.float32(7.0)))
    codes = np.clip(np.rint(w / sc[:, :, None]), -8, 7).astype(np.int16).reshape(32, -1)
    assert np.array_equal(bf16_bits_to_f32(s), sc)
    assert np.array_equal(_signed_nibbles(q), codes)


def _signed_crumbs(q):
    out = np.empty(q.shape[:-1] + (q.shape[-1] * 4,), np.int16)
    for h in range(4):
        out[..., h::4] = (q >> (2 * h)) & 0x3
    return np.where(out >= 2, out - 4, out)


def test_int2_quantizer_codes_packing_and_bounds(dxo):
    # absmax 1 -> scale exactly 1; .5 ties go to the even code; the range is {-1, 0, 1} (q_max = 1)
    row = np.zeros(32, np.float32)
    vals = [1.0, 0.5, 0.75, -0.5, -0.75, -1.0, 0.25, 0.0]
    row[:len(vals)] = vals
    q, s = dxo.quantize2(_bits(row)[None, :], 32)
    assert bf16_bits_to_f32(s)[0, 0] == 1.0
    assert _signed_crumbs(q)[0, :len(vals)].tolist() == [1, 0, 1, 0, -1, -1, 0, 0]
    # byte i holds elements 4i .. 4i+3, element 4i in the two low bits, two's complement
    assert q[0, 0] == (1 & 3) | ((0 & 3) << 2) | ((1 & 3) << 4) | ((0 & 3) << 6)
    assert q[0, 1] == ((-1) & 3) | (((-1) & 3) << 2)
    g = np.random.default_rng(41)
    group = 64
    wb = _bits(0.02 * g.standard_normal((24, 512)))
    wv = bf16_bits_to_f32(wb).astype(np.float64)
    q, s = dxo.quantize2(wb, group)
    sv = np.repeat(bf16_bits_to_f32(s).astype(np.float64), group, axis=1)
    codes = _signed_crumbs(q).astype(np.float64)
    assert set(np.unique(codes).tolist()) <= {-1.0, 0.0, 1.0}
    deq = dxo.dequantize2(q, s, group).astype(np.float64)
    assert np.array_equal(deq, codes * sv)
    assert np.all(np.abs(deq - wv) <= sv / 2 + np.abs(wv) * 2.0 ** -23)      # half a step
    amax = np.abs(wv).reshape(24, -1, group).max(2)
    assert np.array_equal(bf16_bits_to_f32(s).astype(np.float64), amax)      # absmax / 1 is already bf16
    assert np.all(np.abs(codes).reshape(24, -1, group).max(2) == 1)          # the absmax element maps to +-1
    # independent numpy fp32 formulation
    w3 = bf16_bits_to_f32(wb).reshape(24, -1, group)
    sc = np.abs(w3).max(2)
    ref = np.clip(np.rint(w3 / sc[:, :, None]), -2, 1).astype(np.int16).reshape(24, -1)
    assert np.array_equal(_signed_crumbs(q), ref)
    # on-grid weights come back exactly; an all-zero group has scale 0 and codes 0
    c = g.integers(-1, 2, (4, 128)).astype(np.float32)
    c[:, ::group] = 1.0
    w = c * np.repeat((2.0 ** g.integers(-8, -2, (4, 2))).astype(np.float32), group, axis=1)
    w[1, :group] = 0.0
    q, s = dxo.quantize2(_bits(w), group)
    assert np.array_equal(dxo.dequantize2(q, s, group), w)
    assert bf16_bits_to_f32(s)[1, 0] == 0.0 and np.all(q[1, :group // 4] == 0)
    with pytest.raises(ValueError):
        dxo.quantize2(np.zeros((2, 96), np.uint16), 64)


def test_int2_experts_in_the_layer_equal_dense_on_dequantised_weights(dxo):
    """A table of int4 and int2 experts (the second precision pair): the layer output is the dense MoE
    on the dequantised matrices; byte sizes follow the format."""
    x, ids, w, masters, versions, (T, d, f, E, k, group) = _tiny_layer(dxo, 24, n_int4=2)
    versions = [dxo.ExpertVersion.int2_from_master(*masters[e], group) if e % 2 else
                dxo.ExpertVersion.int4_from_master(*masters[e], group) for e in range(E)]
    y = dxo.moe_forward(versions, d, f, group, x, ids, w)
    ref = np.zeros((T, d))
    for t in range(T):
        for j in range(k):
            e = int(ids[t, j])
            a = versions[e].arrays
            deq = dxo.dequantize2 if versions[e].fmt == dxo.FMT_INT2 else dxo.dequantize
            mats = [deq(a[i], a[3 + i], group) for i in range(3)]
            ref[t] += w[t, j] * _torch_expert(*mats, bf16_bits_to_f32(x[t:t + 1])).numpy()[0]
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)
    assert dxo.expert_bytes(2048, 512, 128, dxo.FMT_INT2) == 3 * 2048 * 512 // 4 + 2 * 3 * 2048 * 512 // 128
    assert dxo.expert_bytes(2048, 512, 128, dxo.FMT_INT4) == 3 * 2048 * 512 // 2 + 2 * 3 * 2048 * 512 // 128


def test_quantizer_rejects_bad_shapes(dxo):
    wb = np.zeros((2, 96), np.uint16)
    with pytest.raises(ValueError):
        dxo.quantize(wb, 64)


# ---------------------------------------------------------------- layer output
def _torch_expert(wg, wu, wd, x):
    """Library-routine SwiGLU MLP in fp64: W_down(silu(W_gate x) * (W_up x))."""
    Wg, Wu, Wd, X = (torch.from_numpy(np.asarray(a, np.float64)) for a in (wg, wu, wd, x))
    return (torch.nn.functional.silu(X @ Wg.T) * (X @ Wu.T)) @ Wd.T


def _tiny_layer(dxo, seed, T=6, d=32, f=16, E=4, k=2, group=16, n_int4=2):
    g = np.random.default_rng(seed)
    x = _bits(g.standard_normal((T, d)))
    logits = g.standard_normal((T, E)).astype(np.float32)
    masters = [tuple(_bits(0.3 * g.standard_normal(s)) for s in ((f, d), (f, d), (d, f))) for _ in range(E)]
    versions = []
    for e, m in enumerate(masters):
        versions.append(dxo.ExpertVersion.int4_from_master(*m, group) if e < n_int4 else dxo.ExpertVersion.bf16(*m))
    ids, w = dxo.topk(logits, k)
    return x, ids, w, masters, versions, (T, d, f, E, k, group)


def test_single_expert_equals_library_mlp(dxo):
    g = np.random.default_rng(5)
    T, d, f = 5, 64, 48
    x = _bits(g.standard_normal((T, d)))
    m = tuple(_bits(0.1 * g.standard_normal(s)) for s in ((f, d), (f, d), (d, f)))
    ids = np.zeros((T, 1), np.int32)
    w = np.ones((T, 1), np.float64)
    y = dxo.moe_forward([dxo.ExpertVersion.bf16(*m)], d, f, 16, x, ids, w)
    ref = _torch_expert(*(bf16_bits_to_f32(a) for a in m), bf16_bits_to_f32(x)).numpy()
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-14)


def test_all_bf16_table_equals_dense_moe(dxo):
    x, ids, w, masters, _, (T, d, f, E, k, group) = _tiny_layer(dxo, 21)
    versions = [dxo.ExpertVersion.bf16(*m) for m in masters]
    y = dxo.moe_forward(versions, d, f, group, x, ids, w)
    # dense formulation: every expert on every token, combined with a [T,E] weight matrix
    dense_w = np.zeros((T, E))
    for t in range(T):
        dense_w[t, ids[t]] = w[t]
    outs = np.stack([_torch_expert(*(bf16_bits_to_f32(a) for a in m), bf16_bits_to_f32(x)).numpy() for m in masters], 1)
    ref = np.einsum("te,ted->td", dense_w, outs)
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)


def test_mixed_table_equals_dense_on_dequantised_weights(dxo):
    x, ids, w, masters, versions, (T, d, f, E, k, group) = _tiny_layer(dxo, 22, n_int4=3)
    y = dxo.moe_forward(versions, d, f, group, x, ids, w)
    ref = np.zeros((T, d))
    for t in range(T):
        for j in range(k):
            e = int(ids[t, j])
            if versions[e].fmt == dxo.FMT_INT4:
                a = versions[e].arrays
                mats = [dxo.dequantize(a[i], a[3 + i], group) for i in range(3)]
            else:
                mats = [bf16_bits_to_f32(a) for a in masters[e]]
            ref[t] += w[t, j] * _torch_expert(*mats, bf16_bits_to_f32(x[t:t + 1])).numpy()[0]
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)
    # quantised experts really differ from their masters
    y_hi = dxo.moe_forward([dxo.ExpertVersion.bf16(*m) for m in masters], d, f, group, x, ids, w)
    assert not np.allclose(y, y_hi, rtol=1e-4)


def test_pure_python_brute_force(dxo):
    x, ids, w, masters, versions, (T, d, f, E, k, group) = _tiny_layer(dxo, 23, T=3, d=16, f=8, E=3, k=2, group=8, n_int4=1)
    y = dxo.moe_forward(versions, d, f, group, x, ids, w)
    xv = bf16_bits_to_f32(x).astype(float)

    def stored(e, which, r, c):
        a = versions[e].arrays
        if versions[e].fmt == dxo.FMT_BF16:
            return float(bf16_bits_to_f32(a[which][r:r + 1, c:c + 1])[0, 0])
        byte = int(a[which][r, c // 2])
        nib = (byte >> 4) if c % 2 else (byte & 0xF)
        nib = nib - 16 if nib >= 8 else nib
        return nib * float(bf16_bits_to_f32(a[3 + which][r:r + 1, c // group:c // group + 1])[0, 0])

    for t in range(T):
        ref = [0.0] * d
        for j in range(k):
            e = int(ids[t, j])
            h = []
            for n in range(f):
                gsum = math.fsum(stored(e, 0, n, c) * xv[t, c] for c in range(d))
                usum = math.fsum(stored(e, 1, n, c) * xv[t, c] for c in range(d))
                h.append(gsum / (1.0 + math.exp(-gsum)) * usum)
            for n in range(d):
                ref[n] += w[t, j] * math.fsum(stored(e, 2, n, c) * h[c] for c in range(f))
        assert np.allclose(y[t], ref, rtol=1e-11, atol=1e-13)


def test_layer_invariants(dxo):
    x, ids, w, masters, versions, (T, d, f, E, k, group) = _tiny_layer(dxo, 24)
    y = dxo.moe_forward(versions, d, f, group, x, ids, w)
    # linear in the routing weights
    assert np.allclose(dxo.moe_forward(versions, d, f, group, x, ids, 3.0 * w), 3.0 * y, rtol=1e-12)
    # linear in W_down of a bf16 expert (a factor 2 is exact in bf16), only where it is routed
    e = E - 1
    wg, wu, wd = masters[e]
    wd2 = _bits(2.0 * bf16_bits_to_f32(wd))
    v2 = list(versions)
    v2[e] = dxo.ExpertVersion.bf16(wg, wu, wd2)
    y2 = dxo.moe_forward(v2, d, f, group, x, ids, w)
    only = dxo.moe_forward(versions, d, f, group, x, ids, np.where(ids == e, w, 0.0))
    assert np.allclose(y2 - y, only, rtol=1e-10, atol=1e-13)
    # relabelling experts consistently changes nothing
    pi = np.array([2, 0, 3, 1])
    vperm = [None] * E
    for old in range(E):
        vperm[pi[old]] = versions[old]
    assert np.allclose(dxo.moe_forward(vperm, d, f, group, x, pi[ids].astype(np.int32), w), y, rtol=1e-13)
    # token subset returns the same rows
    sub = np.array([4, 1], np.int32)
    assert np.array_equal(dxo.moe_forward(versions, d, f, group, x, ids, w, tokens=sub), y[sub])


def test_shared_expert_is_a_plain_added_mlp(dxo):
    x, ids, w, masters, versions, (T, d, f, E, k, group) = _tiny_layer(dxo, 25)
    g = np.random.default_rng(9)
    fs = 24
    sm = tuple(_bits(0.2 * g.standard_normal(s)) for s in ((fs, d), (fs, d), (d, fs)))
    y0 = dxo.moe_forward(versions, d, f, group, x, ids, w)
    y1 = dxo.moe_forward(versions, d, f, group, x, ids, w, shared=dxo.ExpertVersion.bf16(*sm), shared_f=fs)
    ref = _torch_expert(*(bf16_bits_to_f32(a) for a in sm), bf16_bits_to_f32(x)).numpy()
    assert np.allclose(y1 - y0, ref, rtol=1e-9, atol=1e-12)


# --------------------------------------------------------------------- policy
def test_hotness_counts_and_window(dxo):
    E = 8
    c = np.zeros(E, np.int64)
    S = np.zeros(E, np.uint64)
    total = np.zeros(E, np.int64)
    g = np.random.default_rng(2)
    for _ in range(5):
        ids = np.stack([g.permutation(E)[:3] for _ in range(10)]).astype(np.int32)
        counts, _, _ = dxo.permute(ids, E)
        dxo.hotness_update(c, counts)
        total += np.bincount(ids.ravel(), minlength=E)
    assert np.array_equal(c, total) and c.sum() == 5 * 10 * 3
    dxo.window_end(S, c, 0)
    assert np.array_equal(S, total.astype(np.uint64) << np.uint64(16))      # alpha = 0: plain window counts
    assert not c.any()                                                       # counters reset


def test_ema_fixed_point_matches_exact_rationals(dxo):
    E = 4
    alpha_q16 = 49152                                                        # alpha = 0.75
    S = np.zeros(E, np.uint64)
    ref = [Fraction(0)] * E
    g = np.random.default_rng(4)
    for _ in range(20):
        cw = g.integers(0, 5000, E).astype(np.int64)
        c = cw.copy()
        dxo.window_end(S, c, alpha_q16)
        # exact recurrence on S*2^16 with the floor the oracle states
        ref = [Fraction(math.floor(Fraction(alpha_q16, 65536) * r + Fraction(65536 - alpha_q16, 65536) * int(x) * 65536))
               for r, x in zip(ref, cw)]
        assert [int(v) for v in S] == [int(r) for r in ref]
    # constant input converges to it: S/2^16 -> c
    S[:] = 0
    for _ in range(200):
        c = np.full(E, 1000, np.int64)
        dxo.window_end(S, c, alpha_q16)
    assert np.all(np.abs(S.astype(np.float64) / 65536 - 1000) < 1e-2)
    with pytest.raises(ValueError):
        dxo.window_end(S, c, 65536)


def _golden_table():
    out = {}
    with open(os.path.join(GOLDEN, "table1_model_config.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                key, val = line.split("=")
                out[key.strip()] = int(val)
    return out


def test_expert_bytes_match_the_papers_model_table(dxo):
    tab = _golden_table()
    # 30B-shaped: bf16 experts of all layers = the printed 54 "GB" (GiB)
    wl = WORKLOADS["C2"]
    assert tab["qwen3_30b.experts_per_layer"] == wl.E and tab["qwen3_30b.top_k"] == wl.k
    b_hi = dxo.expert_bytes(wl.d, wl.f, wl.group, dxo.FMT_BF16)
    assert b_hi == 3 * 2048 * 768 * 2 == 9437184
    total = tab["qwen3_30b.layers"] * tab["qwen3_30b.experts_per_layer"] * b_hi
    assert round(total / 2 ** 30) == tab["qwen3_30b.expert_weight_size_gb"]
    # 80B-shaped, int4 g=128 with bf16 scales = the printed 37 "GB"
    w4 = WORKLOADS["C4"]
    assert tab["qwen3_80b_int4.experts_per_layer"] == w4.E and tab["qwen3_80b_int4.top_k"] == w4.k
    b_lo = dxo.expert_bytes(w4.d, w4.f, w4.group, dxo.FMT_INT4)
    assert b_lo == 3 * 2048 * 512 // 2 + 3 * 2048 * 512 // 128 * 2 == 1622016
    total = tab["qwen3_80b_int4.layers"] * tab["qwen3_80b_int4.experts_per_layer"] * b_lo
    assert round(total / 2 ** 30) == tab["qwen3_80b_int4.expert_weight_size_gb"]
    # ratio lo/hi = (1/2 + 2/g) / 2
    assert Fraction(dxo.expert_bytes(2048, 768, 128, 1), b_hi) == (Fraction(1, 2) + Fraction(2, 128)) / 2
    assert dxo.expert_bytes(256, 128, 64, 1) == 52224 and dxo.expert_bytes(256, 128, 64, 0) == 196608


def test_budget_capacity_is_feasible_and_maximal(dxo):
    wl = WORKLOADS["C2"]
    b_hi = dxo.expert_bytes(wl.d, wl.f, wl.group, 0)
    b_lo = dxo.expert_bytes(wl.d, wl.f, wl.group, 1)
    assert dxo.budget_capacity(535560192, wl.E, b_hi, b_lo) == 32
    assert dxo.budget_capacity(535560191, wl.E, b_hi, b_lo) == 31
    assert dxo.budget_capacity(wl.E * b_lo - 1, wl.E, b_hi, b_lo) == -1
    assert dxo.budget_capacity(wl.E * b_lo, wl.E, b_hi, b_lo) == 0
    assert dxo.budget_capacity(10 ** 12, wl.E, b_hi, b_lo) == wl.E
    g = np.random.default_rng(8)
    for _ in range(200):
        E = int(g.integers(1, 600))
        budget = int(g.integers(0, E * b_hi * 1.2))
        n = dxo.budget_capacity(budget, E, b_hi, b_lo)
        if n < 0:
            assert E * b_lo > budget
            continue
        assert n * b_hi + (E - n) * b_lo <= budget                          # never exceeds the budget
        assert n == E or (n + 1) * b_hi + (E - n - 1) * b_lo > budget       # and is maximal
        assert n == min(E, (budget - E * b_lo) // (b_hi - b_lo))            # closed form
    # 80B-shaped stack under 40 GiB with the 48 bf16 shared experts counted: 12 per layer
    w4 = WORKLOADS["C4"]
    bh, bl = dxo.expert_bytes(w4.d, w4.f, w4.group, 0), dxo.expert_bytes(w4.d, w4.f, w4.group, 1)
    shared = dxo.expert_bytes(w4.d, w4.shared_f, w4.group, 0)
    per_layer = (40 * 2 ** 30 - w4.L * shared) // w4.L
    assert dxo.budget_capacity(per_layer, w4.E, bh, bl) == w4.n_hi == 12
    assert dxo.budget_capacity(40 * 10 ** 9 // w4.L, w4.E, bh, bl) <= 0


def test_select_is_exactly_top_n(dxo):
    g = np.random.default_rng(6)
    for E, n in [(8, 2), (128, 32), (512, 12), (16, 16), (16, 0)]:
        S = g.integers(0, 40, E).astype(np.uint64) << np.uint64(16)          # many ties
        ids = dxo.select_topn(S, n)
        ref = sorted(range(E), key=lambda e: (-int(S[e]), e))[:n]
        assert ids.tolist() == ref
        if 0 < n < E:
            rest = np.setdiff1d(np.arange(E), ids)
            assert S[ids].min() >= S[rest].max()
    assert dxo.select_topn(np.zeros(10, np.uint64), 3).tolist() == [0, 1, 2]
    with pytest.raises(ValueError):
        dxo.select_topn(np.zeros(4, np.uint64), 5)


def test_transition_sets_are_set_differences(dxo):
    g = np.random.default_rng(12)
    for _ in range(20):
        E = 64
        cur = (g.random(E) < 0.3).astype(np.uint8)
        new = (g.random(E) < 0.3).astype(np.uint8)
        pro, dem = dxo.transition_sets(cur, new)
        H, Hc = set(np.flatnonzero(new)), set(np.flatnonzero(cur))
        assert pro.tolist() == sorted(H - Hc) and dem.tolist() == sorted(Hc - H)


def test_router_logits_closed_forms(dxo):
    g = np.random.default_rng(31)
    T, E, d = 5, 7, 64
    wr = wlmod.f32_to_bf16_bits(g.standard_normal((E, d)).astype(np.float32))
    bias = g.standard_normal(E).astype(np.float32)
    # one-hot tokens pick out a column of W_r: token t = unit vector c_t  ->  logits[t, e] = W_r[e, c_t] + bias[e]
    cols = [3, 0, 63, 17, 17]
    x = np.zeros((T, d), np.float32)
    x[np.arange(T), cols] = 1.0
    got = dxo.router_logits(wlmod.f32_to_bf16_bits(x), wr, bias)
    want = (wlmod.bf16_bits_to_f32(wr)[:, cols].T.astype(np.float64) + bias.astype(np.float64)).astype(np.float32)
    assert np.array_equal(got, want)
    # small integers: every product and sum is exact, the result is the integer dot product
    xi = g.integers(-4, 5, (T, d)).astype(np.float32)
    wi = g.integers(-4, 5, (E, d)).astype(np.float32)
    got = dxo.router_logits(wlmod.f32_to_bf16_bits(xi), wlmod.f32_to_bf16_bits(wi))
    assert np.array_equal(got, (xi.astype(np.int64) @ wi.astype(np.int64).T).astype(np.float32))
    # x and W_r swap roles under transposition; doubling x doubles the bias-free logits exactly
    xr = wlmod.f32_to_bf16_bits(g.standard_normal((T, d)).astype(np.float32))
    a = dxo.router_logits(xr, wr)
    assert np.array_equal(a, dxo.router_logits(wr, xr).T)
    x2 = wlmod.f32_to_bf16_bits(2.0 * wlmod.bf16_bits_to_f32(xr))
    assert np.array_equal(dxo.router_logits(x2, wr), 2.0 * a)
    # the generator's fp32 logits of the workload recipe are the same numbers up to fp32 summation error
    wl = WORKLOADS["C1"]
    xb = wlmod.activations(wl, 0, 0, 0)
    wrb = wlmod.router_matrix(wl, 0, 0)
    zb = wlmod.zipf_bias(wl.E, wl.zipf_s, 0, wl.config_id, 0) if wl.zipf_s is not None else None
    assert np.allclose(dxo.router_logits(xb, wrb, zb), wlmod.router_logits(wl, xb, wrb, 0, 0), rtol=0, atol=2e-5)


def _rank_key(S):
    return lambda e: (-int(S[e]), e)


def test_hysteresis_worked_example(dxo):
    """Five experts with scores 10, 9, 8, 7, 6, capacity 2, current set {2, 3}: worked by hand."""
    S = np.array([10, 9, 8, 7, 6], np.uint64)
    cur = np.array([0, 0, 1, 1, 0], np.uint8)
    assert dxo.select_hysteresis(S, cur, 2, 0).tolist() == [0, 1]       # no margin: plain top-2
    # margin 2: 10 > 7 + 2 replaces expert 3; then 9 > 8 + 2 fails and expert 2 stays
    assert dxo.select_hysteresis(S, cur, 2, 2).tolist() == [0, 2]
    # margin 3: 10 > 7 + 3 fails ("exceeds by a margin" is strict): nothing moves
    assert dxo.select_hysteresis(S, cur, 2, 3).tolist() == [2, 3]
    # rank slack 1: the top 3 hold expert 2 but not expert 3, whose place goes to expert 0
    assert dxo.select_rank_slack(S, cur, 2, 1).tolist() == [0, 2]
    assert dxo.select_rank_slack(S, cur, 2, 2).tolist() == [2, 3]
    assert dxo.select_rank_slack(S, cur, 2, 0).tolist() == [0, 1]
    # an empty place is filled without a margin; a set above capacity sheds its lowest-ranked member
    assert dxo.select_hysteresis(S, np.array([0, 0, 0, 1, 0], np.uint8), 2, 100).tolist() == [0, 3]
    assert dxo.select_hysteresis(S, np.array([0, 1, 1, 1, 0], np.uint8), 2, 100).tolist() == [1, 2]


def test_hysteresis_without_margin_is_top_n(dxo):
    g = np.random.default_rng(21)
    for E, n in [(8, 2), (128, 32), (64, 0), (16, 16), (40, 7)]:
        for _ in range(6):
            S = g.integers(0, 12, E).astype(np.uint64) << np.uint64(16)      # many ties
            cur = (g.random(E) < g.random()).astype(np.uint8)                # any size, not only n
            ref = dxo.select_topn(S, n).tolist()
            assert dxo.select_hysteresis(S, cur, n, 0).tolist() == ref
            assert dxo.select_rank_slack(S, cur, n, 0).tolist() == ref


def test_hysteresis_matches_sorted_pairing_and_its_invariants(dxo):
    """Independent formulation: pair the i-th best outsider with the i-th worst member; the swaps are
    the leading pairs whose score gap exceeds the margin.  Plus what the rule promises."""
    g = np.random.default_rng(22)
    for trial in range(60):
        E = int(g.integers(4, 80))
        n = int(g.integers(1, E))
        S = g.integers(0, 50, E).astype(np.uint64)
        margin = int(g.integers(1, 12))
        cur_ids = g.choice(E, n, replace=False)
        cur = np.zeros(E, np.uint8)
        cur[cur_ids] = 1
        got = dxo.select_hysteresis(S, cur, n, margin)
        members = sorted(cur_ids.tolist(), key=_rank_key(S), reverse=True)       # worst first
        outsiders = sorted(set(range(E)) - set(cur_ids.tolist()), key=_rank_key(S))  # best first
        H = set(cur_ids.tolist())
        for m, o in zip(members, outsiders):
            if int(S[o]) - int(S[m]) > margin:
                H.remove(m)
                H.add(o)
            else:
                break
        assert set(got.tolist()) == H
        assert got.tolist() == sorted(H, key=_rank_key(S))                      # rank order
        new, gone, rest = H - set(cur_ids.tolist()), set(cur_ids.tolist()) - H, set(range(E)) - H
        assert len(H) == n
        assert all(int(S[p]) - int(S[q]) > margin for p in new for q in gone)
        assert all(int(S[o]) - int(S[m]) <= margin for o in rest for m in H)    # a fixed point
        again = np.zeros(E, np.uint8)
        again[got] = 1
        assert dxo.select_hysteresis(S, again, n, margin).tolist() == got.tolist()   # idempotent
        # a wider margin never moves more experts
        wider = dxo.select_hysteresis(S, cur, n, margin + 5)
        assert len(set(wider.tolist()) - set(cur_ids.tolist())) <= len(new)


def test_rank_slack_keeps_members_inside_the_wider_set(dxo):
    g = np.random.default_rng(23)
    for trial in range(60):
        E = int(g.integers(4, 80))
        n = int(g.integers(1, E))
        slack = int(g.integers(0, 6))
        S = g.integers(0, 30, E).astype(np.uint64)
        cur_ids = g.choice(E, n, replace=False).tolist()
        cur = np.zeros(E, np.uint8)
        cur[cur_ids] = 1
        got = dxo.select_rank_slack(S, cur, n, slack).tolist()
        order = sorted(range(E), key=_rank_key(S))
        wide = set(order[:n + slack])
        keep = [e for e in cur_ids if e in wide]
        fill = [e for e in order if e not in keep][:n - len(keep)]
        assert set(got) == set(keep) | set(fill)
        assert got == sorted(got, key=_rank_key(S)) and len(got) == n


# --------------------------------------------------- the workload recipe itself
def test_zipf_routing_is_heavy_tailed():
    wl = WORKLOADS["C2"]
    x, logits = wlmod.layer_inputs(wl, seed=0)
    assert x.shape == (32, 2048) and logits.shape == (32, 128) and logits.dtype == np.float32
    bias = wlmod.zipf_bias(wl.E, wl.zipf_s, 0, wl.config_id, 0)
    assert abs(np.exp(bias.astype(np.float64)).sum() - 1.0) < 1e-5
    assert abs((bias.max() - bias.min()) - 1.1 * math.log(128)) < 1e-4
    assert not np.array_equal(bias, wlmod.zipf_bias(wl.E, wl.zipf_s, 0, wl.config_id, 0, epoch=1))
    assert sorted(bias.tolist()) == sorted(wlmod.zipf_bias(wl.E, wl.zipf_s, 0, wl.config_id, 0, epoch=1).tolist())
