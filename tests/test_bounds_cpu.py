"""CPU checks of the element-wise tolerance the GPU parity tests use: an output that differs from the
oracle's only by the roundings the bound models passes, one wrong element fails."""
import numpy as np
import pytest

from paper_2511_15015_amd import workloads as W
from tests.bounds import assert_elementwise, elementwise_tolerance


def _c1(dxo):
    wl = W.WORKLOADS["C1"]
    x, lg = W.layer_inputs(wl, 0)
    wg, wu, wd = W.layer_masters(wl, 0, 0)
    ids, w, *_ = dxo.route(lg, wl.k)
    versions = [dxo.ExpertVersion.bf16(wg[e], wu[e], wd[e]) if e in (1, 6)
                else dxo.ExpertVersion.int4_from_master(wg[e], wu[e], wd[e], wl.group) for e in range(wl.E)]
    return wl, x, ids, w, versions, dxo.moe_forward(versions, wl.d, wl.f, wl.group, x, ids, w)


def test_rounded_output_passes_and_one_wrong_element_fails(dxo):
    wl, x, ids, w, versions, y = _c1(dxo)
    yb = W.f32_to_bf16_bits(y.astype(np.float32))
    assert assert_elementwise(dxo, yb, y, versions, wl.group, x, ids, w) < 1.0
    bad = y.copy()
    t = 3
    i = (t, int(np.argsort(np.abs(y[t]))[-20]))          # an element of ordinary size in its row
    bad[i] *= 0.9                                        # 10 % off on one element barely moves the row's norm
    row_err = np.linalg.norm(bad[i[0]] - y[i[0]]) / np.linalg.norm(y[i[0]])
    assert row_err < 2e-2                                # the per-token norm gate would let it through
    with pytest.raises(AssertionError):
        assert_elementwise(dxo, W.f32_to_bf16_bits(bad.astype(np.float32)), y, versions, wl.group, x, ids, w)


def test_bound_covers_the_rounding_of_h_in_the_worst_case(dxo):
    """Perturb H by its full bf16 half-ulp with the sign pattern that hurts most for one output column:
    the resulting change of y stays inside the bound (that is the inequality the bound states)."""
    wl, x, ids, w, versions, y = _c1(dxo)
    tol = elementwise_tolerance(dxo, versions, wl.group, x, ids, w, y)
    from tests.bounds import dense_matrices
    xf = W.bf16_bits_to_f32(x).astype(np.float64)
    t, c = 5, 17
    dy = 0.0
    for j in range(wl.k):
        wg, wu, wd = (m.astype(np.float64) for m in dense_matrices(dxo, versions[int(ids[t, j])], wl.group))
        g, u = wg @ xf[t], wu @ xf[t]
        h = g / (1.0 + np.exp(-g)) * u
        dy += w[t, j] * np.sum(np.abs(wd[c]) * np.abs(h)) * 2.0 ** -9
    assert dy <= tol[t, c]
