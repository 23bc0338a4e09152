"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its pure host rules agree with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2511_15015_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_15015_amd import build
        build.build(verbose=False)
    binding.load()
    return binding


def test_library_exports_every_declared_symbol(B):
    text = open(os.path.join(ROOT, "include", "dynaexq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(dx_[a-z_0-9]+)\s*\(", text)))
    assert len(declared) >= 20
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in dynaexq.h but not exported"
    assert sorted(B.EXPORTS) == declared


def test_struct_sizes_match_the_header(B):
    assert C.sizeof(B.DxHandle) == 64
    assert C.sizeof(B.DxConfig) == 64
    assert C.sizeof(B.DxStats) == 104
    assert C.sizeof(B.DxProfile) == 40     # calls + four summed durations


def test_host_rules_agree_with_oracle(B, dxo):
    g = np.random.default_rng(0)
    for d, f, grp in [(256, 128, 64), (2048, 768, 128), (2048, 512, 128), (64, 32, 32)]:
        for fmt in (0, 1):
            assert B.dx_expert_bytes(d, f, grp, fmt) == dxo.expert_bytes(d, f, grp, fmt)
    b_hi, b_lo = B.dx_expert_bytes(2048, 768, 128, 0), B.dx_expert_bytes(2048, 768, 128, 1)
    for _ in range(300):
        E = int(g.integers(1, 600))
        budget = int(g.integers(0, int(E * b_hi * 1.2)))
        assert B.dx_budget_capacity(budget, E, b_hi, b_lo) == dxo.budget_capacity(budget, E, b_hi, b_lo)
    for E, n in [(8, 2), (128, 32), (512, 12), (7, 7), (7, 0)]:
        S = g.integers(0, 30, E).astype(np.uint64) << np.uint64(16)
        assert np.array_equal(B.dx_select_topn(S, n), dxo.select_topn(S, n))
    with pytest.raises(B.DxError):
        B.dx_select_topn(np.zeros(4, np.uint64), 5)


def test_hysteresis_rules_agree_with_oracle(B, dxo):
    """The library's selection with hysteresis (its own implementation) against the oracle's, on
    random scores with many ties, current sets of any size, the whole range of margins and slacks."""
    g = np.random.default_rng(5)
    for trial in range(300):
        E = int(g.integers(1, 140))
        n = int(g.integers(0, E + 1))
        S = g.integers(0, 25, E).astype(np.uint64) << np.uint64(14)
        cur = (g.random(E) < g.random()).astype(np.uint8)
        if trial % 3 == 0:                                   # a current set of exactly n members
            cur[:] = 0
            cur[g.choice(E, n, replace=False)] = 1
        margin = int(g.integers(0, 6)) << 14 if trial % 4 else 0
        slack = int(g.integers(0, 8))
        assert np.array_equal(B.dx_select_hysteresis(S, cur, n, margin), dxo.select_hysteresis(S, cur, n, margin))
        assert np.array_equal(B.dx_select_rank_slack(S, cur, n, slack), dxo.select_rank_slack(S, cur, n, slack))
    with pytest.raises(B.DxError):
        B.dx_select_hysteresis(np.zeros(4, np.uint64), np.zeros(4, np.uint8), 5, 0)
    with pytest.raises(B.DxError):
        B.dx_select_rank_slack(np.zeros(4, np.uint64), np.zeros(4, np.uint8), 2, -1)


def test_no_fallback_when_library_is_missing(B, monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libdynaexq.so")
    with pytest.raises(ImportError):
        B.load()


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_15015_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in src.replace("the CPU oracle", "").replace("CPU oracle", ""), fn
                assert "dxo" not in src, fn


def test_route_static_refuses_sizes_beyond_its_scratch_without_touching_a_gpu(B):
    """The entry point for callers that cannot allocate checks its limits before any HIP call."""
    lib = B.load()
    for T, E, k in [(8192, 1024, 8), (64, 2048, 8), (64, 0, 1), (64, 128, 0), (64, 128, 65), (-1, 128, 8)]:
        assert lib.dx_route_static(None, T, E, k, None, None, None, None, None, None) == B.DX_ERR_INVALID
        assert lib.dx_route_static_last_error().decode().startswith("dx_route_static:")


def test_create_refuses_configurations_outside_its_range_without_touching_a_gpu(B):
    """dx_create checks the configuration before any HIP call: experts beyond the table's range, a group size
    the kernels do not have, a dimension that is not a multiple of 32 and an expert matrix of 4 GiB (the
    kernels address inside a matrix with 32-bit byte offsets) are all DX_ERR_INVALID."""
    import ctypes as C
    lib = B.load()
    good = dict(L=1, E=8, d=256, f=128, top_k=2, group=64, shared_f=0, max_tokens=16, window_steps=1, alpha_q16=0,
                route_updates_hotness=0, hi_fmt=B.DX_FMT_BF16, budget_bytes=0, transient_bytes=0)
    for change in (dict(E=2000), dict(group=48), dict(d=250), dict(top_k=9), dict(d=65536, f=32768, group=128),
                   dict(shared_f=65536, d=32768, group=128), dict(max_tokens=0), dict(alpha_q16=65536)):
        cfg = B.DxConfig(**{**good, **change})
        out = C.c_void_p()
        assert lib.dx_create(C.byref(cfg), None, C.byref(out)) == B.DX_ERR_INVALID, change
        assert not out.value
