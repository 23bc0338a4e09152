"""Thin ctypes binding of libdynaexq.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch appears
here only as the provider of device memory and of the compute stream.  The
wrappers carry the same names as the C entry points.  There is no CPU
fallback: loading fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DYNAEXQ_LIB", os.path.join(_PKG, "libdynaexq.so"))

DX_OK, DX_ERR_INVALID, DX_ERR_BUDGET, DX_ERR_BUSY, DX_ERR_NOMEM, DX_ERR_HIP = range(6)
DX_FMT_BF16, DX_FMT_INT4G, DX_FMT_INT2G = 0, 1, 2
DX_STATE_EMPTY, DX_STATE_RESIDENT_HI, DX_STATE_RESIDENT_LO, DX_STATE_PROMOTING, DX_STATE_DEMOTING = range(5)

EXPORTS = [
    "dx_create", "dx_destroy", "dx_last_error", "dx_status_str",
    "dx_route", "dx_route_static", "dx_route_static_last_error", "dx_router_logits", "dx_moe_forward", "dx_route_forward", "dx_hotness_update", "dx_window_end", "dx_select_resident",
    "dx_expert_bytes", "dx_budget_capacity", "dx_select_topn", "dx_plan_transitions",
    "dx_select_hysteresis", "dx_select_rank_slack", "dx_select_resident_stable",
    "dx_register_host_master", "dx_register_host_packed", "dx_transitions_limits", "dx_transitions_enqueue", "dx_transitions_pump",
    "dx_quantize_expert", "dx_quantize_expert_int2", "dx_swap_handle",
    "dx_handle_table", "dx_get_handle", "dx_get_formats", "dx_get_states", "dx_get_counters", "dx_get_stats", "dx_get_pool",
    "dx_set_profiling", "dx_get_profile", "dx_probe_read",
    "dx_pools_create", "dx_expert_install", "dx_promote_async", "dx_demote_async", "dx_migrate_poll",
]


class DxConfig(C.Structure):
    _fields_ = [("L", C.c_int32), ("E", C.c_int32), ("d", C.c_int32), ("f", C.c_int32),
                ("top_k", C.c_int32), ("group", C.c_int32), ("shared_f", C.c_int32),
                ("max_tokens", C.c_int32), ("window_steps", C.c_int32), ("alpha_q16", C.c_uint32),
                ("route_updates_hotness", C.c_int32), ("hi_fmt", C.c_int32),
                ("budget_bytes", C.c_uint64), ("transient_bytes", C.c_uint64)]


class DxHandle(C.Structure):
    _fields_ = [("w_gate", C.c_void_p), ("w_up", C.c_void_p), ("w_down", C.c_void_p),
                ("s_gate", C.c_void_p), ("s_up", C.c_void_p), ("s_down", C.c_void_p),
                ("fmt", C.c_uint32), ("version", C.c_uint32), ("reserved", C.c_uint64)]


class DxStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "promotions_issued", "promotions_published", "demotions_issued", "demotions_published",
        "h2d_bytes", "quantize_read_bytes", "quantize_write_bytes", "reserved_bytes",
        "peak_reserved_bytes", "deferred", "in_flight", "peak_in_flight", "queued")]

    def asdict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class DxProfile(C.Structure):
    _fields_ = [("calls", C.c_uint64), ("gate_up_ms", C.c_double), ("down_ms", C.c_double),
                ("combine_ms", C.c_double), ("empty_ms", C.c_double)]


class DxError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        super().__init__(f"{where}: {status_str(status)}: {text}")
        self.status = status


_lib = None


def load():
    """Load libdynaexq.so; raises if it is missing (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or paper_2511_15015_amd/build.py) first; there is no CPU fallback")
    # PyTorch ships its own HIP runtime (same soname as the system one).  Import it
    # first so that this library binds to the runtime that owns torch's memory and
    # streams instead of bringing a second runtime into the process.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, u64 = C.c_void_p, C.c_int, C.c_uint64
    L.dx_create.argtypes = [C.POINTER(DxConfig), vp, C.POINTER(vp)]
    L.dx_destroy.argtypes = [vp]
    L.dx_destroy.restype = None
    L.dx_last_error.argtypes = [vp]
    L.dx_last_error.restype = C.c_char_p
    L.dx_status_str.argtypes = [i32]
    L.dx_status_str.restype = C.c_char_p
    L.dx_route.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp]
    L.dx_route_static.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.dx_route_static_last_error.argtypes = []
    L.dx_route_static_last_error.restype = C.c_char_p
    L.dx_router_logits.argtypes = [vp, vp, vp, vp, i32, vp]
    L.dx_moe_forward.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp, vp]
    L.dx_route_forward.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    L.dx_hotness_update.argtypes = [vp, i32, vp]
    L.dx_window_end.argtypes = [vp, vp]
    L.dx_select_resident.argtypes = [vp, i32, u64, vp, C.POINTER(C.c_int32)]
    L.dx_expert_bytes.argtypes = [i32, i32, i32, i32]
    L.dx_expert_bytes.restype = u64
    L.dx_budget_capacity.argtypes = [u64, i32, u64, u64]
    L.dx_budget_capacity.restype = i32
    L.dx_select_topn.argtypes = [vp, i32, i32, vp]
    L.dx_select_hysteresis.argtypes = [vp, i32, vp, i32, u64, vp]
    L.dx_select_rank_slack.argtypes = [vp, i32, vp, i32, i32, vp]
    L.dx_select_resident_stable.argtypes = [vp, i32, u64, u64, i32, vp, C.POINTER(C.c_int32)]
    L.dx_plan_transitions.argtypes = [vp, i32, vp, i32, vp, C.POINTER(C.c_int32), vp, C.POINTER(C.c_int32)]
    L.dx_quantize_expert.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    L.dx_quantize_expert_int2.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    L.dx_swap_handle.argtypes = [vp, i32, i32, C.POINTER(DxHandle), vp]
    L.dx_handle_table.argtypes = [vp, i32]
    L.dx_handle_table.restype = vp
    L.dx_get_handle.argtypes = [vp, i32, i32, C.POINTER(DxHandle)]
    L.dx_get_formats.argtypes = [vp, vp]
    L.dx_get_states.argtypes = [vp, vp]
    L.dx_get_counters.argtypes = [vp, vp]
    L.dx_get_stats.argtypes = [vp, C.POINTER(DxStats)]
    L.dx_get_pool.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(u64), C.POINTER(C.c_int32)]
    L.dx_set_profiling.argtypes = [vp, i32]
    L.dx_get_profile.argtypes = [vp, C.POINTER(DxProfile)]
    L.dx_probe_read.argtypes = [vp, vp, C.c_uint64]
    L.dx_pools_create.argtypes = [vp, i32, i32]
    L.dx_register_host_master.argtypes = [vp, i32, i32, vp, vp, vp]
    L.dx_register_host_packed.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.dx_transitions_limits.argtypes = [vp, i32]
    L.dx_transitions_enqueue.argtypes = [vp, i32, vp, i32, vp, i32]
    L.dx_transitions_pump.argtypes = [vp, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.dx_expert_install.argtypes = [vp, i32, i32, i32, vp, vp, vp, i32]
    L.dx_promote_async.argtypes = [vp, i32, i32, vp, vp, vp]
    L.dx_demote_async.argtypes = [vp, i32, i32]
    L.dx_migrate_poll.argtypes = [vp, i32, C.POINTER(C.c_int)]
    _lib = L
    return L


def status_str(s: int) -> str:
    return load().dx_status_str(int(s)).decode()


def _ptr(t):
    """Device/host address of a torch tensor, numpy array, int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        assert t.flags.c_contiguous
        return t.ctypes.data
    assert t.is_contiguous(), "tensors must be contiguous"
    return t.data_ptr()


# ---- pure host helpers (no context, no device) -----------------------------
def dx_expert_bytes(d: int, f: int, group: int, fmt: int) -> int:
    return int(load().dx_expert_bytes(d, f, group, fmt))


def dx_budget_capacity(budget_bytes: int, E: int, b_hi: int, b_lo: int) -> int:
    return int(load().dx_budget_capacity(budget_bytes, E, b_hi, b_lo))


def dx_select_topn(scores: np.ndarray, n: int) -> np.ndarray:
    scores = np.ascontiguousarray(scores, np.uint64)
    out = np.empty(max(n, 0), np.int32)
    s = load().dx_select_topn(scores.ctypes.data, scores.size, n, out.ctypes.data)
    if s:
        raise DxError(s, "dx_select_topn", "invalid argument")
    return out


def dx_select_hysteresis(scores: np.ndarray, cur: np.ndarray, n: int, margin: int) -> np.ndarray:
    scores = np.ascontiguousarray(scores, np.uint64)
    cur = np.ascontiguousarray(cur, np.uint8)
    out = np.empty(max(n, 0), np.int32)
    s = load().dx_select_hysteresis(scores.ctypes.data, scores.size, cur.ctypes.data, n, int(margin), out.ctypes.data)
    if s:
        raise DxError(s, "dx_select_hysteresis", "invalid argument")
    return out


def dx_select_rank_slack(scores: np.ndarray, cur: np.ndarray, n: int, slack: int) -> np.ndarray:
    scores = np.ascontiguousarray(scores, np.uint64)
    cur = np.ascontiguousarray(cur, np.uint8)
    out = np.empty(max(n, 0), np.int32)
    s = load().dx_select_rank_slack(scores.ctypes.data, scores.size, cur.ctypes.data, n, slack, out.ctypes.data)
    if s:
        raise DxError(s, "dx_select_rank_slack", "invalid argument")
    return out


def dx_route_static(logits, T, E, top_k, topk_ids, topk_w, counts, offsets, perm, stream=None):
    """dx_route without a context and without any allocation (static device scratch)."""
    lib = load()
    s = lib.dx_route_static(_ptr(logits), T, E, top_k, _ptr(topk_ids), _ptr(topk_w), _ptr(counts), _ptr(offsets),
                            _ptr(perm), C.c_void_p(stream) if stream else None)
    if s:
        raise DxError(s, "dx_route_static", lib.dx_route_static_last_error().decode())


class Context:
    """Owns one dx_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, *, L, E, d, f, top_k, group, max_tokens, shared_f=0, window_steps=256,
                 alpha_q16=0, budget_bytes=0, transient_bytes=0, route_updates_hotness=False, stream=None,
                 hi_fmt=DX_FMT_BF16):
        import torch
        self.lib = load()
        self.cfg = DxConfig(L, E, d, f, top_k, group, shared_f, max_tokens, window_steps, alpha_q16,
                            1 if route_updates_hotness else 0, hi_fmt, budget_bytes, transient_bytes)
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.stream = stream
        h = C.c_void_p()
        s = self.lib.dx_create(C.byref(self.cfg), C.c_void_p(stream), C.byref(h))
        if s:
            raise DxError(s, "dx_create", self.lib.dx_last_error(None).decode())
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.dx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, s, where):
        if s:
            raise DxError(s, where, self.lib.dx_last_error(self.h).decode())

    # hot path
    def dx_route(self, layer, logits, T, topk_ids, topk_w, counts, offsets, perm):
        self._chk(self.lib.dx_route(self.h, layer, _ptr(logits), T, _ptr(topk_ids), _ptr(topk_w),
                                    _ptr(counts), _ptr(offsets), _ptr(perm)), "dx_route")

    def dx_router_logits(self, x, w_router, bias, T, logits):
        self._chk(self.lib.dx_router_logits(self.h, _ptr(x), _ptr(w_router), _ptr(bias), T, _ptr(logits)),
                  "dx_router_logits")

    def dx_moe_forward(self, layer, handle_table, x, T, topk_ids, topk_w, offsets, perm, y):
        self._chk(self.lib.dx_moe_forward(self.h, layer, _ptr(handle_table), _ptr(x), T, _ptr(topk_ids),
                                          _ptr(topk_w), _ptr(offsets), _ptr(perm), _ptr(y)), "dx_moe_forward")

    def dx_route_forward(self, layer, handle_table, logits, x, T, topk_ids, topk_w, counts, offsets, perm, y):
        self._chk(self.lib.dx_route_forward(self.h, layer, _ptr(handle_table), _ptr(logits), _ptr(x), T,
                                            _ptr(topk_ids), _ptr(topk_w), _ptr(counts), _ptr(offsets), _ptr(perm),
                                            _ptr(y)), "dx_route_forward")

    def dx_hotness_update(self, layer, counts):
        self._chk(self.lib.dx_hotness_update(self.h, layer, _ptr(counts)), "dx_hotness_update")

    def dx_window_end(self):
        out = np.empty(self.cfg.L * self.cfg.E, np.uint64)
        self._chk(self.lib.dx_window_end(self.h, out.ctypes.data), "dx_window_end")
        return out.reshape(self.cfg.L, self.cfg.E)

    def dx_select_resident(self, layer, budget_bytes):
        ids = np.empty(self.cfg.E, np.int32)
        n = C.c_int32(0)
        self._chk(self.lib.dx_select_resident(self.h, layer, budget_bytes, ids.ctypes.data, C.byref(n)),
                  "dx_select_resident")
        return ids[:n.value].copy()

    def dx_select_resident_stable(self, layer, budget_bytes, margin_q16=0, rank_slack=0):
        ids = np.empty(self.cfg.E, np.int32)
        n = C.c_int32(0)
        self._chk(self.lib.dx_select_resident_stable(self.h, layer, budget_bytes, int(margin_q16), rank_slack,
                                                     ids.ctypes.data, C.byref(n)), "dx_select_resident_stable")
        return ids[:n.value].copy()

    def dx_plan_transitions(self, layer, target_ids):
        tgt = np.ascontiguousarray(target_ids, np.int32)
        pro = np.empty(self.cfg.E, np.int32)
        dem = np.empty(self.cfg.E, np.int32)
        npro, ndem = C.c_int32(0), C.c_int32(0)
        self._chk(self.lib.dx_plan_transitions(self.h, layer, tgt.ctypes.data, tgt.size, pro.ctypes.data,
                                               C.byref(npro), dem.ctypes.data, C.byref(ndem)), "dx_plan_transitions")
        return pro[:npro.value].copy(), dem[:ndem.value].copy()

    def dx_quantize_expert(self, w_bf16, rows, K, group, q_out, s_out, stream=None):
        self._chk(self.lib.dx_quantize_expert(self.h, _ptr(w_bf16), rows, K, group, _ptr(q_out), _ptr(s_out),
                                              C.c_void_p(stream) if stream else None), "dx_quantize_expert")

    def dx_quantize_expert_int2(self, w_bf16, rows, K, group, q_out, s_out, stream=None):
        self._chk(self.lib.dx_quantize_expert_int2(self.h, _ptr(w_bf16), rows, K, group, _ptr(q_out), _ptr(s_out),
                                                   C.c_void_p(stream) if stream else None), "dx_quantize_expert_int2")

    def dx_swap_handle(self, layer, expert, handle: DxHandle, producer_event=None):
        self._chk(self.lib.dx_swap_handle(self.h, layer, expert, C.byref(handle),
                                          C.c_void_p(producer_event) if producer_event else None), "dx_swap_handle")

    # inspection
    def dx_handle_table(self, layer) -> int:
        return int(self.lib.dx_handle_table(self.h, layer) or 0)

    def dx_get_handle(self, layer, expert) -> DxHandle:
        h = DxHandle()
        self._chk(self.lib.dx_get_handle(self.h, layer, expert, C.byref(h)), "dx_get_handle")
        return h

    def dx_get_formats(self):
        out = np.empty(self.cfg.L * self.cfg.E, np.uint8)
        self._chk(self.lib.dx_get_formats(self.h, out.ctypes.data), "dx_get_formats")
        return out.reshape(self.cfg.L, self.cfg.E)

    def dx_get_states(self):
        out = np.empty(self.cfg.L * self.cfg.E, np.uint8)
        self._chk(self.lib.dx_get_states(self.h, out.ctypes.data), "dx_get_states")
        return out.reshape(self.cfg.L, self.cfg.E)

    def dx_get_counters(self):
        out = np.empty(self.cfg.L * self.cfg.E, np.int64)
        self._chk(self.lib.dx_get_counters(self.h, out.ctypes.data), "dx_get_counters")
        return out.reshape(self.cfg.L, self.cfg.E)

    def dx_get_stats(self) -> dict:
        st = DxStats()
        self._chk(self.lib.dx_get_stats(self.h, C.byref(st)), "dx_get_stats")
        return st.asdict()

    def dx_get_pool(self, which: int):
        """-> (base address, block bytes, blocks) of pool_hi (0) or pool_lo (1)"""
        base, bb, n = C.c_void_p(), C.c_uint64(0), C.c_int32(0)
        self._chk(self.lib.dx_get_pool(self.h, which, C.byref(base), C.byref(bb), C.byref(n)), "dx_get_pool")
        return int(base.value or 0), int(bb.value), int(n.value)

    def dx_set_profiling(self, enable: bool):
        self._chk(self.lib.dx_set_profiling(self.h, 1 if enable else 0), "dx_set_profiling")

    def dx_get_profile(self) -> dict:
        p = DxProfile()
        self._chk(self.lib.dx_get_profile(self.h, C.byref(p)), "dx_get_profile")
        return {"calls": int(p.calls), "gate_up_ms": p.gate_up_ms, "down_ms": p.down_ms, "combine_ms": p.combine_ms,
                "empty_ms": p.empty_ms}

    def dx_probe_read(self, buf, nbytes):
        self._chk(self.lib.dx_probe_read(self.h, _ptr(buf), nbytes), "dx_probe_read")

    # pools and transitions
    def dx_pools_create(self, hi_blocks, lo_blocks):
        self._chk(self.lib.dx_pools_create(self.h, hi_blocks, lo_blocks), "dx_pools_create")

    def dx_expert_install(self, layer, expert, fmt, gate, up, down, src_on_device=True):
        self._chk(self.lib.dx_expert_install(self.h, layer, expert, fmt, _ptr(gate), _ptr(up), _ptr(down),
                                             1 if src_on_device else 0), "dx_expert_install")

    def dx_promote_async(self, layer, expert, pinned_gate=None, pinned_up=None, pinned_down=None):
        self._chk(self.lib.dx_promote_async(self.h, layer, expert, _ptr(pinned_gate), _ptr(pinned_up),
                                            _ptr(pinned_down)), "dx_promote_async")

    def dx_demote_async(self, layer, expert):
        self._chk(self.lib.dx_demote_async(self.h, layer, expert), "dx_demote_async")

    def dx_register_host_master(self, layer, expert, pinned_gate, pinned_up, pinned_down):
        self._chk(self.lib.dx_register_host_master(self.h, layer, expert, _ptr(pinned_gate), _ptr(pinned_up),
                                                   _ptr(pinned_down)), "dx_register_host_master")

    def dx_register_host_packed(self, layer, expert, fmt, q_gate, q_up, q_down, s_gate, s_up, s_down):
        self._chk(self.lib.dx_register_host_packed(self.h, layer, expert, fmt, _ptr(q_gate), _ptr(q_up), _ptr(q_down),
                                                   _ptr(s_gate), _ptr(s_up), _ptr(s_down)), "dx_register_host_packed")

    def dx_transitions_limits(self, max_inflight):
        self._chk(self.lib.dx_transitions_limits(self.h, max_inflight), "dx_transitions_limits")

    def dx_transitions_enqueue(self, layer, promote, demote):
        pro = np.ascontiguousarray(promote, np.int32)
        dem = np.ascontiguousarray(demote, np.int32)
        self._chk(self.lib.dx_transitions_enqueue(self.h, layer, pro.ctypes.data, pro.size, dem.ctypes.data, dem.size),
                  "dx_transitions_enqueue")

    def dx_transitions_pump(self, max_issue):
        """-> (issued, published, still queued)"""
        a, b, q = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        self._chk(self.lib.dx_transitions_pump(self.h, max_issue, C.byref(a), C.byref(b), C.byref(q)),
                  "dx_transitions_pump")
        return a.value, b.value, q.value

    def dx_migrate_poll(self, wait=False) -> int:
        n = C.c_int(0)
        self._chk(self.lib.dx_migrate_poll(self.h, 1 if wait else 0, C.byref(n)), "dx_migrate_poll")
        return n.value


def make_handle(fmt, w_gate, w_up, w_down, s_gate=None, s_up=None, s_down=None) -> DxHandle:
    """Handle struct from device tensors (the caller keeps them alive while published)."""
    return DxHandle(_ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(s_gate), _ptr(s_up), _ptr(s_down), fmt, 0, 0)
