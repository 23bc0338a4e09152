"""ctypes front end of the CPU oracle (``dxo.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing on the product path imports this
module, and this module imports nothing from the HIP package.

bf16 tensors are ``numpy.uint16`` bit patterns; everything is a host array.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dxo.c")
_LIB = os.path.join(_HERE, "libdxo.so")

FMT_BF16 = 0
FMT_INT4 = 1
FMT_INT2 = 2


def build(force: bool = False) -> str:
    """Compile dxo.c with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Expert(C.Structure):
    _fields_ = [("w_gate", C.c_void_p), ("w_up", C.c_void_p), ("w_down", C.c_void_p),
                ("s_gate", C.c_void_p), ("s_up", C.c_void_p), ("s_down", C.c_void_p),
                ("fmt", C.c_int32), ("pad", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.dxo_threads.restype = C.c_int
        L.dxo_expert_bytes.restype = C.c_uint64
        L.dxo_expert_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int]
        L.dxo_budget_capacity.restype = C.c_int
        L.dxo_budget_capacity.argtypes = [C.c_uint64, C.c_int, C.c_uint64, C.c_uint64]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def threads() -> int:
    return int(lib().dxo_threads())


# ----------------------------------------------------------------- routing
def router_logits(x_bits: np.ndarray, wr_bits: np.ndarray, bias=None) -> np.ndarray:
    """fp32 logits [T,E] = x . W_r^T (+ bias) from bf16 bit patterns, fp64 sums."""
    x = np.ascontiguousarray(x_bits, np.uint16)
    wr = np.ascontiguousarray(wr_bits, np.uint16)
    T, d = x.shape
    E = wr.shape[0]
    assert wr.shape[1] == d
    b = None if bias is None else np.ascontiguousarray(bias, np.float32)
    out = np.empty((T, E), np.float32)
    rc = lib().dxo_router_logits(_p(x), _p(wr), _p(b) if b is not None else None, C.c_int(T), C.c_int(E), C.c_int(d),
                                 _p(out))
    if rc:
        raise ValueError(f"dxo_router_logits rc={rc}")
    return out


def topk(logits: np.ndarray, k: int):
    """ids int32 [T,k] (descending logit, ties to the lower index), w fp64 [T,k]."""
    logits = np.ascontiguousarray(logits, np.float32)
    T, E = logits.shape
    ids = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float64)
    rc = lib().dxo_topk(_p(logits), C.c_int(T), C.c_int(E), C.c_int(k), _p(ids), _p(w))
    if rc:
        raise ValueError(f"dxo_topk rc={rc}")
    return ids, w


def permute(ids: np.ndarray, E: int):
    """counts [E], offsets [E+1], perm [T*k] (int32)."""
    ids = np.ascontiguousarray(ids, np.int32)
    T, k = ids.shape
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    perm = np.empty(T * k, np.int32)
    rc = lib().dxo_permute(_p(ids), C.c_int(T), C.c_int(E), C.c_int(k), _p(counts), _p(offsets), _p(perm))
    if rc:
        raise ValueError(f"dxo_permute rc={rc}")
    return counts, offsets, perm


def route(logits: np.ndarray, k: int):
    ids, w = topk(logits, k)
    counts, offsets, perm = permute(ids, logits.shape[1])
    return ids, w, counts, offsets, perm


# --------------------------------------------------------------- quantizer
def quantize(w_bits: np.ndarray, group: int):
    """bf16 bits [rows,K] -> (packed u8 [rows,K/2], bf16 scale bits [rows,K/group])."""
    w_bits = np.ascontiguousarray(w_bits, np.uint16)
    rows, K = w_bits.shape
    q = np.empty((rows, K // 2), np.uint8)
    s = np.empty((rows, K // group), np.uint16)
    rc = lib().dxo_quantize(_p(w_bits), C.c_int(rows), C.c_int(K), C.c_int(group), _p(q), _p(s))
    if rc:
        raise ValueError(f"dxo_quantize rc={rc}")
    return q, s


def dequantize(q: np.ndarray, s: np.ndarray, group: int) -> np.ndarray:
    q = np.ascontiguousarray(q, np.uint8)
    s = np.ascontiguousarray(s, np.uint16)
    rows, K = q.shape[0], q.shape[1] * 2
    out = np.empty((rows, K), np.float32)
    rc = lib().dxo_dequantize(_p(q), _p(s), C.c_int(rows), C.c_int(K), C.c_int(group), _p(out))
    if rc:
        raise ValueError(f"dxo_dequantize rc={rc}")
    return out


def quantize2(w_bits: np.ndarray, group: int):
    """bf16 bits [rows,K] -> (packed 2-bit codes u8 [rows,K/4], bf16 scale bits [rows,K/group])."""
    w_bits = np.ascontiguousarray(w_bits, np.uint16)
    rows, K = w_bits.shape
    q = np.empty((rows, K // 4), np.uint8)
    s = np.empty((rows, K // group), np.uint16)
    rc = lib().dxo_quantize2(_p(w_bits), C.c_int(rows), C.c_int(K), C.c_int(group), _p(q), _p(s))
    if rc:
        raise ValueError(f"dxo_quantize2 rc={rc}")
    return q, s


def dequantize2(q: np.ndarray, s: np.ndarray, group: int) -> np.ndarray:
    q = np.ascontiguousarray(q, np.uint8)
    s = np.ascontiguousarray(s, np.uint16)
    rows, K = q.shape[0], q.shape[1] * 4
    out = np.empty((rows, K), np.float32)
    rc = lib().dxo_dequantize2(_p(q), _p(s), C.c_int(rows), C.c_int(K), C.c_int(group), _p(out))
    if rc:
        raise ValueError(f"dxo_dequantize2 rc={rc}")
    return out


# ------------------------------------------------------------------- layer
class ExpertVersion:
    """One stored version of an expert: bf16 matrices, or int4 + scales."""

    def __init__(self, fmt, w_gate, w_up, w_down, s_gate=None, s_up=None, s_down=None):
        self.fmt = fmt
        self.arrays = [np.ascontiguousarray(a) if a is not None else None
                       for a in (w_gate, w_up, w_down, s_gate, s_up, s_down)]

    @classmethod
    def bf16(cls, wg, wu, wd):
        return cls(FMT_BF16, np.asarray(wg, np.uint16), np.asarray(wu, np.uint16), np.asarray(wd, np.uint16))

    @classmethod
    def int4_from_master(cls, wg, wu, wd, group):
        (qg, sg), (qu, su), (qd, sd) = (quantize(m, group) for m in (wg, wu, wd))
        return cls(FMT_INT4, qg, qu, qd, sg, su, sd)

    @classmethod
    def int2_from_master(cls, wg, wu, wd, group):
        (qg, sg), (qu, su), (qd, sd) = (quantize2(m, group) for m in (wg, wu, wd))
        return cls(FMT_INT2, qg, qu, qd, sg, su, sd)

    def struct(self) -> _Expert:
        ptr = [a.ctypes.data if a is not None else None for a in self.arrays]
        return _Expert(ptr[0], ptr[1], ptr[2], ptr[3], ptr[4], ptr[5], self.fmt, 0)


def moe_forward(experts, d: int, f: int, group: int, x_bits: np.ndarray,
                ids: np.ndarray, w: np.ndarray, shared: ExpertVersion | None = None,
                shared_f: int = 0, tokens=None) -> np.ndarray:
    """fp64 layer output.  ``experts``: list of ExpertVersion, length E.  With
    ``tokens`` (int array) only those rows are computed, in that order."""
    x_bits = np.ascontiguousarray(x_bits, np.uint16)
    ids = np.ascontiguousarray(ids, np.int32)
    w = np.ascontiguousarray(w, np.float64)
    T, k = ids.shape
    E = len(experts)
    arr = (_Expert * E)(*[e.struct() for e in experts])
    sh = shared.struct() if shared is not None else None
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, np.int32)
        n = int(tokens.size)
    else:
        n = T
    y = np.empty((n, d), np.float64)
    rc = lib().dxo_moe_forward(arr, C.c_int(E), C.c_int(d), C.c_int(f), C.c_int(group),
                               _p(x_bits), C.c_int(T), C.c_int(k), _p(ids), _p(w),
                               C.byref(sh) if sh is not None else None, C.c_int(shared_f),
                               _p(tokens) if tokens is not None else None, C.c_int(n), _p(y))
    if rc:
        raise ValueError(f"dxo_moe_forward rc={rc}")
    return y


# ------------------------------------------------------------------ policy
def hotness_update(c: np.ndarray, counts: np.ndarray) -> None:
    assert c.dtype == np.int64 and c.flags.c_contiguous
    counts = np.ascontiguousarray(counts, np.int32)
    lib().dxo_hotness_update(_p(c), _p(counts), C.c_int(c.size))


def window_end(S: np.ndarray, c: np.ndarray, alpha_q16: int = 0) -> None:
    assert S.dtype == np.uint64 and c.dtype == np.int64
    rc = lib().dxo_window_end(_p(S), _p(c), C.c_int(S.size), C.c_uint32(alpha_q16))
    if rc:
        raise ValueError("alpha_q16 must be < 65536")


def expert_bytes(d: int, f: int, group: int, fmt: int) -> int:
    return int(lib().dxo_expert_bytes(d, f, group, fmt))


def budget_capacity(budget: int, E: int, b_hi: int, b_lo: int) -> int:
    return int(lib().dxo_budget_capacity(budget, E, b_hi, b_lo))


def select_topn(S: np.ndarray, n: int) -> np.ndarray:
    S = np.ascontiguousarray(S, np.uint64)
    out = np.empty(n, np.int32)
    rc = lib().dxo_select_topn(_p(S), C.c_int(S.size), C.c_int(n), _p(out))
    if rc:
        raise ValueError(f"dxo_select_topn rc={rc}")
    return out


def select_hysteresis(S: np.ndarray, cur: np.ndarray, n: int, margin: int) -> np.ndarray:
    """Additive-margin hysteresis; `cur` = 0/1 flags of the current set; ids in rank order."""
    S = np.ascontiguousarray(S, np.uint64)
    cur = np.ascontiguousarray(cur, np.uint8)
    out = np.empty(n, np.int32)
    rc = lib().dxo_select_hysteresis(_p(S), C.c_int(S.size), _p(cur), C.c_int(n), C.c_uint64(int(margin)), _p(out))
    if rc:
        raise ValueError(f"dxo_select_hysteresis rc={rc}")
    return out


def select_rank_slack(S: np.ndarray, cur: np.ndarray, n: int, slack: int) -> np.ndarray:
    """Rank-slack hysteresis; ids in rank order."""
    S = np.ascontiguousarray(S, np.uint64)
    cur = np.ascontiguousarray(cur, np.uint8)
    out = np.empty(n, np.int32)
    rc = lib().dxo_select_rank_slack(_p(S), C.c_int(S.size), _p(cur), C.c_int(n), C.c_int(slack), _p(out))
    if rc:
        raise ValueError(f"dxo_select_rank_slack rc={rc}")
    return out


def transition_sets(is_hi_cur: np.ndarray, is_hi_new: np.ndarray):
    cur = np.ascontiguousarray(is_hi_cur, np.uint8)
    new = np.ascontiguousarray(is_hi_new, np.uint8)
    E = cur.size
    pro = np.empty(E, np.int32)
    dem = np.empty(E, np.int32)
    npro = C.c_int32(0)
    ndem = C.c_int32(0)
    lib().dxo_transition_sets(_p(cur), _p(new), C.c_int(E), _p(pro), C.byref(npro), _p(dem), C.byref(ndem))
    return pro[:npro.value].copy(), dem[:ndem.value].copy()
