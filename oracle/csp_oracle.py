"""ctypes wrapper around the C oracle (oracle/csp_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg.  It imports nothing from the HIP package.

The wrapper only slices a batch into (sequence, head) problems, converts the
stored values (float32, or bf16 bit patterns) to float64 and calls the C
functions; all of the method's arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csp_oracle.c")
_LIB = os.path.join(_HERE, "libcsp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP only around independent problems)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c99",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        dp, u8p, i32p = C.POINTER(C.c_double), C.POINTER(C.c_uint8), C.POINTER(C.c_int32)
        L.csp_oracle_head_scores.argtypes = [dp, dp, u8p, C.c_int, C.c_int, C.c_int, C.c_int,
                                             C.c_double, C.c_int, dp, dp, dp]
        L.csp_oracle_head_scores.restype = None
        L.csp_oracle_budget.argtypes = [C.c_int, C.c_int, C.c_double, C.c_int, C.c_int,
                                        C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.csp_oracle_budget.restype = C.c_int
        L.csp_oracle_select.argtypes = [dp, dp, u8p, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_double, C.c_int, i32p, i32p]
        L.csp_oracle_select.restype = C.c_int
        L.csp_oracle_gather.argtypes = [C.c_void_p, C.c_size_t, i32p, C.c_int, C.c_void_p]
        L.csp_oracle_gather.restype = None
        L.csp_oracle_decode.argtypes = [dp, dp, dp, C.c_int, C.c_int, C.c_double, dp, dp]
        L.csp_oracle_decode.restype = None
        L.csp_oracle_scores_batch.argtypes = [dp, dp, u8p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                              C.c_double, C.c_int, dp, dp]
        L.csp_oracle_scores_batch.restype = None
        L.csp_oracle_decode_batch.argtypes = [dp, dp, dp, C.c_int, C.c_int, C.c_int, C.c_double, dp]
        L.csp_oracle_decode_batch.restype = None
        L.csp_oracle_max_threads.restype = C.c_int
        L.csp_oracle_set_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray, t):
    return a.ctypes.data_as(C.POINTER(t))


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (storage decoding, not arithmetic)."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    return bf16_bits_to_f64(a) if dtype == "bf16" else np.asarray(a, dtype=np.float64)


def max_threads() -> int:
    return int(lib().csp_oracle_max_threads())


def set_threads(n: int) -> None:
    lib().csp_oracle_set_threads(int(n))


# ---------------------------------------------------------------------------
def head_scores(q, k, mod, R: int, n_score: float = 0.0, causal: bool = True,
                a_self: Optional[np.ndarray] = None, a_cross: Optional[np.ndarray] = None,
                want_row_sum: bool = False):
    """Scores of one head.  q [O,D], k [L,D], mod uint8[L].  Accumulates into
    a_self / a_cross when given.  Returns (a_self, a_cross[, row_sum])."""
    q, k = _d(q), _d(k)
    mod = np.ascontiguousarray(mod, dtype=np.uint8)
    O, D = q.shape
    L = k.shape[0]
    assert k.shape[1] == D and mod.shape[0] == L and O <= L and R <= L
    if a_self is None:
        a_self = np.zeros(L, dtype=np.float64)
    if a_cross is None:
        a_cross = np.zeros(L, dtype=np.float64)
    rs = np.zeros(O, dtype=np.float64) if want_row_sum else None
    lib().csp_oracle_head_scores(_p(q, C.c_double), _p(k, C.c_double), _p(mod, C.c_uint8),
                                 L, O, R, D, float(n_score), int(bool(causal)),
                                 _p(a_self, C.c_double), _p(a_cross, C.c_double),
                                 _p(rs, C.c_double) if rs is not None else None)
    return (a_self, a_cross, rs) if want_row_sum else (a_self, a_cross)


def budget(T: int, R: int, cross_ratio: float, n_s: int, n_c: int) -> Tuple[int, int]:
    ks, kc = C.c_int(0), C.c_int(0)
    rc = lib().csp_oracle_budget(int(T), int(R), float(cross_ratio), int(n_s), int(n_c),
                                 C.byref(ks), C.byref(kc))
    if rc != 0:
        raise ValueError("budget T smaller than the recent size R")
    return ks.value, kc.value


def select(a_self, a_cross, mod, O: int, R: int, T: int, cross_ratio: float = 0.5,
           combine: str = "union"):
    """Returns (idx int32[kept] ascending, counts dict)."""
    a_self, a_cross = _d(a_self), _d(a_cross)
    mod = np.ascontiguousarray(mod, dtype=np.uint8)
    L = mod.shape[0]
    # room for every key: no reading of the method keeps more, and a wrong count (which the pins
    # check) must never write past the buffer
    idx = np.full(max(L, 1), -1, dtype=np.int32)
    cnt = np.zeros(4, dtype=np.int32)
    n = lib().csp_oracle_select(_p(a_self, C.c_double), _p(a_cross, C.c_double), _p(mod, C.c_uint8),
                                L, int(O), int(R), int(T), float(cross_ratio),
                                0 if combine == "union" else 1, _p(idx, C.c_int32), _p(cnt, C.c_int32))
    if n < 0:
        raise ValueError("invalid arguments to select (O, R, T against L)")
    return idx[:n].copy(), {"kept": int(cnt[0]), "K_s": int(cnt[1]), "K_c": int(cnt[2]), "both": int(cnt[3])}


def gather(rows: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """rows [L, ...] any dtype -> rows[idx] as a bit copy."""
    rows = np.ascontiguousarray(rows)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    out = np.empty((idx.shape[0],) + rows.shape[1:], dtype=rows.dtype)
    row_bytes = rows.dtype.itemsize * int(np.prod(rows.shape[1:], dtype=np.int64))
    lib().csp_oracle_gather(rows.ctypes.data, row_bytes, _p(idx, C.c_int32), idx.shape[0], out.ctypes.data)
    return out


def decode(q, kc, vc, n: float = 1.0, want_p: bool = False):
    """One n-softmax decode step.  q [D], kc/vc [T,D] -> out [D] (float64)."""
    q, kc, vc = _d(q), _d(kc), _d(vc)
    T, D = kc.shape
    out = np.zeros(D, dtype=np.float64)
    p = np.zeros(max(T, 1), dtype=np.float64) if want_p else None
    lib().csp_oracle_decode(_p(q, C.c_double), _p(kc, C.c_double), _p(vc, C.c_double), T, D, float(n),
                            _p(out, C.c_double), _p(p, C.c_double) if p is not None else None)
    return (out, p[:T]) if want_p else out


def scores_batch(q, k, mod, R: int, n_score: float = 0.0, causal: bool = True):
    """n_prob independent problems of one shape: q [P,O,D], k [P,L,D], mod [P,L]."""
    q, k = _d(q), _d(k)
    mod = np.ascontiguousarray(mod, dtype=np.uint8)
    P, O, D = q.shape
    L = k.shape[1]
    a_s = np.zeros((P, L), dtype=np.float64)
    a_c = np.zeros((P, L), dtype=np.float64)
    lib().csp_oracle_scores_batch(_p(q, C.c_double), _p(k, C.c_double), _p(mod, C.c_uint8), P, L, O, R, D,
                                  float(n_score), int(bool(causal)), _p(a_s, C.c_double), _p(a_c, C.c_double))
    return a_s, a_c


def decode_batch(q, kc, vc, n: float = 1.0):
    """q [P,D], kc/vc [P,T,D] -> out [P,D]."""
    q, kc, vc = _d(q), _d(kc), _d(vc)
    P, T, D = kc.shape
    out = np.zeros((P, D), dtype=np.float64)
    lib().csp_oracle_decode_batch(_p(q, C.c_double), _p(kc, C.c_double), _p(vc, C.c_double), P, T, D,
                                  float(n), _p(out, C.c_double))
    return out


# ---------------------------------------------------------------------------
# Whole-case helpers: loop the per-head functions over a csp_workloads.Case.
# ---------------------------------------------------------------------------
def group_scores(case, b: int, s: int):
    """Scores of selection group s of sequence b, summed over the group's query
    heads (head axis handling, "Cross-self pruning": one mechanism, the group)."""
    lo, hi = int(case.cu_seqlens[b]), int(case.cu_seqlens[b + 1])
    G = case.H_q // case.H_kv
    mod = case.modality[lo:hi]
    a_s = np.zeros(hi - lo, dtype=np.float64)
    a_c = np.zeros(hi - lo, dtype=np.float64)
    for hq in range(s * case.sel_group, (s + 1) * case.sel_group):
        q = to_f64(case.q_win[b, hq], case.dtype)
        k = to_f64(case.k[hq // G, lo:hi], case.dtype)
        head_scores(q, k, mod, case.R, case.n_score, True, a_s, a_c)
    return a_s, a_c


def prune_group(case, b: int, s: int, scores=None, combine: str = "union"):
    """score -> select for one (sequence, selection group).  Returns dict."""
    lo, hi = int(case.cu_seqlens[b]), int(case.cu_seqlens[b + 1])
    mod = case.modality[lo:hi]
    L, T = hi - lo, int(case.budget_T[b])
    if scores is None:
        scores = group_scores(case, b, s) if L > T else (np.zeros(L), np.zeros(L))
    idx, cnt = select(scores[0], scores[1], mod, case.O, case.R, T, case.cross_ratio, combine)
    return {"a_self": scores[0], "a_cross": scores[1], "idx": idx, "counts": cnt}


def reprune_group(windows, keys, mod, O: int, R: int, T: int, cross_ratio: float = 0.5, n_score: float = 0.0,
                  causal: bool = True):
    """The body of Algorithm 1's generation loop for one (sequence, selection group) whose cache
    holds L keys: early-out when L <= T, otherwise the scores of the last O queries against the
    cached keys (in cache order, which is temporal order; window row i sees cache rows
    t <= L-O+i), summed over the group's heads, then the same selection as after prefill.
    windows: per query head of the group, the last O queries [O,D], oldest first;
    keys: per query head, the cached keys of its KV head [L,D]; mod: uint8[L], modality flag of
    every cached key (0 for tokens appended while decoding).  Returns dict as prune_group."""
    mod = np.ascontiguousarray(mod, dtype=np.uint8)
    L = mod.shape[0]
    a_s, a_c = np.zeros(L), np.zeros(L)
    if L > T:
        for q, k in zip(windows, keys):
            head_scores(q, k, mod, R, n_score, causal, a_s, a_c)
    idx, cnt = select(a_s, a_c, mod, O, R, T, cross_ratio)
    return {"a_self": a_s, "a_cross": a_c, "idx": idx, "counts": cnt}
