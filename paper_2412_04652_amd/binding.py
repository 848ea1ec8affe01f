"""ctypes binding of libcsp.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libcsp.so")
_lib = None

CSP_BF16, CSP_F32 = 0, 1

EXPORTED_SYMBOLS = [
    "csp_strerror", "csp_version",
    "csp_score_workspace_bytes", "csp_score", "csp_score_lse",
    "csp_select_workspace_bytes", "csp_select",
    "csp_compact",
    "csp_decode_workspace_bytes", "csp_decode_attn", "csp_static_scratch_bytes", "csp_decode_attn_static", "csp_decode_step", "csp_decode_step_phase",
    "csp_append_kv",
    "csp_gather_modality", "csp_window_push", "csp_decode_step_window", "csp_reprune_workspace_bytes", "csp_reprune",
    "csp_probe_stream",
]


class CspError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {csp_strerror(code)} ({code})")


class _CDesc(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("B", C.c_int32), ("H_q", C.c_int32), ("H_kv", C.c_int32),
        ("D", C.c_int32), ("sel_group", C.c_int32), ("window_O", C.c_int32), ("recent_R", C.c_int32),
        ("causal", C.c_int32), ("max_seqlen", C.c_int32),
        ("n_score", C.c_double), ("n_decode", C.c_double), ("cross_ratio", C.c_double),
        ("cu_seqlens_host", C.c_void_p), ("budget_T_host", C.c_void_p),
        ("cu_seqlens", C.c_void_p), ("budget_T", C.c_void_p),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("score_wait_us", C.c_int32),
    ]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libcsp.so.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2412_04652_amd.build` "
                "(hipcc, gfx950); the HIP library is the only implementation")
        # The process must hold ONE HIP runtime: the one torch ships, which owns the device memory
        # and the streams handed to this library.  torch's libraries ask for "libamdhip64.so" and
        # libcsp.so for the soname "libamdhip64.so.7"; loaded first, libcsp.so pulls in the system
        # runtime and torch then maps its own copy beside it (two runtimes, two HSA instances; their
        # exit handlers have aborted finished processes, and a stream of one means nothing to the
        # other).  With torch's copy already mapped the loader resolves libcsp.so against it.
        import torch  # noqa: F401
        L = C.CDLL(_LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        dp = C.POINTER(_CDesc)
        L.csp_strerror.argtypes = [C.c_int]; L.csp_strerror.restype = C.c_char_p
        L.csp_version.argtypes = []; L.csp_version.restype = C.c_char_p
        L.csp_score_workspace_bytes.argtypes = [dp]; L.csp_score_workspace_bytes.restype = sz
        L.csp_select_workspace_bytes.argtypes = [dp]; L.csp_select_workspace_bytes.restype = sz
        L.csp_decode_workspace_bytes.argtypes = [dp, i32]; L.csp_decode_workspace_bytes.restype = sz
        L.csp_score.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]; L.csp_score.restype = C.c_int
        L.csp_score_lse.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]; L.csp_score_lse.restype = C.c_int
        L.csp_select.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, sz, vp]; L.csp_select.restype = C.c_int
        L.csp_compact.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp, i64, i64, i64, vp, vp]; L.csp_compact.restype = C.c_int
        L.csp_decode_attn.argtypes = [dp, vp, vp, vp, i64, i64, i64, vp, i32, vp, vp, sz, vp]; L.csp_decode_attn.restype = C.c_int
        L.csp_static_scratch_bytes.argtypes = []; L.csp_static_scratch_bytes.restype = sz
        L.csp_decode_attn_static.argtypes = [dp, vp, vp, vp, i64, i64, i64, vp, i32, vp, vp]; L.csp_decode_attn_static.restype = C.c_int
        L.csp_decode_step.argtypes = [dp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, vp, sz, vp]; L.csp_decode_step.restype = C.c_int
        L.csp_decode_step_phase.argtypes = [dp, i32, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, vp, sz, vp]; L.csp_decode_step_phase.restype = C.c_int
        L.csp_append_kv.argtypes = [dp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp]; L.csp_append_kv.restype = C.c_int
        L.csp_gather_modality.argtypes = [dp, vp, vp, i32, vp, vp, i32, vp]; L.csp_gather_modality.restype = C.c_int
        L.csp_window_push.argtypes = [dp, vp, vp, i32, vp]; L.csp_window_push.restype = C.c_int
        L.csp_probe_stream.argtypes = [vp, vp, C.c_size_t, vp, vp]; L.csp_probe_stream.restype = C.c_int
        L.csp_decode_step_window.argtypes = [dp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, vp, i32, vp, sz, vp]
        L.csp_decode_step_window.restype = C.c_int
        L.csp_reprune_workspace_bytes.argtypes = [dp, i32]; L.csp_reprune_workspace_bytes.restype = sz
        L.csp_reprune.argtypes = [dp, vp, i32, vp, vp, i64, i64, i64, i32, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.csp_reprune.restype = C.c_int
        _lib = L
    return _lib


def csp_strerror(code: int) -> str:
    return load_library().csp_strerror(int(code)).decode()


def csp_version() -> str:
    return load_library().csp_version().decode()


class Desc:
    """Python mirror of `csp_desc`.  Host arrays are kept alive by this object;
    device arrays are torch int32 tensors (or raw pointers for validation tests)."""

    def __init__(self, *, dtype: str, B: int, H_q: int, H_kv: int, D: int, sel_group: int,
                 window_O: int, recent_R: int, max_seqlen: int, cu_seqlens_host: Optional[Sequence[int]],
                 budget_T_host: Optional[Sequence[int]], cu_seqlens=None, budget_T=None,
                 k_strides=(0, 0), v_strides=(0, 0), causal: bool = True, n_score: float = 0.0,
                 n_decode: float = 1.0, cross_ratio: float = 0.5, score_wait_us: int = 0):
        self._cu_host = (C.c_int32 * (B + 1))(*[int(x) for x in cu_seqlens_host]) if cu_seqlens_host is not None else None
        self._bt_host = (C.c_int32 * B)(*[int(x) for x in budget_T_host]) if budget_T_host is not None else None
        self._keep = (cu_seqlens, budget_T)
        c = _CDesc()
        c.dtype = {"bf16": CSP_BF16, "f32": CSP_F32}.get(dtype, dtype if isinstance(dtype, int) else -1)
        c.B, c.H_q, c.H_kv, c.D, c.sel_group = B, H_q, H_kv, D, sel_group
        c.window_O, c.recent_R, c.causal, c.max_seqlen = window_O, recent_R, int(bool(causal)), max_seqlen
        c.n_score, c.n_decode, c.cross_ratio = float(n_score), float(n_decode), float(cross_ratio)
        c.cu_seqlens_host = C.cast(self._cu_host, C.c_void_p) if self._cu_host is not None else None
        c.budget_T_host = C.cast(self._bt_host, C.c_void_p) if self._bt_host is not None else None
        c.cu_seqlens = _ptr(cu_seqlens)
        c.budget_T = _ptr(budget_T)
        c.k_stride_tok, c.k_stride_head = int(k_strides[0]), int(k_strides[1])
        c.v_stride_tok, c.v_stride_head = int(v_strides[0]), int(v_strides[1])
        c.score_wait_us = int(score_wait_us)
        self.c = c

    def ref(self):
        return C.byref(self.c)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise CspError(rc, where)


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def csp_score_workspace_bytes(desc: Desc) -> int:
    return int(load_library().csp_score_workspace_bytes(desc.ref()))


def csp_select_workspace_bytes(desc: Desc) -> int:
    return int(load_library().csp_select_workspace_bytes(desc.ref()))


def csp_decode_workspace_bytes(desc: Desc, max_kv_len: int) -> int:
    return int(load_library().csp_decode_workspace_bytes(desc.ref(), int(max_kv_len)))


def csp_score(desc: Desc, q_win, k, modality, score_self, score_cross, ws, stream=None) -> None:
    _check(load_library().csp_score(desc.ref(), _ptr(q_win), _ptr(k), _ptr(modality), _ptr(score_self),
                                    _ptr(score_cross), _ptr(ws), _nbytes(ws), _stream(stream)), "csp_score")


def csp_score_lse(desc: Desc, q_win, k, modality, row_lse, score_self, score_cross, ws, stream=None) -> None:
    _check(load_library().csp_score_lse(desc.ref(), _ptr(q_win), _ptr(k), _ptr(modality), _ptr(row_lse), _ptr(score_self),
                                        _ptr(score_cross), _ptr(ws), _nbytes(ws), _stream(stream)), "csp_score_lse")


def csp_select(desc: Desc, score_self, score_cross, modality, kept_idx, kept_cap: int, kept_cnt,
               ws=None, stream=None) -> None:
    _check(load_library().csp_select(desc.ref(), _ptr(score_self), _ptr(score_cross), _ptr(modality),
                                     _ptr(kept_idx), int(kept_cap), _ptr(kept_cnt), _ptr(ws), _nbytes(ws),
                                     _stream(stream)), "csp_select")


def csp_compact(desc: Desc, k, v, kept_idx, kept_cap: int, kept_cnt, k_out, v_out, out_strides,
                kv_len=None, stream=None) -> None:
    """out_strides = (stride_b, stride_head, stride_tok) of the pruned cache, in elements."""
    _check(load_library().csp_compact(desc.ref(), _ptr(k), _ptr(v), _ptr(kept_idx), int(kept_cap), _ptr(kept_cnt),
                                      _ptr(k_out), _ptr(v_out), int(out_strides[0]), int(out_strides[1]),
                                      int(out_strides[2]), _ptr(kv_len), _stream(stream)), "csp_compact")


def csp_decode_attn(desc: Desc, q, k_cache, v_cache, cache_strides, kv_len, max_kv_len: int, out, ws,
                    stream=None) -> None:
    _check(load_library().csp_decode_attn(desc.ref(), _ptr(q), _ptr(k_cache), _ptr(v_cache), int(cache_strides[0]),
                                          int(cache_strides[1]), int(cache_strides[2]), _ptr(kv_len), int(max_kv_len),
                                          _ptr(out), _ptr(ws), _nbytes(ws), _stream(stream)), "csp_decode_attn")


def csp_static_scratch_bytes() -> int:
    return int(load_library().csp_static_scratch_bytes())


def csp_decode_attn_static(desc: Desc, q, k_cache, v_cache, cache_strides, kv_len, max_kv_len: int, out, stream=None) -> None:
    """csp_decode_attn without a workspace argument: the library's own device scratch array is used"""
    _check(load_library().csp_decode_attn_static(desc.ref(), _ptr(q), _ptr(k_cache), _ptr(v_cache), int(cache_strides[0]),
                                                 int(cache_strides[1]), int(cache_strides[2]), _ptr(kv_len), int(max_kv_len),
                                                 _ptr(out), _stream(stream)), "csp_decode_attn_static")


def csp_append_kv(desc: Desc, k_new, v_new, k_cache, v_cache, cache_strides, cache_cap: int, kv_len,
                  stream=None) -> None:
    _check(load_library().csp_append_kv(desc.ref(), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                        int(cache_strides[0]), int(cache_strides[1]), int(cache_strides[2]),
                                        int(cache_cap), _ptr(kv_len), _stream(stream)), "csp_append_kv")


def csp_decode_step(desc: Desc, q, k_new, v_new, k_cache, v_cache, cache_strides, cache_cap: int, kv_len, out, ws,
                    stream=None) -> None:
    _check(load_library().csp_decode_step(desc.ref(), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                          int(cache_strides[0]), int(cache_strides[1]), int(cache_strides[2]),
                                          int(cache_cap), _ptr(kv_len), _ptr(out), _ptr(ws), _nbytes(ws),
                                          _stream(stream)), "csp_decode_step")


def csp_decode_step_phase(desc: Desc, phase: int, q, k_new, v_new, k_cache, v_cache, cache_strides, cache_cap: int,
                          kv_len, out, ws, stream=None) -> None:
    _check(load_library().csp_decode_step_phase(desc.ref(), int(phase), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                                _ptr(v_cache), int(cache_strides[0]), int(cache_strides[1]),
                                                int(cache_strides[2]), int(cache_cap), _ptr(kv_len), _ptr(out), _ptr(ws),
                                                _nbytes(ws), _stream(stream)), "csp_decode_step_phase")


def csp_gather_modality(desc: Desc, modality, kept_idx, kept_cap: int, kept_cnt, mod_cache, cache_cap: int,
                        stream=None) -> None:
    _check(load_library().csp_gather_modality(desc.ref(), _ptr(modality), _ptr(kept_idx), int(kept_cap), _ptr(kept_cnt),
                                              _ptr(mod_cache), int(cache_cap), _stream(stream)), "csp_gather_modality")


def csp_window_push(desc: Desc, q_new, q_ring, slot: int, stream=None) -> None:
    _check(load_library().csp_window_push(desc.ref(), _ptr(q_new), _ptr(q_ring), int(slot), _stream(stream)),
           "csp_window_push")


def csp_probe_stream(src, dst, sink, stream=None) -> None:
    """Reads all of `src` (dst None) or copies it to `dst`: the box's read / copy rate (measurement aid)."""
    _check(load_library().csp_probe_stream(_ptr(src), _ptr(dst) if dst is not None else None, _nbytes(src), _ptr(sink),
                                           _stream(stream)), "csp_probe_stream")


def csp_reprune_workspace_bytes(desc: Desc, cache_cap: int) -> int:
    return int(load_library().csp_reprune_workspace_bytes(desc.ref(), int(cache_cap)))


def csp_reprune(desc: Desc, q_ring, ring_start: int, k_cache, v_cache, cache_strides, cache_cap: int, mod_cache, kv_len,
                score_self, score_cross, kept_idx, kept_cap: int, kept_cnt, ws, stream=None) -> None:
    _check(load_library().csp_reprune(desc.ref(), _ptr(q_ring), int(ring_start), _ptr(k_cache), _ptr(v_cache),
                                      int(cache_strides[0]), int(cache_strides[1]), int(cache_strides[2]), int(cache_cap),
                                      _ptr(mod_cache), _ptr(kv_len), _ptr(score_self), _ptr(score_cross), _ptr(kept_idx),
                                      int(kept_cap), _ptr(kept_cnt), _ptr(ws), _nbytes(ws), _stream(stream)), "csp_reprune")


def csp_decode_step_window(desc: Desc, q, k_new, v_new, k_cache, v_cache, cache_strides, cache_cap: int, kv_len, out,
                           q_ring, slot: int, ws, stream=None) -> None:
    _check(load_library().csp_decode_step_window(desc.ref(), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                                 int(cache_strides[0]), int(cache_strides[1]), int(cache_strides[2]),
                                                 int(cache_cap), _ptr(kv_len), _ptr(out), _ptr(q_ring), int(slot), _ptr(ws),
                                                 _nbytes(ws), _stream(stream)), "csp_decode_step_window")
