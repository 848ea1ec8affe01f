"""Device-memory plumbing around the C ABI: owns the intermediate buffers of one
layer's pruning pass and decode loop and calls the binding in order.  No
arithmetic happens here; every step runs in the HIP kernels."""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as B_


def _tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class CspLayer:
    """Buffers and descriptor for one attention layer of one batch.

    K and V are token-packed, head-major: [H_kv, total_tokens, D]
    (k_strides=(D, total_tokens*D)) unless other strides are given.  The pruned
    cache is [B, H_kv, cache_cap, D]."""

    def __init__(self, *, dtype: str, H_q: int, H_kv: int, D: int, O: int, R: int,
                 cu_seqlens: Sequence[int], budgets: Sequence[int], sel_group: int = 1,
                 cross_ratio: float = 0.5, n_score: float = 0.0, n_decode: float = 1.0,
                 decode_cap: int = 0, device="cuda:0", k_strides=None, v_strides=None, causal: bool = True,
                 reprune: bool = False, score_wait_us: int = 0):
        self.device = torch.device(device)
        self.dtype, self.H_q, self.H_kv, self.D, self.O, self.R = dtype, H_q, H_kv, D, O, R
        self.B = len(budgets)
        self.cu_host = [int(x) for x in cu_seqlens]
        self.budgets = [int(x) for x in budgets]
        self.total = self.cu_host[-1]
        lens = [self.cu_host[b + 1] - self.cu_host[b] for b in range(self.B)]
        self.max_seqlen = max(lens)
        self.sel_group = sel_group
        self.H_sel = H_q // sel_group
        self.kept_cap = max(min(t, l) for t, l in zip(self.budgets, lens))
        self.cache_cap = self.kept_cap + decode_cap
        dev = self.device
        self.cu = torch.tensor(self.cu_host, dtype=torch.int32, device=dev)
        self.bt = torch.tensor(self.budgets, dtype=torch.int32, device=dev)
        ks = k_strides if k_strides is not None else (D, self.total * D)
        vs = v_strides if v_strides is not None else (D, self.total * D)
        self.desc = B_.Desc(dtype=dtype, B=self.B, H_q=H_q, H_kv=H_kv, D=D, sel_group=sel_group, window_O=O,
                            recent_R=R, max_seqlen=self.max_seqlen, cu_seqlens_host=self.cu_host,
                            budget_T_host=self.budgets, cu_seqlens=self.cu, budget_T=self.bt,
                            k_strides=ks, v_strides=vs, causal=causal, n_score=n_score, n_decode=n_decode,
                            cross_ratio=cross_ratio, score_wait_us=score_wait_us)
        self.score_self = torch.empty((self.H_sel, self.total), dtype=torch.float32, device=dev)
        self.score_cross = torch.empty((self.H_sel, self.total), dtype=torch.float32, device=dev)
        self.ws_score = torch.empty(max(B_.csp_score_workspace_bytes(self.desc), 16), dtype=torch.uint8, device=dev)
        self.kept_idx = torch.empty((self.B, self.H_sel, self.kept_cap), dtype=torch.int32, device=dev)
        self.kept_cnt = torch.empty((self.B, self.H_sel, 4), dtype=torch.int32, device=dev)
        self.k_cache = torch.empty((self.B, H_kv, self.cache_cap, D), dtype=_tdtype(dtype), device=dev)
        self.v_cache = torch.empty((self.B, H_kv, self.cache_cap, D), dtype=_tdtype(dtype), device=dev)
        self.cache_strides = (H_kv * self.cache_cap * D, self.cache_cap * D, D)
        self.kv_len = torch.zeros((self.B, H_kv), dtype=torch.int32, device=dev)
        self.ws_decode = torch.empty(max(B_.csp_decode_workspace_bytes(self.desc, self.cache_cap), 16),
                                     dtype=torch.uint8, device=dev)
        self.out = torch.empty((self.B, H_q, D), dtype=torch.float32, device=dev)
        # re-pruning while decoding: modality of the cached keys, the ring of the last O queries,
        # scores and kept positions in cache coordinates
        self.reprune_enabled = reprune
        if reprune:
            self.mod_cache = torch.zeros((self.B, self.H_sel, self.cache_cap), dtype=torch.uint8, device=dev)
            self.q_ring = torch.zeros((self.B, H_q, O, D), dtype=_tdtype(dtype), device=dev)
            self.pushes = 0
            self.rp_self = torch.empty((self.B, self.H_sel, self.cache_cap), dtype=torch.float32, device=dev)
            self.rp_cross = torch.empty((self.B, self.H_sel, self.cache_cap), dtype=torch.float32, device=dev)
            self.rp_cap = max(self.budgets)
            self.rp_idx = torch.empty((self.B, self.H_sel, self.rp_cap), dtype=torch.int32, device=dev)
            self.rp_cnt = torch.empty((self.B, self.H_sel, 4), dtype=torch.int32, device=dev)
            self.ws_reprune = torch.empty(max(B_.csp_reprune_workspace_bytes(self.desc, self.cache_cap), 16),
                                          dtype=torch.uint8, device=dev)

    # -- the four calls of the path, in order ---------------------------------
    def score(self, q_win, k, modality, stream=None):
        B_.csp_score(self.desc, q_win, k, modality, self.score_self, self.score_cross, self.ws_score, stream)

    def score_fallbacks(self) -> int:
        """tasks of the last csp_score call whose wait for the other chunks ran out (first counter of the workspace)"""
        return int(self.ws_score[:4].view(torch.int32).item())

    def score_lse(self, q_win, k, modality, row_lse, stream=None):
        """score with the window rows' log-sum-exp supplied (the keys are read once)"""
        B_.csp_score_lse(self.desc, q_win, k, modality, row_lse, self.score_self, self.score_cross, self.ws_score, stream)

    def select(self, modality, stream=None, score_self=None, score_cross=None):
        B_.csp_select(self.desc, self.score_self if score_self is None else score_self,
                      self.score_cross if score_cross is None else score_cross, modality,
                      self.kept_idx, self.kept_cap, self.kept_cnt, None, stream)

    def compact(self, k, v, stream=None):
        B_.csp_compact(self.desc, k, v, self.kept_idx, self.kept_cap, self.kept_cnt, self.k_cache, self.v_cache,
                       self.cache_strides, self.kv_len, stream)

    def prune(self, q_win, k, v, modality, stream=None):
        self.score(q_win, k, modality, stream)
        self.select(modality, stream)
        self.compact(k, v, stream)
        if self.reprune_enabled:
            B_.csp_gather_modality(self.desc, modality, self.kept_idx, self.kept_cap, self.kept_cnt, self.mod_cache,
                                   self.cache_cap, stream)
            # the prefill window, in temporal order: slot 0 is the oldest
            if stream is None or isinstance(stream, int):
                self.q_ring.copy_(q_win)
            else:
                with torch.cuda.stream(stream):
                    self.q_ring.copy_(q_win)
            self.pushes = 0

    def push_query(self, q, stream=None):
        """records the current step's queries in the ring of the last O"""
        B_.csp_window_push(self.desc, q, self.q_ring, self.pushes % self.O, stream)
        self.pushes += 1

    def decode_step_window(self, q, k_new, v_new, stream=None, out: Optional[torch.Tensor] = None):
        """decode_step + push_query in the same launches"""
        o = self.out if out is None else out
        B_.csp_decode_step_window(self.desc, q, k_new, v_new, self.k_cache, self.v_cache, self.cache_strides,
                                  self.cache_cap, self.kv_len, o, self.q_ring, self.pushes % self.O, self.ws_decode, stream)
        self.pushes += 1
        return o

    def reprune(self, stream=None):
        """prunes the grown cache in place (sequences within their budget are left alone)"""
        B_.csp_reprune(self.desc, self.q_ring, self.pushes % self.O, self.k_cache, self.v_cache, self.cache_strides,
                       self.cache_cap, self.mod_cache, self.kv_len, self.rp_self, self.rp_cross, self.rp_idx,
                       self.rp_cap, self.rp_cnt, self.ws_reprune, stream)

    def append(self, k_new, v_new, stream=None):
        B_.csp_append_kv(self.desc, k_new, v_new, self.k_cache, self.v_cache, self.cache_strides,
                         self.cache_cap, self.kv_len, stream)

    def decode(self, q, stream=None, out: Optional[torch.Tensor] = None):
        o = self.out if out is None else out
        B_.csp_decode_attn(self.desc, q, self.k_cache, self.v_cache, self.cache_strides, self.kv_len,
                           self.cache_cap, o, self.ws_decode, stream)
        return o

    def decode_step(self, q, k_new, v_new, stream=None, out: Optional[torch.Tensor] = None):
        """append + attend in one call"""
        o = self.out if out is None else out
        B_.csp_decode_step(self.desc, q, k_new, v_new, self.k_cache, self.v_cache, self.cache_strides,
                           self.cache_cap, self.kv_len, o, self.ws_decode, stream)
        return o

    def decode_step_phase(self, phase, q, k_new, v_new, stream=None, out: Optional[torch.Tensor] = None):
        """one of the two launches of decode_step (1: stream the cache, 2: merge)"""
        o = self.out if out is None else out
        B_.csp_decode_step_phase(self.desc, phase, q, k_new, v_new, self.k_cache, self.v_cache, self.cache_strides,
                                 self.cache_cap, self.kv_len, o, self.ws_decode, stream)
        return o
