"""Helpers of the GPU parity tests: host<->device marshalling of a
csp_workloads.Case and the comparison rules (tolerances)."""
from __future__ import annotations

import numpy as np
import torch

from paper_2412_04652_amd.runner import CspLayer

REL = 2e-3          # spec tolerance: fp32 accumulation of bf16 inputs
ABS_FLOOR = 1e-6    # times the largest score of the vector


def to_dev(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """numpy array of float32 values or bf16 bit patterns -> device tensor."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def from_dev_bits(t: torch.Tensor, dtype: str) -> np.ndarray:
    """device tensor -> numpy float32 values or bf16 bit patterns (uint16)."""
    if dtype == "bf16":
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


# ---- guard bands -------------------------------------------------------------------------------
# Every buffer a layer hands to the library (outputs, workspaces, caches) is re-seated inside a larger
# allocation with GUARD bytes of a known pattern on both sides; after each GPU test the pattern must be
# intact (tests/conftest.py): a kernel that writes outside what it was given fails the test that ran it.
GUARD = 4096
CANARY = 0xA5
_GUARDED_FIELDS = ("score_self", "score_cross", "ws_score", "kept_idx", "kept_cnt", "k_cache", "v_cache", "kv_len",
                   "ws_decode", "out", "mod_cache", "q_ring", "rp_self", "rp_cross", "rp_idx", "rp_cnt", "ws_reprune")
_LIVE = []   # (name, whole allocation, payload bytes) of the layers guarded since the last check


def guard_layer(layer) -> None:
    for name in _GUARDED_FIELDS:
        t = getattr(layer, name, None)
        if t is None:
            continue
        n = t.numel() * t.element_size()
        whole = torch.full((n + 2 * GUARD,), CANARY, dtype=torch.uint8, device=t.device)
        inner = whole[GUARD:GUARD + n].view(t.dtype).view(t.shape)
        inner.copy_(t)   # (kv_len and the re-pruning state start from defined values)
        setattr(layer, name, inner)
        _LIVE.append((name, whole, n))


_ORIG_INIT = None


def install_guards() -> None:
    """From now on every CspLayer that is built has its buffers guarded (until remove_guards)."""
    global _ORIG_INIT
    if _ORIG_INIT is None:
        _ORIG_INIT = CspLayer.__init__

        def guarded_init(self, *a, **kw):
            _ORIG_INIT(self, *a, **kw)
            guard_layer(self)

        CspLayer.__init__ = guarded_init


def remove_guards() -> None:
    global _ORIG_INIT
    if _ORIG_INIT is not None:
        CspLayer.__init__ = _ORIG_INIT
        _ORIG_INIT = None


def check_guards() -> None:
    """Asserts that no guard band of the layers guarded since the last call was written to."""
    try:
        for name, whole, n in _LIVE:
            lo, hi = whole[:GUARD], whole[GUARD + n:]
            assert bool((lo == CANARY).all()), f"{name}: bytes in front of the buffer were overwritten"
            assert bool((hi == CANARY).all()), f"{name}: bytes behind the buffer were overwritten"
    finally:
        _LIVE.clear()


class DeviceCase:
    def __init__(self, case, decode_cap: int = 0, device="cuda:0", reprune: bool = False, score_wait_us: int = 0):
        self.case = case
        self.q_win = to_dev(case.q_win, case.dtype, device)
        self.k = to_dev(case.k, case.dtype, device)
        self.v = to_dev(case.v, case.dtype, device)
        self.modality = torch.from_numpy(case.modality).to(device)
        self.layer = CspLayer(dtype=case.dtype, H_q=case.H_q, H_kv=case.H_kv, D=case.D, O=case.O, R=case.R,
                              cu_seqlens=case.cu_seqlens.tolist(), budgets=case.budget_T.tolist(),
                              sel_group=case.sel_group, cross_ratio=case.cross_ratio, n_score=case.n_score,
                              n_decode=case.n_decode, decode_cap=decode_cap, device=device, reprune=reprune,
                              score_wait_us=score_wait_us)


def assert_scores_close(gpu: np.ndarray, ref: np.ndarray, what: str = "") -> None:
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    assert gpu.shape == ref.shape, f"{what}: shape {gpu.shape} vs {ref.shape}"
    if ref.size == 0:
        return
    tol = REL * np.abs(ref) + ABS_FLOOR * np.abs(ref).max()
    bad = np.abs(gpu - ref) > tol
    if bad.any():
        i = int(np.argmax(np.abs(gpu - ref) - tol))
        raise AssertionError(f"{what}: {int(bad.sum())} of {ref.size} scores out of tolerance; "
                             f"worst at {i}: gpu={gpu.flat[i]!r} ref={ref.flat[i]!r}")


def assert_decode_close(gpu: np.ndarray, ref: np.ndarray, what: str = "") -> None:
    """Per head vector: |g-o| <= REL * max(|o_d|, max|o|)."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    scale = np.maximum(np.abs(ref), np.abs(ref).max(axis=-1, keepdims=True))
    bad = np.abs(gpu - ref) > REL * scale + 1e-30
    if bad.any():
        raise AssertionError(f"{what}: {int(bad.sum())} of {ref.size} outputs out of tolerance; "
                             f"max err {np.abs(gpu - ref).max():.3e} vs scale {scale.max():.3e}")


def assert_kept_equivalent(gpu_idx: np.ndarray, ref_idx: np.ndarray, a_self: np.ndarray, a_cross: np.ndarray,
                           mod: np.ndarray, L: int, R: int, what: str = "") -> int:
    """Kept sets must be identical except for keys whose oracle score lies within
    REL of the oracle's K-th score of that key's region (single-modality window:
    text keys rank by a_self, visual keys by a_cross or the reverse).  Returns the
    number of differing keys."""
    g, r = set(gpu_idx.tolist()), set(ref_idx.tolist())
    assert len(gpu_idx) == len(ref_idx), f"{what}: kept {len(gpu_idx)} vs oracle {len(ref_idx)}"
    assert (np.diff(gpu_idx) > 0).all(), f"{what}: indices not ascending/unique"
    assert gpu_idx[-R:].tolist() == list(range(L - R, L)) if R else True, f"{what}: recent keys missing"
    diff = sorted(g ^ r)
    if not diff:
        return 0
    qmod = int(mod[L - 1])          # all-window-one-modality cases only
    for m in (0, 1):
        score = a_self if m == qmod else a_cross
        kept_m = [j for j in ref_idx if j < L - R and mod[j] == m]
        if not kept_m:
            assert not [j for j in diff if mod[j] == m], f"{what}: modality {m} differs with empty region"
            continue
        tau = min(score[j] for j in kept_m)
        floor = ABS_FLOOR * float(np.max(score[: L - R]))
        for j in diff:
            if mod[j] != m:
                continue
            assert abs(score[j] - tau) <= REL * tau + floor, \
                f"{what}: key {j} differs but its score {score[j]!r} is not near the threshold {tau!r}"
        gm = sum(1 for j in gpu_idx if j < L - R and mod[j] == m)
        assert gm == len(kept_m), f"{what}: modality {m} kept {gm} vs {len(kept_m)}"
    return len(diff)


def assert_kept_equivalent_mixed(gpu_idx: np.ndarray, ref_idx: np.ndarray, a_self: np.ndarray, a_cross: np.ndarray,
                                 K_s: int, K_c: int, L: int, R: int, what: str = "") -> int:
    """A window with both modalities: every prefix key ranks in both regions and the kept set is
    the union of the two top-K sets plus the recent keys.  A key kept by one side only must have
    a score within REL of one of the two thresholds (the oracle's K-th largest self / cross score).
    Returns the number of differing keys."""
    P = L - R
    assert (np.diff(gpu_idx) > 0).all(), f"{what}: indices not ascending/unique"
    assert R == 0 or gpu_idx[-R:].tolist() == list(range(P, L)), f"{what}: recent keys missing"
    diff = sorted(set(gpu_idx.tolist()) ^ set(ref_idx.tolist()))
    tau_s = np.sort(a_self[:P])[P - K_s] if K_s > 0 else np.inf
    tau_c = np.sort(a_cross[:P])[P - K_c] if K_c > 0 else np.inf
    for j in diff:
        near_s = K_s > 0 and abs(a_self[j] - tau_s) <= REL * tau_s + ABS_FLOOR * float(np.max(a_self[:P]))
        near_c = K_c > 0 and abs(a_cross[j] - tau_c) <= REL * tau_c + ABS_FLOOR * float(np.max(a_cross[:P]))
        assert near_s or near_c, f"{what}: key {j} differs, self {a_self[j]!r} vs {tau_s!r}, cross {a_cross[j]!r} vs {tau_c!r}"
    return len(diff)
