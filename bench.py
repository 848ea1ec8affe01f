#!/usr/bin/env python3
"""Benchmark of the CSP hot path on one MI355X.

A step is one pass of the whole path over the 7B-shape 16k-token batch
(32 layers x batch 4 x 32 heads x 16384 tokens, head_dim 128, bf16, window 64):
per layer score -> select -> compact at the given budget, then the decode loop
(append + n-softmax attention over the pruned cache) for every layer and every
decode step.  Inputs are synthetic, seeded, and resident in HBM before the timed
region starts.

Prints ONE JSON line: `value` is pruned KV tokens per second over
score+select+compact (layers x tokens / time of the pruning phase); the decode
attention bandwidth, the roofline of the dominant kernel and the CPU-oracle
baseline ride along in the same object.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak

WORKLOADS = {
    # name: (layers, B, H, D, L, window, images, vis_per_image, text, decode_steps)
    "7b_16k": dict(layers=32, B=4, H=32, D=128, L=16384, O=64, images=20, vis=576, text=4864, steps=128),
    "7b_4k": dict(layers=1, B=1, H=32, D=128, L=4096, O=64, images=4, vis=576, text=1792, steps=16),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="7b_16k", choices=list(WORKLOADS))
    ap.add_argument("--budget", type=float, default=0.5, help="cache budget as a fraction of the sequence length")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = workload's)")
    ap.add_argument("--decode-steps", type=int, default=-1, help="override the decode steps per pass")
    ap.add_argument("--streams", type=int, default=2,
                    help="HIP streams the independent layers of the pruning phase alternate over (1 = strictly serial)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-second-budget", action="store_true")
    ap.add_argument("--sel-group", type=int, default=1,
                    help="query heads whose scores are summed into one index set (1 = per head, H = one set per layer)")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the extra passes over 8 layers: mixed-modality window, n-softmax scoring, cross-ratio sweep")
    ap.add_argument("--no-head-averaged", action="store_true",
                    help="skip the extra pass with one index set per layer (scores summed over all heads)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the lines for the other configurations (single 4k layer, GQA ragged, 64k)")
    return ap.parse_args()


def build_inputs(cfg, n_layers, device, window_text=0):
    """window_text > 0: the sequences end with an image and `window_text` text tokens, so the
    observation window holds queries of both modalities."""
    import numpy as np
    import csp_workloads as W
    layers = []
    for l in range(n_layers):
        rng = np.random.default_rng(1000 + l)
        if window_text:
            layouts = [W.layout_mixed_window(rng, [cfg["vis"]] * cfg["images"], cfg["text"], window_text)
                       for _ in range(cfg["B"])]
        elif cfg["L"] == 4096:
            layouts = [W.layout_7b_4k() for _ in range(cfg["B"])]
        else:
            layouts = [W.layout_random(rng, [cfg["vis"]] * cfg["images"], cfg["text"], cfg["O"]) for _ in range(cfg["B"])]
        q, k, v, mod, cu_dev, cu = W.device_qkv(layouts, H_q=cfg["H"], H_kv=cfg["H"], D=cfg["D"], O=cfg["O"],
                                                seed=l, device=device)
        layers.append(dict(q=q, k=k, v=v, mod=mod, cu=cu.tolist(), layouts=layouts))
    return layers


def make_layers(cfg, inputs, budget_frac, decode_steps, device, sel_group=1, cross_ratio=0.5, n_score=0.0):
    from paper_2412_04652_amd.runner import CspLayer
    T = int(cfg["L"] * budget_frac)
    return [CspLayer(dtype="bf16", H_q=cfg["H"], H_kv=cfg["H"], D=cfg["D"], O=cfg["O"], R=cfg["O"],
                     cu_seqlens=inp["cu"], budgets=[T] * cfg["B"], decode_cap=decode_steps, device=device,
                     sel_group=sel_group, cross_ratio=cross_ratio, n_score=n_score)
            for inp in inputs], T


def with_row_lse(cfg, inputs):
    """Copies of the inputs that carry the log-sum-exp of every window row (what the prefill
    attention of the layer would hand over), computed here with torch outside any timed region."""
    import torch
    out = []
    O, D = cfg["O"], cfg["D"]
    for inp in inputs:
        cu = inp["cu"]
        lse = torch.empty((cfg["B"], cfg["H"], O), dtype=torch.float32, device=inp["q"].device)
        for b in range(cfg["B"]):
            lo, hi = cu[b], cu[b + 1]
            L = hi - lo
            S = torch.matmul(inp["q"][b].float(), inp["k"][:, lo:hi].float().transpose(1, 2)) / (D ** 0.5)  # [H, O, L]
            pos = torch.arange(L - O, L, device=S.device)[:, None]
            S.masked_fill_(torch.arange(L, device=S.device)[None, :] > pos, float("-inf"))
            lse[b] = torch.logsumexp(S, dim=-1)
            del S
        d = dict(inp)
        d["lse"] = lse
        out.append(d)
    return out


def _score(lay, inp):
    if "lse" in inp:
        lay.score_lse(inp["q"], inp["k"], inp["mod"], inp["lse"])
    else:
        lay.score(inp["q"], inp["k"], inp["mod"])


class Timer:
    """HIP events on torch's current stream (the stream every kernel here is launched on)."""

    def __init__(self):
        import torch
        self.torch = torch
        self.pairs = {}

    def span(self, name):
        t = self.torch
        a, b = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        self.pairs.setdefault(name, []).append((a, b))
        return a, b

    def totals_ms(self):
        return {k: [a.elapsed_time(b) for a, b in v] for k, v in self.pairs.items()}


def run_pass(cfg, inputs, layers, dec, decode_steps, timer, sample_every=8, streams=None):
    """One step: prune every layer, then the decode loop.  Event pairs bracket the
    phases; every `sample_every`-th call of each kernel family is bracketed on its own."""
    import torch
    n_call = 0
    a, b = timer.span("prune")
    a.record()
    if streams is None:
        for inp, lay in zip(inputs, layers):
            sampled = (n_call % sample_every) == 0
            n_call += 1
            if sampled:
                e0, e1 = timer.span("score"); e0.record()
            _score(lay, inp)
            if sampled:
                e1.record(); e2, e3 = timer.span("select"); e2.record()
            lay.select(inp["mod"])
            if sampled:
                e3.record(); e4, e5 = timer.span("compact"); e4.record()
            lay.compact(inp["k"], inp["v"])
            if sampled:
                e5.record()
    else:
        # layers are independent: alternate them over the streams so that one layer's
        # latency-bound selection overlaps with another layer's streaming kernels
        main = torch.cuda.current_stream()
        for s in streams:
            s.wait_stream(main)
        for li, (inp, lay) in enumerate(zip(inputs, layers)):
            with torch.cuda.stream(streams[li % len(streams)]):
                _score(lay, inp)
                lay.select(inp["mod"])
                lay.compact(inp["k"], inp["v"])
        for s in streams:
            main.wait_stream(s)
    b.record()
    a, b = timer.span("decode")
    a.record()
    n_call = 0
    for t in range(decode_steps):
        dq, dk, dv = dec["q"][t % dec["n"]], dec["k"][t % dec["n"]], dec["v"][t % dec["n"]]
        if t % sample_every == 0:
            # every `sample_every`-th step issues the two launches of decode_step layer by layer in two
            # sweeps (the layers are independent): one event pair brackets the streaming kernels of all
            # layers back to back, so the per-launch figure carries no per-launch event overhead
            e0, e1 = timer.span("decode_split_sweep"); e0.record()
            for lay in layers:
                lay.decode_step_phase(1, dq, dk, dv)
            e1.record()
            for lay in layers:
                lay.decode_step_phase(2, dq, dk, dv)
        else:
            for lay in layers:
                lay.decode_step(dq, dk, dv)  # append + attend
    b.record()


_STREAMS = {}


def measure(cfg, inputs, budget_frac, decode_steps, steps, warmup, device, n_streams=1, sel_group=1,
            cross_ratio=0.5, n_score=0.0):
    import torch
    # one set of streams for the whole process: pairs created later did not run concurrently on
    # this box (they appear to share a hardware queue), which under-reported every later measurement
    if n_streams > 1 and n_streams not in _STREAMS:
        _STREAMS[n_streams] = [torch.cuda.Stream(device=device) for _ in range(n_streams)]
    streams = _STREAMS[n_streams] if n_streams > 1 else None
    layers, T = make_layers(cfg, inputs, budget_frac, decode_steps, device, sel_group, cross_ratio, n_score)
    g = torch.Generator(device=device); g.manual_seed(777)
    nd = 4
    dec = dict(n=nd,
               q=[torch.randn((cfg["B"], cfg["H"], cfg["D"]), generator=g, device=device).to(torch.bfloat16) for _ in range(nd)],
               k=[torch.randn((cfg["B"], cfg["H"], cfg["D"]), generator=g, device=device).to(torch.bfloat16) for _ in range(nd)],
               v=[torch.randn((cfg["B"], cfg["H"], cfg["D"]), generator=g, device=device).to(torch.bfloat16) for _ in range(nd)])
    for _ in range(warmup):
        run_pass(cfg, inputs, layers, dec, decode_steps, Timer(), streams=streams)
    torch.cuda.synchronize()
    timer = Timer()
    t0 = time.perf_counter()
    for _ in range(steps):
        run_pass(cfg, inputs, layers, dec, decode_steps, timer, streams=streams)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = timer.totals_ms()
    if streams is not None:
        # per-call figures of the pruning kernels: one extra, untimed pass on a single stream
        probe = Timer()
        run_pass(cfg, inputs, layers, dec, 0, probe, sample_every=1)
        torch.cuda.synchronize()
        ms.update({k: v for k, v in probe.totals_ms().items() if k in ("score", "select", "compact")})
    n_layers, B, H, D, L, O = len(layers), cfg["B"], cfg["H"], cfg["D"], cfg["L"], cfg["O"]
    e = 2
    Hs = H // sel_group                           # index sets per sequence
    avg = lambda xs: sum(xs) / max(len(xs), 1)
    med = lambda xs: sorted(xs)[len(xs) // 2] if xs else 0.0
    # algorithmic bytes per launch (one layer)
    by_score = B * (H * L * D * e + H * O * D * e + L + 2 * Hs * (L - O) * 4)
    by_select = B * (2 * Hs * (L - O) * 4 + Hs * T * 4)
    by_compact = B * (4 * H * T * D * e + Hs * T * 4)
    kv_mean = T + (decode_steps + 1) / 2.0
    by_decode = B * (2 * H * kv_mean * D * e + H * D * (e + 4))
    prune_ms = avg(ms["prune"])
    res = dict(
        budget=budget_frac, T=T, layers=n_layers, sel_group=sel_group,
        prune_ms=prune_ms,
        tokens_per_s=n_layers * B * L / (prune_ms * 1e-3),
        prune_gbps=n_layers * (by_score + by_select + by_compact) / (prune_ms * 1e-3) / 1e9,
        ms_per_step=wall / steps * 1e3,
        kernels={
            "score": dict(ms=avg(ms["score"]), ms_median=med(ms["score"]), samples=len(ms["score"]),
                                     gbps=by_score / (avg(ms["score"]) * 1e-3) / 1e9, bytes=by_score),
            "select": dict(ms=avg(ms["select"]), ms_median=med(ms["select"]), samples=len(ms["select"]),
                           gbps=by_select / (avg(ms["select"]) * 1e-3) / 1e9, bytes=by_select),
            "compact": dict(ms=avg(ms["compact"]), ms_median=med(ms["compact"]), samples=len(ms["compact"]),
                            gbps=by_compact / (avg(ms["compact"]) * 1e-3) / 1e9, bytes=by_compact),
        })
    # kept keys per (sequence, index set): below T when the two top-K sets overlap (mixed windows)
    res["kept_mean"] = float(torch.stack([l.kept_cnt[:, :, 0].float().mean() for l in layers]).mean())
    # tasks of the last scoring launch of each layer whose wait for another workgroup's statistics ran
    # out (they recompute them themselves, with the same result): 0 unless the chip was shared
    res["score_fallbacks"] = int(sum(l.score_fallbacks() for l in layers))
    if decode_steps > 0:
        dec_ms = avg(ms["decode"])
        sweeps = [x / n_layers for x in ms["decode_split_sweep"]]   # per launch
        ms["decode_split"] = sweeps
        call_ms = avg(sweeps)
        res.update(decode_ms_per_token=dec_ms / decode_steps,
                   decode_gbps=by_decode * n_layers * decode_steps / (dec_ms * 1e-3) / 1e9)
        # the whole step: algorithmic bytes of both phases over the sum of their event times
        res["step_gbps"] = n_layers * (by_score + by_select + by_compact + by_decode * decode_steps) / ((prune_ms + dec_ms) * 1e-3) / 1e9
        res["kernels"]["decode_split"] = dict(ms=call_ms, ms_median=med(ms["decode_split"]), samples=len(ms["decode_split"]) * n_layers,
                                              gbps=by_decode / (call_ms * 1e-3) / 1e9, bytes=by_decode)
    del layers
    torch.cuda.empty_cache()
    return res


def measure_reprune(cfg, inputs, budget_frac, period, cycles, device):
    """Re-pruning while decoding: every layer is pruned after prefill, then `cycles` times: `period`
    decode steps (append + attend + window push, one call) followed by csp_reprune on every layer (cache
    T + period -> T).  Times one csp_reprune call per layer and the decode steps between them."""
    import torch
    from paper_2412_04652_amd.runner import CspLayer
    T = int(cfg["L"] * budget_frac)
    B, H, D, O = cfg["B"], cfg["H"], cfg["D"], cfg["O"]
    layers = [CspLayer(dtype="bf16", H_q=H, H_kv=H, D=D, O=O, R=O, cu_seqlens=inp["cu"], budgets=[T] * B,
                       decode_cap=period, device=device, reprune=True) for inp in inputs]
    g = torch.Generator(device=device); g.manual_seed(778)
    dq, dk, dv = (torch.randn((B, H, D), generator=g, device=device).to(torch.bfloat16) for _ in range(3))
    for inp, lay in zip(inputs, layers):
        lay.prune(inp["q"], inp["k"], inp["v"], inp["mod"])
    rp_ms, dec_ms = [], []
    for c in range(cycles + 1):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for t in range(period):
            for lay in layers:
                lay.decode_step_window(dq, dk, dv)
        b.record()
        pairs = []
        for lay in layers:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); lay.reprune(); e1.record()
            pairs.append((e0, e1))
        torch.cuda.synchronize()
        if c > 0:  # first cycle warms up
            rp_ms += [x.elapsed_time(y) for x, y in pairs]
            dec_ms.append(a.elapsed_time(b))
    kept = float(torch.stack([l.kv_len.float().mean() for l in layers]).mean())
    e = 2
    rp = sum(rp_ms) / len(rp_ms)
    step = sum(dec_ms) / len(dec_ms) / period / len(layers)
    # keys of the grown cache read for scoring + kept K/V rows read and written by the compaction
    by = B * H * ((T + period) * D * e + 4 * T * D * e)
    del layers
    torch.cuda.empty_cache()
    return dict(budget=budget_frac, T=T, period=period, layers=len(inputs), reprune_ms_per_layer=rp,
                reprune_gbps=by / (rp * 1e-3) / 1e9, bytes=by, decode_step_ms_per_layer=step,
                share_of_decode_time=rp / (rp + period * step), kv_len_after=kept)


def stream_peaks(device):
    """The library's streaming probe over 2 GiB: bytes read per second by a kernel that only reads,
    bytes read + written per second by one that copies."""
    import torch
    import paper_2412_04652_amd as pkg
    n = 1 << 31
    src = torch.empty(n, dtype=torch.uint8, device=device).fill_(1)
    dst = torch.empty_like(src)
    sink = torch.zeros(4096, dtype=torch.uint8, device=device)
    out = {}
    for name, d, factor in (("read", None, 1), ("copy", dst, 2)):
        for _ in range(3):
            pkg.csp_probe_stream(src, d, sink)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            pkg.csp_probe_stream(src, d, sink)
        b.record()
        torch.cuda.synchronize()
        out[name] = 10 * factor * n / (a.elapsed_time(b) * 1e-3) / 1e9
    del src, dst
    torch.cuda.empty_cache()
    return out


def copy_peak(device):
    """Plain device-to-device copy of 2 GiB (torch's copy kernel): the achievable stream bandwidth on this machine."""
    import torch
    n = 1 << 30
    src = torch.empty(n, dtype=torch.int16, device=device).fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    return 10 * 2 * n * 2 / (a.elapsed_time(b) * 1e-3) / 1e9


# The other configurations of the workload list (they are parity-test cases first; one line each here,
# pruning on one stream): single 4k layer, GQA with ragged lengths, one 64k sequence with window 128.
OTHER_CONFIGS = {
    "7b_4k_single_layer": dict(kind="4k", B=1, H_q=32, H_kv=32, D=128, O=64, budget=0.5, sel_group=1, layers=8, steps=16, heavy=0.0),
    "gqa_28q_4kv_ragged_8k": dict(kind="gqa", B=8, H_q=28, H_kv=4, D=128, O=64, budget=0.5, sel_group=7, layers=8, steps=16, heavy=0.0),
    "long_64k_window_128": dict(kind="64k", B=1, H_q=32, H_kv=32, D=128, O=128, budget=0.1, sel_group=1, layers=4, steps=16, heavy=0.01),
}


def measure_config(name, c, device, passes=3):
    """`layers` independent layers of the configuration (different seeds), each pruned and decoded like
    a layer of the main workload; figures are per layer."""
    import numpy as np
    import torch
    import csp_workloads as W
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng({"4k": 11, "gqa": 1000, "64k": 5}[c["kind"]])
    if c["kind"] == "4k":
        layouts = [W.layout_7b_4k() for _ in range(c["B"])]
    elif c["kind"] == "gqa":
        layouts = [W.layout_gqa_ragged(rng, 8192) for _ in range(c["B"])]
    else:
        layouts = [W.layout_64k(rng) for _ in range(c["B"])]
    lens = [sum(n for _, n in seq) for seq in layouts]
    budgets = [int(L * c["budget"]) for L in lens]
    H_q, H_kv, D, O, steps = c["H_q"], c["H_kv"], c["D"], c["O"], c["steps"]
    layers = []
    for l in range(c["layers"]):
        q, k, v, mod, cu_dev, cu = W.device_qkv(layouts, H_q=H_q, H_kv=H_kv, D=D, O=O, seed=l, device=device,
                                                heavy_visual_frac=c["heavy"])
        lay = CspLayer(dtype="bf16", H_q=H_q, H_kv=H_kv, D=D, O=O, R=O, cu_seqlens=cu.tolist(), budgets=budgets,
                       sel_group=c["sel_group"], decode_cap=steps, device=device)
        layers.append((q, k, v, mod, lay))
    g = torch.Generator(device=device); g.manual_seed(779)
    B = c["B"]
    dq = torch.randn((B, H_q, D), generator=g, device=device).to(torch.bfloat16)
    dk = torch.randn((B, H_kv, D), generator=g, device=device).to(torch.bfloat16)
    dv = torch.randn((B, H_kv, D), generator=g, device=device).to(torch.bfloat16)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    spans = {"score": [], "select": [], "compact": [], "prune": [], "decode": []}

    def one_pass(timed):
        p0, p1 = ev(), ev()
        p0.record()
        marks = []
        for q, k, v, mod, lay in layers:
            e = [ev() for _ in range(4)]
            e[0].record(); lay.score(q, k, mod)
            e[1].record(); lay.select(mod)
            e[2].record(); lay.compact(k, v)
            e[3].record()
            marks.append(e)
        p1.record()
        d0, d1 = ev(), ev()
        d0.record()
        for _ in range(steps):
            for *_, lay in layers:
                lay.decode_step(dq, dk, dv)
        d1.record()
        torch.cuda.synchronize()
        if timed:
            spans["prune"].append(p0.elapsed_time(p1) / len(layers))
            spans["decode"].append(d0.elapsed_time(d1) / (len(layers) * steps))
            for e in marks:
                for i, kname in enumerate(("score", "select", "compact")):
                    spans[kname].append(e[i].elapsed_time(e[i + 1]))

    for _ in range(2):
        one_pass(False)
    for _ in range(passes):
        one_pass(True)
    e2, Hs = 2, H_q // c["sel_group"]
    by = dict(score=sum(H_kv * L * D * e2 + H_q * O * D * e2 + L + 2 * Hs * (L - O) * 4 for L in lens),
              select=sum(2 * Hs * (L - O) * 4 + Hs * T * 4 for L, T in zip(lens, budgets)),
              compact=sum(4 * H_kv * T * D * e2 + Hs * T * 4 for T in budgets))
    by_decode = sum(2 * H_kv * (T + (steps + 1) / 2.0) * D * e2 + H_q * D * (e2 + 4) for T in budgets)
    avg = lambda xs: sum(xs) / len(xs)
    prune_ms = avg(spans["prune"])
    res = dict(config=f"{name}: B{B} x {H_q} query / {H_kv} KV heads x D{D}, lengths {min(lens)}..{max(lens)}, window {O}, "
                      f"budget {c['budget']:g}, one index set per {c['sel_group']} query heads, {len(layers)} independent layers",
               tokens=sum(lens), prune_ms_per_layer=prune_ms, tokens_per_s=sum(lens) / (prune_ms * 1e-3),
               prune_gbps=sum(by.values()) / (prune_ms * 1e-3) / 1e9,
               prune_frac_of_peak=sum(by.values()) / (prune_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
               decode_ms_per_layer_step=avg(spans["decode"]), decode_gbps=by_decode / (avg(spans["decode"]) * 1e-3) / 1e9,
               score_fallbacks=int(sum(lay.score_fallbacks() for *_, lay in layers)),
               kernels={k: dict(ms=avg(spans[k]), gbps=by[k] / (avg(spans[k]) * 1e-3) / 1e9, bytes=by[k]) for k in by})
    del layers
    torch.cuda.empty_cache()
    return res


REL_TOL, ABS_FLOOR = 2e-3, 1e-6    # the parity bar of the tests: relative error of a score, floor as a fraction of the largest


def _same_result(a_s, a_c, idx, m, g_self, g_cross, g_idx, L, R):
    """The GPU's scores and kept indices of one (sequence, head) problem against the oracle's, to the bar
    of the parity tests: scores within REL_TOL; the same kept set except for keys whose oracle score is
    within REL_TOL of the threshold of their region (windows of one modality)."""
    import numpy as np
    P = L - R
    for g, r in ((g_self, a_s), (g_cross, a_c)):
        tol = REL_TOL * np.abs(r[:P]) + ABS_FLOOR * np.abs(r[:P]).max()
        if (np.abs(g[:P] - r[:P]) > tol).any():
            return False
    if len(g_idx) != len(idx) or (np.diff(g_idx) <= 0).any():
        return False
    diff = sorted(set(g_idx.tolist()) ^ set(idx.tolist()))
    qmod = int(m[L - 1])
    for mm in (0, 1):
        score = a_s if mm == qmod else a_c
        kept = [j for j in idx.tolist() if j < P and m[j] == mm]
        mine = [j for j in diff if m[j] == mm]
        if not mine:
            continue
        if not kept:
            return False
        tau = min(score[j] for j in kept)
        if any(abs(score[j] - tau) > REL_TOL * tau + ABS_FLOOR * float(score[:P].max()) for j in mine):
            return False
    return True


def cpu_baseline(cfg, inputs, budget_frac, target_s, device):
    """The CPU oracle, as it stands, on a bounded sample of (sequence, head) problems of layer 0:
    score -> select -> gather -> one decode step each.  The GPU's result for the same problems (layer 0
    pruned once more, outside any timed region) is compared with the oracle's on the way."""
    import numpy as np
    import torch
    from oracle import csp_oracle as orc
    L, O, D, H = cfg["L"], cfg["O"], cfg["D"], cfg["H"]
    T = int(L * budget_frac)
    inp = inputs[0]
    threads = orc.max_threads()
    lay0 = make_layers(cfg, inputs[:1], budget_frac, 0, device)[0][0]
    lay0.prune(inp["q"], inp["k"], inp["v"], inp["mod"])
    torch.cuda.synchronize()
    gpu_self, gpu_cross = lay0.score_self.cpu().numpy(), lay0.score_cross.cpu().numpy()
    gpu_idx, gpu_cnt = lay0.kept_idx.cpu().numpy(), lay0.kept_cnt.cpu().numpy()
    del lay0
    checked = {"n": 0, "bad": 0}

    def fetch_range(start, n):
        qs, ks, vs, ms = [], [], [], []
        for p in range(start, start + n):
            b, h = divmod(p, H)
            b %= cfg["B"]
            lo = inp["cu"][b]
            qs.append(inp["q"][b, h].float().cpu().numpy().astype(np.float64))
            ks.append(inp["k"][h, lo:lo + L].float().cpu().numpy().astype(np.float64))
            vs.append(inp["v"][h, lo:lo + L].float().cpu().numpy().astype(np.float64))
            ms.append(inp["mod"][lo:lo + L].cpu().numpy())
        return np.stack(qs), np.stack(ks), np.stack(vs), np.stack(ms)

    def run(q, k, v, m, start=None):
        t0 = time.perf_counter()
        a_s, a_c = orc.scores_batch(q, k, m, O, 0.0, True)
        dq = np.ones((q.shape[0], D))
        kc, vc, kept = [], [], []
        for p in range(q.shape[0]):
            idx, _ = orc.select(a_s[p], a_c[p], m[p], O, O, T, 0.5)
            kept.append(idx)
            kc.append(orc.gather(k[p], idx)); vc.append(orc.gather(v[p], idx))
        orc.decode_batch(dq, np.stack(kc), np.stack(vc), 1.0)
        dt = time.perf_counter() - t0
        if start is not None:   # (not part of the oracle's time)
            for p in range(q.shape[0]):
                b, h = divmod(start + p, H)
                b %= cfg["B"]
                lo = inp["cu"][b]
                n = int(gpu_cnt[b, h, 0])
                ok = _same_result(a_s[p], a_c[p], kept[p], m[p], gpu_self[h, lo:lo + L], gpu_cross[h, lo:lo + L],
                                  gpu_idx[b, h, :n], L, O)
                checked["n"] += 1
                checked["bad"] += 0 if ok else 1
        return dt

    # batches of 4 problems per thread (different heads each time) until the time target is met
    per_batch, n, t1, start = 4 * threads, 0, 0.0, 0
    while t1 < target_s and n < 256 * threads:
        q, k, v, m = fetch_range(start, per_batch)
        t1 += run(q, k, v, m, start)
        n += per_batch
        start += per_batch
    seq_layers = n / H                             # one (layer, sequence) needs all H heads
    # the same code on one thread, on two problems
    orc.set_threads(1)
    q, k, v, m = fetch_range(0, 2)
    t_one = run(q, k, v, m)
    orc.set_threads(threads)
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return dict(value=seq_layers * L / t1, unit="tokens/s", cores=threads, kind="oracle", cpu_model=model,
                one_thread_value=(2 / H) * L / t_one,
                parity_checked=checked["n"], mismatches=checked["bad"],
                sample=f"{n} (sequence, head) problems of layer 0 at L={L}: score+select+gather and one decode step each, "
                       f"{t1:.1f} s of wall time on {threads} OpenMP threads, scaled linearly (heads are independent)")


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2412_04652_amd as pkg
    pkg.load_library()                              # no fallback: the HIP library must be there
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    device = torch.device("cuda:0")
    cfg = WORKLOADS[args.workload]
    n_layers = args.layers or cfg["layers"]
    decode_steps = cfg["steps"] if args.decode_steps < 0 else args.decode_steps
    inputs = build_inputs(cfg, n_layers, device)
    torch.cuda.synchronize()
    main_res = measure(cfg, inputs, args.budget, decode_steps, args.steps, args.warmup, device, args.streams,
                       args.sel_group)
    second = head_avg = None
    if not args.no_second_budget and args.workload == "7b_16k":
        second = measure(cfg, inputs, 0.2 if abs(args.budget - 0.5) < 1e-9 else 0.5, decode_steps, 2, 1, device, args.streams,
                         args.sel_group)
    if not args.no_head_averaged and args.workload == "7b_16k" and args.sel_group == 1:
        # the paper-literal head axis: scores summed over all heads, one index set per layer and sequence
        head_avg = measure(cfg, inputs, args.budget, 0, 1, 1, device, args.streams, cfg["H"])
    variants = None
    if not args.no_variants and args.workload == "7b_16k" and args.sel_group == 1:
        # same shapes, 8 layers, pruning phase only
        keys = ("budget", "T", "prune_ms", "tokens_per_s", "prune_gbps", "kept_mean")
        variants = {}
        sub = inputs[:8]
        r = measure(cfg, sub, args.budget, 0, 2, 1, device, args.streams, n_score=1.0)
        variants["n_score_1"] = {k: r[k] for k in keys}
        for ratio in (0.0, 0.25, 0.75, 1.0):
            r = measure(cfg, sub, args.budget, 0, 2, 1, device, args.streams, cross_ratio=ratio)
            variants[f"cross_ratio_{ratio:g}"] = {k: r[k] for k in keys}
        # the window rows' normalisers supplied by the caller (csp_score_lse): the keys are read once
        r = measure(cfg, with_row_lse(cfg, sub), args.budget, 0, 2, 1, device, args.streams)
        variants["row_lse_supplied"] = {k: r[k] for k in keys}
        variants["row_lse_supplied"]["kernels"] = r["kernels"]
        mixed = build_inputs(cfg, 8, device, window_text=16)
        r = measure(cfg, mixed, args.budget, 0, 2, 1, device, args.streams)
        variants["mixed_window_48v_16t"] = {k: r[k] for k in keys}
        variants["mixed_window_48v_16t"]["kernels"] = r["kernels"]
        del mixed
        torch.cuda.empty_cache()
    reprune = None
    if not args.no_variants and args.workload == "7b_16k" and args.sel_group == 1:
        reprune = measure_reprune(cfg, inputs[:8], args.budget, cfg["O"], 2, device)
    others = None
    if not args.no_other_configs and args.workload == "7b_16k":
        del inputs[8:]                              # (the passes below need the first layers only)
        torch.cuda.empty_cache()
        others = {name: measure_config(name, c, device) for name, c in OTHER_CONFIGS.items()}
    peak_copy = copy_peak(device)
    peaks = stream_peaks(device)
    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg, inputs, args.budget, args.cpu_seconds, device)

    # dominant kernel of the step by time
    kern = main_res["kernels"]
    step_share = {k: v["ms"] * (n_layers * (decode_steps if k.startswith("decode") else 1)) for k, v in kern.items()}
    dom = max(step_share, key=step_share.get)
    # measured HBM traffic per launch of that kernel (rocprofv3 --pmc, see profiles/), if recorded
    # (a stored figure: `traffic_commit` names the commit of the library it was measured on)
    traffic, traffic_commit = None, None
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            stored = json.load(f)
        rec = stored.get(f"{args.workload}@{args.budget:g}", {}).get(dom.split("(")[0])
        if rec:
            traffic = rec["fetch_bytes"] + rec["write_bytes"]
            traffic_commit = stored.get("commit")
    except (OSError, ValueError, KeyError):
        traffic = None
    roof = dict(bound="hbm", kernel=dom, achieved=kern[dom]["gbps"], peak=HBM_PEAK_GBPS, unit="GB/s",
                frac=kern[dom]["gbps"] / HBM_PEAK_GBPS, traffic=traffic, traffic_commit=traffic_commit,
                algorithmic_bytes_per_launch=kern[dom]["bytes"], avg_launch_ms=kern[dom]["ms"])
    out = {
        "metric": "pruned KV tokens/sec (score+select+compact) and decode attn HBM GB/s, 1 GPU",
        "value": main_res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {n_layers} layers x B{cfg['B']} x H{cfg['H']} x L{cfg['L']} x D{cfg['D']} bf16, "
                               f"window {cfg['O']}, budget {args.budget:g}, {decode_steps} decode steps",
                   "budget": args.budget, "layers": n_layers, "decode_steps": decode_steps, "sel_group": args.sel_group,
                   "prune_streams": args.streams},
        "prune_ms_all_layers": main_res["prune_ms"],
        "prune_hbm_gbps": main_res["prune_gbps"], "prune_frac_of_peak": main_res["prune_gbps"] / HBM_PEAK_GBPS,
        "decode_attn_hbm_gbps": main_res.get("decode_gbps"),
        "decode_frac_of_peak": (main_res.get("decode_gbps") or 0.0) / HBM_PEAK_GBPS,
        "decode_ms_per_token_all_layers": main_res.get("decode_ms_per_token"),
        "step_hbm_gbps": main_res.get("step_gbps"),
        "step_frac_of_peak": (main_res.get("step_gbps") or 0.0) / HBM_PEAK_GBPS,
        "copy_peak_gbps": peak_copy,
        "read_peak_gbps": peaks["read"], "copy_probe_gbps": peaks["copy"],
        "score_frac_of_read_peak": kern["score"]["gbps"] / peaks["read"],
        "score_fallbacks": main_res["score_fallbacks"],
        "prune_frac_of_copy_peak": main_res["prune_gbps"] / peak_copy,
        "decode_frac_of_copy_peak": (main_res.get("decode_gbps") or 0.0) / peak_copy,
        "head_tokens_per_s": main_res["tokens_per_s"] * cfg["H"],
        "kernels": kern,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    if second is not None:
        out["second_budget"] = {k: second[k] for k in ("budget", "T", "prune_ms", "tokens_per_s", "prune_gbps",
                                                       "decode_gbps", "decode_ms_per_token", "score_fallbacks") if k in second}
        out["second_budget"]["kernels"] = second["kernels"]
    if variants is not None:
        out["variants_8_layers"] = variants
    if reprune is not None:
        out["reprune_while_decoding_8_layers"] = reprune
    if others is not None:
        out["other_configs"] = others
    if head_avg is not None:
        out["head_averaged"] = {k: head_avg[k] for k in ("budget", "T", "sel_group", "prune_ms", "tokens_per_s", "prune_gbps")}
        out["head_averaged"]["kernels"] = head_avg["kernels"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
