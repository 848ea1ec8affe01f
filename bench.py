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


def copy_peak(device):
    """Plain device-to-device copy of 2 GiB: the achievable stream bandwidth on this machine."""
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


def cpu_baseline(cfg, inputs, budget_frac, target_s):
    """The CPU oracle, as it stands, on a bounded sample of (sequence, head) problems of layer 0:
    score -> select -> gather -> one decode step each."""
    import numpy as np
    from oracle import csp_oracle as orc
    L, O, D, H = cfg["L"], cfg["O"], cfg["D"], cfg["H"]
    T = int(L * budget_frac)
    inp = inputs[0]
    threads = orc.max_threads()

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

    def run(q, k, v, m):
        t0 = time.perf_counter()
        a_s, a_c = orc.scores_batch(q, k, m, O, 0.0, True)
        dq = np.ones((q.shape[0], D))
        kc, vc = [], []
        for p in range(q.shape[0]):
            idx, _ = orc.select(a_s[p], a_c[p], m[p], O, O, T, 0.5)
            kc.append(orc.gather(k[p], idx)); vc.append(orc.gather(v[p], idx))
        orc.decode_batch(dq, np.stack(kc), np.stack(vc), 1.0)
        return time.perf_counter() - t0

    # batches of 4 problems per thread (different heads each time) until the time target is met
    per_batch, n, t1, start = 4 * threads, 0, 0.0, 0
    while t1 < target_s and n < 256 * threads:
        q, k, v, m = fetch_range(start, per_batch)
        t1 += run(q, k, v, m)
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
    peak_copy = copy_peak(device)
    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg, inputs, args.budget, args.cpu_seconds)

    # dominant kernel of the step by time
    kern = main_res["kernels"]
    step_share = {k: v["ms"] * (n_layers * (decode_steps if k.startswith("decode") else 1)) for k, v in kern.items()}
    dom = max(step_share, key=step_share.get)
    # measured HBM traffic per launch of that kernel (rocprofv3 --pmc, see profiles/), if recorded
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            rec = json.load(f).get(f"{args.workload}@{args.budget:g}", {}).get(dom.split("(")[0])
        if rec:
            traffic = rec["fetch_bytes"] + rec["write_bytes"]
    except (OSError, ValueError, KeyError):
        traffic = None
    roof = dict(bound="hbm", kernel=dom, achieved=kern[dom]["gbps"], peak=HBM_PEAK_GBPS, unit="GB/s",
                frac=kern[dom]["gbps"] / HBM_PEAK_GBPS, traffic=traffic,
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
        "prune_frac_of_copy_peak": main_res["prune_gbps"] / peak_copy,
        "decode_frac_of_copy_peak": (main_res.get("decode_gbps") or 0.0) / peak_copy,
        "head_tokens_per_s": main_res["tokens_per_s"] * cfg["H"],
        "kernels": kern,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    if second is not None:
        out["second_budget"] = {k: second[k] for k in ("budget", "T", "prune_ms", "tokens_per_s", "prune_gbps",
                                                       "decode_gbps", "decode_ms_per_token") if k in second}
        out["second_budget"]["kernels"] = second["kernels"]
    if variants is not None:
        out["variants_8_layers"] = variants
    if reprune is not None:
        out["reprune_while_decoding_8_layers"] = reprune
    if head_avg is not None:
        out["head_averaged"] = {k: head_avg[k] for k in ("budget", "T", "sel_group", "prune_ms", "tokens_per_s", "prune_gbps")}
        out["head_averaged"]["kernels"] = head_avg["kernels"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
