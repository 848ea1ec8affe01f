"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times (same descriptor, same grids): inputs are drawn on
the device with the workload recipe, the rows of a sample of (sequence, head)
problems are copied back, and the oracle checks those problems one by one."""
import numpy as np
import pytest

import csp_workloads as W

pytestmark = pytest.mark.gpu

torch = None  # imported by the `gpu` fixture: runs that select no GPU test never load it


@pytest.fixture(scope="module")
def gpu():
    global torch
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2412_04652_amd as P
    P.load_library()
    return torch.device("cuda:0")


def _bits(t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _oracle_scores(oracle, q, k, mod_h, cu, sample, R, n_score, G, sel_group, chunk=16):
    """Oracle scores of the sampled (sequence, selection group) problems, summed over the group's query
    heads: the heads are independent problems, handed to the oracle's threaded batch entry in chunks
    of equal length."""
    probs = [(b, s, hq) for b, s in sample for hq in range(s * sel_group, (s + 1) * sel_group)]
    by_len = {}
    for pr in probs:
        by_len.setdefault(int(cu[pr[0] + 1]) - int(cu[pr[0]]), []).append(pr)
    out = {}
    for L, group in by_len.items():
        for i in range(0, len(group), chunk):
            part = group[i:i + chunk]
            qs = np.stack([oracle.bf16_bits_to_f64(_bits(q[b, hq])) for b, s, hq in part])
            ks = np.stack([oracle.bf16_bits_to_f64(_bits(k[hq // G, int(cu[b]):int(cu[b + 1])])) for b, s, hq in part])
            ms = np.stack([mod_h[int(cu[b]):int(cu[b + 1])] for b, s, hq in part])
            a_s, a_c = oracle.scores_batch(qs, ks, ms, R, n_score, True)
            for j, (b, s, hq) in enumerate(part):   # (summed in head order, like a loop over the heads)
                acc = out.setdefault((b, s), [np.zeros(L), np.zeros(L)])
                acc[0] += a_s[j]
                acc[1] += a_c[j]
    return out


def _sample_of(n_seq, n_sel, n, seed):
    """n distinct (sequence, selection group) pairs (all of them if there are no more), seeded."""
    pairs = [(b, s) for b in range(n_seq) for s in range(n_sel)]
    if len(pairs) <= n:
        return pairs
    pick = np.random.default_rng(seed).choice(len(pairs), size=n, replace=False)
    return [pairs[i] for i in sorted(pick.tolist())]


def _check_sample(oracle, U, lay, q, k, v, mod, cu, sample, *, O, R, T_of, G, sel_group, dec, what,
                  n_score=0.0, cross_ratio=0.5, fixed_count=True):
    """sample: list of (b, s).  dec: (dq, dk, dv) device tensors of one decode step (appended, then attended)."""
    g_self, g_cross = lay.score_self, lay.score_cross
    idx_all, cnt_all = lay.kept_idx.cpu().numpy(), lay.kept_cnt.cpu().numpy()
    kv_per_sel = sel_group // G
    mod_h = mod.cpu().numpy()
    out = lay.out.cpu().numpy()
    n_diff = 0
    ref_scores = _oracle_scores(oracle, q, k, mod_h, cu, sample, R, n_score, G, sel_group)
    for b, s in sample:
        lo, hi = int(cu[b]), int(cu[b + 1])
        L, T = hi - lo, T_of(b)
        m = mod_h[lo:hi]
        a_s, a_c = ref_scores[(b, s)]
        P = L - R
        U.assert_scores_close(g_self[s, lo:lo + P].cpu().numpy(), a_s[:P], f"{what} b{b} s{s} self")
        U.assert_scores_close(g_cross[s, lo:lo + P].cpu().numpy(), a_c[:P], f"{what} b{b} s{s} cross")
        ref_idx, rc = oracle.select(a_s, a_c, m, O, R, T, cross_ratio)
        n = int(cnt_all[b, s, 0])
        if fixed_count:
            assert n == rc["kept"] == min(T, L)
        else:  # overlapping top-K sets: the count depends on keys near the thresholds
            assert abs(n - rc["kept"]) <= 8 and n <= min(T, L)
        assert cnt_all[b, s, 1:3].tolist() == [rc["K_s"], rc["K_c"]]
        if fixed_count:
            n_diff += U.assert_kept_equivalent(idx_all[b, s, :n], ref_idx, a_s, a_c, m, L, R, f"{what} b{b} s{s}")
        else:
            n_diff += U.assert_kept_equivalent_mixed(idx_all[b, s, :n], ref_idx, a_s, a_c, rc["K_s"], rc["K_c"], L, R,
                                                     f"{what} b{b} s{s}")
        gi = idx_all[b, s, :n]
        for hk in range(s * kv_per_sel, (s + 1) * kv_per_sel):
            kh, vh = _bits(k[hk, lo:hi]), _bits(v[hk, lo:hi])
            np.testing.assert_array_equal(_bits(lay.k_cache[b, hk, :n]), oracle.gather(kh, gi))
            np.testing.assert_array_equal(_bits(lay.v_cache[b, hk, :n]), oracle.gather(vh, gi))
            # decode step over the GPU's own pruned cache + the appended token
            keys = np.concatenate([kh[gi], _bits(dec[1][b, hk])[None]])
            vals = np.concatenate([vh[gi], _bits(dec[2][b, hk])[None]])
            for hq in range(hk * G, (hk + 1) * G):
                ref = oracle.decode(oracle.bf16_bits_to_f64(_bits(dec[0][b, hq])), oracle.bf16_bits_to_f64(keys),
                                    oracle.bf16_bits_to_f64(vals), 1.0)
                U.assert_decode_close(out[b, hq], ref, f"{what} decode b{b} h{hq}")
    return n_diff


def _run(gpu, layouts, *, H_q, H_kv, D, O, budgets, sel_group, seed, heavy=0.0, n_score=0.0, cross_ratio=0.5):
    from paper_2412_04652_amd.runner import CspLayer
    q, k, v, mod, cu_dev, cu = W.device_qkv(layouts, H_q=H_q, H_kv=H_kv, D=D, O=O, seed=seed, device=gpu,
                                            heavy_visual_frac=heavy)
    lay = CspLayer(dtype="bf16", H_q=H_q, H_kv=H_kv, D=D, O=O, R=O, cu_seqlens=cu.tolist(), budgets=budgets,
                   sel_group=sel_group, decode_cap=1, device=gpu, n_score=n_score, cross_ratio=cross_ratio)
    g = torch.Generator(device=gpu); g.manual_seed(seed + 99)
    B = len(layouts)
    dq = torch.randn((B, H_q, D), generator=g, device=gpu).to(torch.bfloat16)
    dk = torch.randn((B, H_kv, D), generator=g, device=gpu).to(torch.bfloat16)
    dv = torch.randn((B, H_kv, D), generator=g, device=gpu).to(torch.bfloat16)
    lay.prune(q, k, v, mod)
    lay.append(dk, dv)
    lay.decode(dq)
    torch.cuda.synchronize()
    return lay, q, k, v, mod, cu, (dq, dk, dv)


@pytest.mark.parametrize("budget", [0.5, 0.2])
def test_7b_16k_layer_sampled(gpu, oracle, budget):
    """One layer of the benchmark workload: B=4, 32 heads, L=16384, D=128, window 64."""
    import gpu_util as U
    rng = np.random.default_rng(1000)
    layouts = [W.layout_7b_16k(rng) for _ in range(4)]
    T = int(16384 * budget)
    print(f"[full] 7b_16k budget={budget} T={T}", flush=True)
    lay, q, k, v, mod, cu, dec = _run(gpu, layouts, H_q=32, H_kv=32, D=128, O=64, budgets=[T] * 4, sel_group=1, seed=0)
    sample = _sample_of(4, 32, 64, seed=int(budget * 100))   # 64 of the layer's 128 (sequence, head) problems
    nd = _check_sample(oracle, U, lay, q, k, v, mod, cu, sample, O=64, R=64, T_of=lambda b: T, G=1, sel_group=1,
                       dec=dec, what=f"7b_16k@{budget}")
    print(f"[full] keys differing near the threshold: {nd}", flush=True)
    assert nd <= 4 * len(sample)
    assert lay.score_fallbacks() == 0
    # properties that hold for every head, checked on all 128 of them
    cnt = lay.kept_cnt.cpu().numpy()
    assert (cnt[:, :, 0] == T).all() and (cnt[:, :, 1] + cnt[:, :, 2] == T - 64).all()
    idx = lay.kept_idx.cpu().numpy()
    assert (np.diff(idx, axis=-1) > 0).all() and (idx[:, :, -64:] == np.arange(16384 - 64, 16384)).all()
    # softmax rows sum to one: the column sums over all ranked keys plus the recent keys' mass = O;
    # so the ranked mass is at most O and, with 64 recent keys of 16384, close to it
    tot = (lay.score_self + lay.score_cross).view(32, 4, 16384).sum(-1).cpu().numpy()
    assert (tot <= 64 * (1 + 1e-3)).all() and (tot > 32).all()


def test_7b_16k_head_averaged_sampled(gpu, oracle):
    """The benchmark workload with the scores summed over all 32 heads (the paper's head axis read
    literally): one index set per sequence, shared by every KV head.  The selection group is cut
    into slices summed by separate workgroups here; the oracle sums the 32 heads of one sequence."""
    import gpu_util as U
    rng = np.random.default_rng(1000)
    layouts = [W.layout_7b_16k(rng) for _ in range(4)]
    T = 8192
    print("[full] 7b_16k head-averaged", flush=True)
    lay, q, k, v, mod, cu, dec = _run(gpu, layouts, H_q=32, H_kv=32, D=128, O=64, budgets=[T] * 4, sel_group=32, seed=0)
    nd = _check_sample(oracle, U, lay, q, k, v, mod, cu, [(2, 0)], O=64, R=64, T_of=lambda b: T, G=1, sel_group=32,
                       dec=dec, what="7b_16k head-averaged")
    print(f"[full] keys differing near the threshold: {nd}", flush=True)
    assert nd <= 4
    cnt = lay.kept_cnt.cpu().numpy()
    assert cnt.shape == (4, 1, 4) and (cnt[:, 0, 0] == T).all()
    tot = (lay.score_self + lay.score_cross).view(4, 16384).sum(-1).cpu().numpy()
    assert (tot <= 32 * 64 * (1 + 1e-3)).all() and (tot > 32 * 32).all()


def test_7b_16k_n_softmax_scoring_ratio_quarter(gpu, oracle):
    """The benchmark workload scored with the n-softmax (n = 1) as the select function and a quarter
    of the selected keys taken from the cross region."""
    import gpu_util as U
    rng = np.random.default_rng(1000)
    layouts = [W.layout_7b_16k(rng) for _ in range(4)]
    T = 8192
    print("[full] 7b_16k n_score=1 cross_ratio=0.25", flush=True)
    lay, q, k, v, mod, cu, dec = _run(gpu, layouts, H_q=32, H_kv=32, D=128, O=64, budgets=[T] * 4, sel_group=1, seed=0,
                                      n_score=1.0, cross_ratio=0.25)
    nd = _check_sample(oracle, U, lay, q, k, v, mod, cu, [(0, 3), (3, 28)], O=64, R=64, T_of=lambda b: T, G=1,
                       sel_group=1, dec=dec, what="7b_16k n=1 ratio .25", n_score=1.0, cross_ratio=0.25)
    assert nd <= 8
    cnt = lay.kept_cnt.cpu().numpy()
    # the self region (text keys) has 4864 - 64 = 4800 candidates, fewer than its share of
    # 8128 - 2032 = 6096: the excess goes to the cross region
    assert (cnt[:, :, 0] == T).all() and (cnt[:, :, 1] == 4800).all() and (cnt[:, :, 2] == 3328).all()
    # n in the denominator: every window row sums to less than one
    tot = (lay.score_self + lay.score_cross).view(32, 4, 16384).sum(-1).cpu().numpy()
    assert (tot < 64).all()


def test_7b_16k_mixed_window_sampled(gpu, oracle):
    """The benchmark shape with sequences that end in an image and 16 text tokens: the window holds
    48 visual and 16 text queries, all four blocks are non-empty, both regions rank every prefix
    key, the two top-K sets overlap and fewer than T keys are kept."""
    import gpu_util as U
    rng = np.random.default_rng(1000)
    layouts = [W.layout_mixed_window(rng, [576] * 20, 4864, 16) for _ in range(4)]
    T = 8192
    print("[full] 7b_16k mixed window", flush=True)
    lay, q, k, v, mod, cu, dec = _run(gpu, layouts, H_q=32, H_kv=32, D=128, O=64, budgets=[T] * 4, sel_group=1, seed=0)
    nd = _check_sample(oracle, U, lay, q, k, v, mod, cu, [(0, 9), (2, 17)], O=64, R=64, T_of=lambda b: T, G=1,
                       sel_group=1, dec=dec, what="7b_16k mixed", fixed_count=False)
    print(f"[full] mixed window: keys differing near the thresholds: {nd}", flush=True)
    assert nd <= 16
    cnt = lay.kept_cnt.cpu().numpy()
    # kept = K_s + K_c - both + R, strictly below T because the sets overlap
    np.testing.assert_array_equal(cnt[:, :, 0], cnt[:, :, 1] + cnt[:, :, 2] - cnt[:, :, 3] + 64)
    assert (cnt[:, :, 3] > 0).all() and (cnt[:, :, 0] < T).all()
    np.testing.assert_array_equal(lay.kv_len.cpu().numpy(), cnt[:, :, 0] + 1)


def test_64k_stress_sampled(gpu, oracle):
    """B=1, 32 heads, L=65536, window 128, budget 10 %, 1 % of the visual keys scaled x4."""
    import gpu_util as U
    rng = np.random.default_rng(5)
    layouts = [W.layout_64k(rng)]
    T = 6553
    print("[full] 64k stress", flush=True)
    for seed in (3, 4):   # two layers, all 32 heads of each: 64 problems
        lay, q, k, v, mod, cu, dec = _run(gpu, layouts, H_q=32, H_kv=32, D=128, O=128, budgets=[T], sel_group=1, seed=seed,
                                          heavy=0.01)
        nd = _check_sample(oracle, U, lay, q, k, v, mod, cu, _sample_of(1, 32, 32, 0), O=128, R=128, T_of=lambda b: T, G=1,
                           sel_group=1, dec=dec, what=f"64k seed {seed}")
        print(f"[full] 64k seed {seed}: keys differing near the threshold: {nd}", flush=True)
        cnt = lay.kept_cnt.cpu().numpy()
        assert (cnt[0, :, 0] == T).all() and (cnt[0, :, 1] == 3213).all() and (cnt[0, :, 2] == 3212).all()
        assert lay.score_fallbacks() == 0
        del lay, q, k, v


def test_gqa_ragged_full_sampled(gpu, oracle):
    """B=8 ragged sequences up to 8192 tokens, 28 query heads on 4 KV heads, one index set per KV head."""
    import gpu_util as U
    rng = np.random.default_rng(1000)
    layouts = [W.layout_gqa_ragged(rng, 8192) for _ in range(8)]
    lens = [sum(n for _, n in s) for s in layouts]
    budgets = [l // 2 for l in lens]
    print(f"[full] gqa ragged lens={lens}", flush=True)
    for seed in (11, 12):   # two layers, all 8 x 4 (sequence, KV head) problems of each: 64 problems, 448 heads
        lay, q, k, v, mod, cu, dec = _run(gpu, layouts, H_q=28, H_kv=4, D=128, O=64, budgets=budgets, sel_group=7, seed=seed)
        _check_sample(oracle, U, lay, q, k, v, mod, cu, _sample_of(8, 4, 32, 0), O=64, R=64, T_of=lambda b: budgets[b], G=7,
                      sel_group=7, dec=dec, what=f"gqa seed {seed}")
        cnt = lay.kept_cnt.cpu().numpy()
        for b in range(8):
            assert (cnt[b, :, 0] == budgets[b]).all()
        np.testing.assert_array_equal(lay.kv_len.cpu().numpy(), np.broadcast_to(np.array(budgets)[:, None] + 1, (8, 4)))
        assert lay.score_fallbacks() == 0


def test_gqa_large_groups_in_slices(gpu, oracle):
    """B=8 sequences of 19k-32k tokens, 64 query heads on 8 KV heads (head_dim 64), one index set per
    KV head: large enough that a group of 8 heads is summed in slices of several heads each (both
    the in-place accumulation over a slice's heads and the ordered sum of the slices run)."""
    import gpu_util as U
    rng = np.random.default_rng(77)
    layouts = [W.layout_random(rng, [576] * int(n_img), 32768 - 576 * 48 + int(extra), 64)
               for n_img, extra in zip(rng.integers(30, 49, size=8), rng.integers(-3000, 1, size=8))]
    layouts[5] = W.layout_random(rng, [576] * 48, 32768 - 576 * 48, 64)   # one sequence at the maximum
    lens = [sum(n for _, n in s) for s in layouts]
    assert max(lens) == 32768
    budgets = [int(l * 0.3) for l in lens]
    print(f"[full] gqa large lens={lens}", flush=True)
    lay, q, k, v, mod, cu, dec = _run(gpu, layouts, H_q=64, H_kv=8, D=64, O=64, budgets=budgets, sel_group=8, seed=21)
    sample = [(5, 0), (1, 7), (6, 3)]
    _check_sample(oracle, U, lay, q, k, v, mod, cu, sample, O=64, R=64, T_of=lambda b: budgets[b], G=8, sel_group=8,
                  dec=dec, what="gqa large")
    cnt = lay.kept_cnt.cpu().numpy()
    for b in range(8):
        assert (cnt[b, :, 0] == budgets[b]).all()


def test_f32_d128_window128_large_chunks(gpu, oracle):
    """fp32 storage, head_dim 128, window 128: the shape whose column-sum pass needs the most LDS (key
    tiles, staged fp32 queries and the chunk's scores); large enough (B=8, 32 heads, L=4096) that the
    chunk size reaches its cap for this shape."""
    import gpu_util as U
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(31)
    layouts = [W.layout_random(rng, [576] * 4, 4096 - 4 * 576, 128) for _ in range(8)]
    q, k, v, mod, cu_dev, cu = W.device_qkv(layouts, H_q=32, H_kv=32, D=128, O=128, seed=5, device=gpu)
    qf, kf = q.float(), k.float()
    lay = CspLayer(dtype="f32", H_q=32, H_kv=32, D=128, O=128, R=128, cu_seqlens=cu.tolist(), budgets=[2048] * 8,
                   device=gpu)
    print("[full] f32 d128 window 128", flush=True)
    lay.score(qf, kf, mod)
    lay.select(mod)
    torch.cuda.synchronize()
    mod_h = mod.cpu().numpy()
    idx, cnt = lay.kept_idx.cpu().numpy(), lay.kept_cnt.cpu().numpy()
    for b, h in [(0, 0), (5, 17), (7, 31)]:
        lo, hi = int(cu[b]), int(cu[b + 1])
        L = hi - lo
        a_s, a_c = oracle.head_scores(qf[b, h].cpu().numpy().astype(np.float64), kf[h, lo:hi].cpu().numpy().astype(np.float64),
                                      mod_h[lo:hi], 128, 0.0, True)
        P = L - 128
        U.assert_scores_close(lay.score_self[h, lo:lo + P].cpu().numpy(), a_s[:P], f"f32 b{b} h{h} self")
        U.assert_scores_close(lay.score_cross[h, lo:lo + P].cpu().numpy(), a_c[:P], f"f32 b{b} h{h} cross")
        ref_idx, rc = oracle.select(a_s, a_c, mod_h[lo:hi], 128, 128, 2048, 0.5)
        n = int(cnt[b, h, 0])
        assert n == rc["kept"] == 2048
        U.assert_kept_equivalent(idx[b, h, :n], ref_idx, a_s, a_c, mod_h[lo:hi], L, 128, f"f32 b{b} h{h}")


def test_7b_16k_two_streams_bit_identical(gpu):
    """Two layers pruned at the same time on two streams (what bench.py does) against the same two
    layers pruned one after the other: scores, kept positions and caches must be bit-identical.
    The single-read score kernel exchanges statistics between workgroups inside a launch; sharing
    the chip with another stream's kernels changes when its workgroups start, which must change
    neither the result nor the path taken (a workgroup whose wait ran out would recompute the
    statistics in another order and differ in the last bit)."""
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(1000)
    layouts = [W.layout_7b_16k(rng) for _ in range(4)]
    T = 8192
    data = []
    for seed in (0, 1):
        q, k, v, mod, cu_dev, cu = W.device_qkv(layouts, H_q=32, H_kv=32, D=128, O=64, seed=seed, device=gpu)
        mk = lambda: CspLayer(dtype="bf16", H_q=32, H_kv=32, D=128, O=64, R=64, cu_seqlens=cu.tolist(),
                              budgets=[T] * 4, sel_group=1, decode_cap=1, device=gpu)
        data.append((q, k, v, mod, mk(), mk()))
    print("[full] two streams vs serial, 2 layers of 7b_16k", flush=True)
    for q, k, v, mod, serial, _ in data:
        serial.prune(q, k, v, mod)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(device=gpu) for _ in range(2)]
    for rep in range(3):
        for st, (q, k, v, mod, _, conc) in zip(streams, data):
            st.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(st):
                conc.prune(q, k, v, mod)
        for st in streams:
            torch.cuda.current_stream().wait_stream(st)
        torch.cuda.synchronize()
        for li, (q, k, v, mod, serial, conc) in enumerate(data):
            assert torch.equal(serial.score_self, conc.score_self) and torch.equal(serial.score_cross, conc.score_cross), (rep, li)
            assert torch.equal(serial.kept_idx, conc.kept_idx) and torch.equal(serial.kept_cnt, conc.kept_cnt), (rep, li)
            assert torch.equal(serial.k_cache[:, :, :T].view(torch.int16), conc.k_cache[:, :, :T].view(torch.int16)), (rep, li)
            assert torch.equal(serial.v_cache[:, :, :T].view(torch.int16), conc.v_cache[:, :, :T].view(torch.int16)), (rep, li)
