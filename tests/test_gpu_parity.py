"""GPU parity: every entry point of the C ABI against the CPU oracle on the same
seeded inputs.  Integer / byte work is compared bit-exactly; floating point to
2e-3 relative (fp32 accumulation of bf16 inputs) with the absolute floors of
tests/gpu_util.py."""
import math

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
    P.load_library()          # fail loudly if the HIP library is not built
    return torch.device("cuda:0")


def _util():
    import gpu_util
    return gpu_util


def _say(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------------------
# csp_score
# ---------------------------------------------------------------------------
def _score_case(name, **kw):
    base = dict(dtype="bf16", H_q=2, H_kv=2, D=128, O=64, R=64, sel_group=1, n_score=0.0, seed=1,
                layouts=[[(0, 100), (1, 300), (0, 90), (1, 211), (0, 130)]], budgets=[300])
    base.update(kw)
    return W.make_case(name, **base)


SCORE_CASES = {
    "bf16_d128_o64": dict(),
    "bf16_d64_o32": dict(D=64, O=32, R=32),
    "f32_d64_o32_tiny_shape": dict(dtype="f32", D=64, O=32, R=32, H_q=3, H_kv=3),
    "f32_d128_o64": dict(dtype="f32"),
    "o8_r3": dict(O=8, R=3),
    "o100_r17": dict(O=100, R=17),
    "o128_r128": dict(O=128, R=128),
    "r_larger_than_o": dict(O=16, R=200),
    "r_zero": dict(O=16, R=0),
    "nscore_1": dict(n_score=1.0),
    "nscore_2p5_f32": dict(n_score=2.5, dtype="f32", D=64),
    "gqa_group4": dict(H_q=8, H_kv=2, sel_group=4),
    "all_heads_one_group": dict(H_q=4, H_kv=2, sel_group=4),
    "ragged_batch": dict(layouts=[[(0, 70), (1, 50), (0, 64)], [(1, 700), (0, 333)], [(0, 64)],
                                  [(0, 10), (1, 2500), (0, 99)]], budgets=[100, 500, 64, 1000]),
    "visual_window": dict(layouts=[[(0, 200), (1, 100), (0, 150), (1, 400)]]),
    "mixed_window": dict(layouts=[[(0, 200), (1, 300), (0, 40), (1, 10), (0, 10), (1, 5)]]),
    "long_multi_chunk": dict(layouts=[[(0, 1000), (1, 5000), (0, 777), (1, 2000), (0, 500)]], H_q=1, H_kv=1),
    # the longest sequence of the single-read kernel: 128 chunks per head, merged in three rounds of 48
    "long_128_chunks": dict(H_q=1, H_kv=1, layouts=[[(0, 1000), (1, 60000), (0, 4536)]], budgets=[4096]),
    # beyond 128 chunks of 512 keys per KV head the single-read kernel hands over to the two passes
    "very_long_takes_two_passes": dict(H_q=2, H_kv=2, layouts=[[(0, 3000), (1, 120000), (0, 772), (1, 8000), (0, 100)]],
                                       budgets=[4096]),
    "ragged_multi_chunk_d64": dict(H_q=3, H_kv=3, D=64, O=32, R=20, n_score=1.0,
                                   layouts=[[(0, 40), (1, 1500), (0, 33)], [(1, 513), (0, 32)], [(0, 32)],
                                            [(0, 3), (1, 1020), (0, 1)]], budgets=[400, 200, 32, 300]),
}


def _check_score(U, oracle, case, name, score_wait_us=0):
    dc = U.DeviceCase(case, score_wait_us=score_wait_us)
    dc.layer.score(dc.q_win, dc.k, dc.modality)
    torch.cuda.synchronize()
    g_self = dc.layer.score_self.cpu().numpy()
    g_cross = dc.layer.score_cross.cpu().numpy()
    for b in range(case.B):
        lo, hi = int(case.cu_seqlens[b]), int(case.cu_seqlens[b + 1])
        L = hi - lo
        for s in range(case.H_q // case.sel_group):
            a_s, a_c = oracle.group_scores(case, b, s)
            P = L - case.R
            U.assert_scores_close(g_self[s, lo:lo + P], a_s[:P], f"{name} b{b} s{s} self")
            U.assert_scores_close(g_cross[s, lo:lo + P], a_c[:P], f"{name} b{b} s{s} cross")
            assert not g_self[s, lo + P:hi].any() and not g_cross[s, lo + P:hi].any()
    return g_self, g_cross, dc.layer.score_fallbacks()


@pytest.mark.parametrize("name", list(SCORE_CASES))
def test_score_matches_oracle(gpu, oracle, name):
    U = _util()
    case = _score_case(name, **SCORE_CASES[name])
    _say(f"[score] case={name} dtype={case.dtype} D={case.D} O={case.O} R={case.R} lens={np.diff(case.cu_seqlens).tolist()}")
    _check_score(U, oracle, case, name)


@pytest.mark.parametrize("name", ["bf16_d128_o64", "bf16_d64_o32", "o8_r3", "o100_r17", "o128_r128", "r_zero", "nscore_1", "ragged_batch",
                                  "visual_window", "mixed_window", "long_multi_chunk", "long_128_chunks", "ragged_multi_chunk_d64",
                                  "gqa_group4", "all_heads_one_group"])
def test_score_single_read_without_waiting(gpu, oracle, name):
    """The single-read kernel with its wait for the other chunks of a head cut short from the host
    (descriptor field score_wait_us).  Never waiting: every task whose statistics are not all there
    at the first look is finished by its workgroup alone, which recomputes the statistics of every
    chunk of the head; 1 us: both paths in one launch.  The scores must not depend on it, bit for bit."""
    U = _util()
    case = _score_case(name, **SCORE_CASES[name])
    _say(f"[score, waits] case={name} dtype={case.dtype} D={case.D} O={case.O} R={case.R}")
    ref_self, ref_cross, n0 = _check_score(U, oracle, case, name)
    assert n0 == 0, f"{n0} tasks gave up with the default wait on an idle GPU"
    for wait in (-1, 1):
        g_self, g_cross, n = _check_score(U, oracle, case, name, score_wait_us=wait)
        _say(f"    wait {wait}: {n} tasks finished alone")
        assert np.array_equal(g_self.view(np.uint32), ref_self.view(np.uint32)), f"{name}: self scores differ with wait {wait}"
        assert np.array_equal(g_cross.view(np.uint32), ref_cross.view(np.uint32)), f"{name}: cross scores differ with wait {wait}"


def _host_row_lse(oracle, case):
    """ln sum_j exp(q_i.k_j / sqrt(D)) over the keys window row i sees: the normaliser a prefill
    attention kernel hands over.  An INPUT of csp_score_lse, computed here in float64."""
    G = case.H_q // case.H_kv
    lse = np.zeros((case.B, case.H_q, case.O), dtype=np.float64)
    for b in range(case.B):
        lo, hi = int(case.cu_seqlens[b]), int(case.cu_seqlens[b + 1])
        L = hi - lo
        for h in range(case.H_q):
            q = oracle.to_f64(case.q_win[b, h], case.dtype)
            k = oracle.to_f64(case.k[h // G, lo:hi], case.dtype)
            S = q @ k.T / np.sqrt(case.D)
            S[np.arange(L)[None, :] > (L - case.O + np.arange(case.O))[:, None]] = -np.inf
            m = S.max(axis=1)
            lse[b, h] = m + np.log(np.exp(S - m[:, None]).sum(axis=1))
    return lse


@pytest.mark.parametrize("name", ["bf16_d128_o64", "f32_d64_o32_tiny_shape", "o100_r17", "nscore_1", "nscore_2p5_f32",
                                  "gqa_group4", "ragged_batch", "mixed_window", "long_multi_chunk"])
def test_score_with_supplied_row_lse(gpu, oracle, name):
    """csp_score_lse: the window rows' log-sum-exp comes from the caller, the keys are read once; the
    scores must match the oracle (which normalises by itself) and csp_score."""
    U = _util()
    case = _score_case(name, **SCORE_CASES[name])
    _say(f"[score_lse] case={name}")
    dc = U.DeviceCase(case)
    lse = torch.from_numpy(_host_row_lse(oracle, case).astype(np.float32)).to(gpu)
    dc.layer.score(dc.q_win, dc.k, dc.modality)
    ref_self, ref_cross = dc.layer.score_self.clone(), dc.layer.score_cross.clone()
    dc.layer.score_self.fill_(-1.0); dc.layer.score_cross.fill_(-1.0)
    dc.layer.ws_score.zero_()          # no statistics left over from csp_score
    dc.layer.score_lse(dc.q_win, dc.k, dc.modality, lse)
    torch.cuda.synchronize()
    g_self, g_cross = dc.layer.score_self.cpu().numpy(), dc.layer.score_cross.cpu().numpy()
    for b in range(case.B):
        lo, hi = int(case.cu_seqlens[b]), int(case.cu_seqlens[b + 1])
        P = hi - lo - case.R
        for s in range(case.H_q // case.sel_group):
            a_s, a_c = oracle.group_scores(case, b, s)
            U.assert_scores_close(g_self[s, lo:lo + P], a_s[:P], f"{name} b{b} s{s} self")
            U.assert_scores_close(g_cross[s, lo:lo + P], a_c[:P], f"{name} b{b} s{s} cross")
            assert not g_self[s, lo + P:hi].any() and not g_cross[s, lo + P:hi].any()
    # against csp_score: the same weights up to the rounding of the normaliser and, where csp_score takes
    # the single-read kernel, of its fp16 copies of the weights (2^-12 each, averaged over the window rows)
    np.testing.assert_allclose(g_self, ref_self.cpu().numpy(), rtol=5e-4, atol=1e-7)
    np.testing.assert_allclose(g_cross, ref_cross.cpu().numpy(), rtol=5e-4, atol=1e-7)


def test_score_noncausal(gpu, oracle):
    U = _util()
    case = _score_case("noncausal", O=32, R=32)
    dc = U.DeviceCase(case)
    from paper_2412_04652_amd.runner import CspLayer
    layer = CspLayer(dtype=case.dtype, H_q=case.H_q, H_kv=case.H_kv, D=case.D, O=case.O, R=case.R,
                     cu_seqlens=case.cu_seqlens.tolist(), budgets=case.budget_T.tolist(), causal=False)
    layer.score(dc.q_win, dc.k, dc.modality)
    torch.cuda.synchronize()
    L = case.seqlen(0)
    for h in range(case.H_q):
        a_s, a_c = oracle.head_scores(oracle.to_f64(case.q_win[0, h], case.dtype), oracle.to_f64(case.k[h], case.dtype),
                                      case.modality, case.R, 0.0, causal=False)
        U.assert_scores_close(layer.score_self[h, : L - case.R].cpu().numpy(), a_s[: L - case.R], "noncausal self")
        U.assert_scores_close(layer.score_cross[h, : L - case.R].cpu().numpy(), a_c[: L - case.R], "noncausal cross")


def test_score_token_major_strides(gpu, oracle):
    """K stored [tokens, H_kv, D] instead of [H_kv, tokens, D]."""
    U = _util()
    case = _score_case("tokmajor", H_q=4, H_kv=4)
    dc = U.DeviceCase(case)
    from paper_2412_04652_amd.runner import CspLayer
    k_tm = dc.k.permute(1, 0, 2).contiguous()
    layer = CspLayer(dtype=case.dtype, H_q=4, H_kv=4, D=case.D, O=case.O, R=case.R,
                     cu_seqlens=case.cu_seqlens.tolist(), budgets=case.budget_T.tolist(),
                     k_strides=(4 * case.D, case.D), v_strides=(4 * case.D, case.D))
    layer.score(dc.q_win, k_tm, dc.modality)
    dc.layer.score(dc.q_win, dc.k, dc.modality)
    torch.cuda.synchronize()
    assert torch.equal(layer.score_self, dc.layer.score_self) and torch.equal(layer.score_cross, dc.layer.score_cross)


# ---------------------------------------------------------------------------
# csp_select: integer work, bit-exact on identical fp32 scores
# ---------------------------------------------------------------------------
def _select_inputs(rng, lens, O, quantise):
    mods, scs, scc = [], [], []
    for L, window in lens:
        m = (rng.random(L) < 0.6).astype(np.uint8)
        if window == "text":
            m[L - O:] = 0
        elif window == "visual":
            m[L - O:] = 1
        else:
            m[L - O:] = rng.integers(0, 2, O)
            m[L - 1], m[L - 2] = 0, 1
        s = rng.random(L).astype(np.float32) ** 4
        c = rng.random(L).astype(np.float32) ** 4
        if quantise:                      # many exact ties
            s = np.round(s * quantise) / np.float32(quantise)
            c = np.round(c * quantise) / np.float32(quantise)
        mods.append(m), scs.append(s.astype(np.float32)), scc.append(c.astype(np.float32))
    return mods, scs, scc


@pytest.mark.parametrize("ratio", [0.0, 0.1, 0.5, 0.9, 1.0])
@pytest.mark.parametrize("quantise", [0, 7, 300])
def test_select_bit_exact(gpu, oracle, ratio, quantise):
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(int(ratio * 10) * 1000 + quantise)
    O, R = 16, 24
    lens = [(1500, "text"), (40, "text"), (5000, "visual"), (3333, "mixed"), (24, "text"), (2048, "text"), (1025, "mixed")]
    budgets = [700, 40, 1200, 2000, 24, 2047, 24]     # identity, T=L-1 and T=R among them
    H_sel = 3
    cu = np.concatenate([[0], np.cumsum([l for l, _ in lens])])
    total = int(cu[-1])
    mods, ss, cc = [], [], []
    for _ in range(H_sel):
        m, s, c = _select_inputs(rng, lens, O, quantise)
        ss.append(np.concatenate(s)), cc.append(np.concatenate(c))
        mods = m if not mods else mods
    # one modality vector for all heads (it is per token)
    mod = np.concatenate(mods)
    _say(f"[select] ratio={ratio} quantise={quantise} lens={[l for l, _ in lens]} budgets={budgets}")
    layer = CspLayer(dtype="bf16", H_q=H_sel, H_kv=H_sel, D=128, O=O, R=R, cu_seqlens=cu.tolist(), budgets=budgets,
                     cross_ratio=ratio)
    d_self = torch.from_numpy(np.stack(ss)).to(gpu)
    d_cross = torch.from_numpy(np.stack(cc)).to(gpu)
    d_mod = torch.from_numpy(mod).to(gpu)
    layer.select(d_mod, score_self=d_self, score_cross=d_cross)
    torch.cuda.synchronize()
    idx = layer.kept_idx.cpu().numpy()
    cnt = layer.kept_cnt.cpu().numpy()
    for b, (L, _) in enumerate(lens):
        lo = int(cu[b])
        for s in range(H_sel):
            ref, rc = oracle.select(ss[s][lo:lo + L], cc[s][lo:lo + L], mod[lo:lo + L], O, R, budgets[b], ratio)
            n = int(cnt[b, s, 0])
            assert n == rc["kept"], (b, s, n, rc)
            np.testing.assert_array_equal(idx[b, s, :n], ref)
            assert (idx[b, s, n:] == -1).all()
            assert cnt[b, s, 1:].tolist() == [rc["K_s"], rc["K_c"], rc["both"]]


@pytest.mark.parametrize("L", [16384, 16385, 24000, 32768, 32769])
def test_select_bit_exact_long(gpu, oracle, L):
    """Lengths around the edges of the kernel instances that keep 16 and 32 keys per thread in
    registers, and just beyond (super-blocks re-read per pass): indices and counts bit for bit, with
    quantised scores so that the thresholds tie."""
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(L)
    O, R, T = 64, 48, L // 3
    lens = [(L, "mixed"), (L - 1000, "text")]
    cu = np.concatenate([[0], np.cumsum([l for l, _ in lens])])
    mods, ss, cc = _select_inputs(rng, lens, O, 500)
    mod = np.concatenate(mods)
    _say(f"[select long] L={L} T={T}")
    layer = CspLayer(dtype="bf16", H_q=1, H_kv=1, D=128, O=O, R=R, cu_seqlens=cu.tolist(), budgets=[T, T], cross_ratio=0.3)
    d_self = torch.from_numpy(np.concatenate(ss)[None]).to(gpu)
    d_cross = torch.from_numpy(np.concatenate(cc)[None]).to(gpu)
    layer.select(torch.from_numpy(mod).to(gpu), score_self=d_self, score_cross=d_cross)
    torch.cuda.synchronize()
    idx = layer.kept_idx.cpu().numpy()
    cnt = layer.kept_cnt.cpu().numpy()
    for b, (Lb, _) in enumerate(lens):
        lo = int(cu[b])
        ref, rc = oracle.select(ss[b], cc[b], mod[lo:lo + Lb], O, R, T, 0.3)
        n = int(cnt[b, 0, 0])
        assert n == rc["kept"], (b, n, rc)
        np.testing.assert_array_equal(idx[b, 0, :n], ref)
        assert (idx[b, 0, n:] == -1).all()
        assert cnt[b, 0, 1:].tolist() == [rc["K_s"], rc["K_c"], rc["both"]]


def test_select_skewed_scores_64k(gpu, oracle):
    """64k keys, scores clustered in a few exponents with a heavy tail (radix skew)."""
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(5)
    L, O, R, T = 65536, 128, 128, 6553
    lay = W.layout_64k(rng)
    mod = W.spans_to_modality(lay)
    s = (1e-5 * (1 + 0.01 * rng.standard_normal(L))).astype(np.float32)
    s[rng.random(L) < 0.01] *= 50
    s = np.abs(s)
    layer = CspLayer(dtype="bf16", H_q=1, H_kv=1, D=128, O=O, R=R, cu_seqlens=[0, L], budgets=[T])
    d = torch.from_numpy(s[None]).to(gpu)
    layer.select(torch.from_numpy(mod).to(gpu), score_self=d, score_cross=d)
    torch.cuda.synchronize()
    ref, rc = oracle.select(s, s, mod, O, R, T, 0.5)
    assert int(layer.kept_cnt[0, 0, 0]) == T == rc["kept"]
    np.testing.assert_array_equal(layer.kept_idx[0, 0].cpu().numpy(), ref)
    assert (rc["K_s"], rc["K_c"]) == (3213, 3212)


# ---------------------------------------------------------------------------
# csp_compact: bit copy
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128)])
def test_compact_bit_exact(gpu, oracle, dtype, D):
    U = _util()
    case = W.make_case("cp", dtype=dtype, H_q=6, H_kv=3, D=D, O=8, R=8, sel_group=2,
                       layouts=[[(0, 300), (1, 900), (0, 77)], [(0, 50)], [(1, 600), (0, 601)]],
                       budgets=[500, 64, 333], seed=9)
    dc = U.DeviceCase(case, decode_cap=4)
    rng = np.random.default_rng(3)
    idx = np.full((case.B, 3, dc.layer.kept_cap), -1, np.int32)
    cnt = np.zeros((case.B, 3, 4), np.int32)
    for b in range(case.B):
        L = case.seqlen(b)
        for s in range(3):
            n = min(L, int(case.budget_T[b])) - (s if L > 10 else 0)     # different counts per group
            idx[b, s, :n] = np.sort(rng.choice(L, n, replace=False))
            cnt[b, s, 0] = n
    dc.layer.kept_idx.copy_(torch.from_numpy(idx))
    dc.layer.kept_cnt.copy_(torch.from_numpy(cnt))
    dc.layer.k_cache.view(torch.uint8).fill_(0xAB)
    dc.layer.v_cache.view(torch.uint8).fill_(0xCD)
    before_k = U.from_dev_bits(dc.layer.k_cache, dtype).copy()
    dc.layer.compact(dc.k, dc.v)
    torch.cuda.synchronize()
    kc = U.from_dev_bits(dc.layer.k_cache, dtype)
    vc = U.from_dev_bits(dc.layer.v_cache, dtype)
    kvl = dc.layer.kv_len.cpu().numpy()
    for b in range(case.B):
        lo = int(case.cu_seqlens[b])
        for h in range(3):
            s = h  # kv_per_sel = sel_group / G = 1
            n = int(cnt[b, s, 0])
            assert kvl[b, h] == n
            np.testing.assert_array_equal(kc[b, h, :n], oracle.gather(case.k[h, lo:lo + case.seqlen(b)], idx[b, s, :n]))
            np.testing.assert_array_equal(vc[b, h, :n], oracle.gather(case.v[h, lo:lo + case.seqlen(b)], idx[b, s, :n]))
            np.testing.assert_array_equal(kc[b, h, n:], before_k[b, h, n:])      # untouched beyond the count


# ---------------------------------------------------------------------------
# csp_decode_attn / csp_append_kv
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,D,H_q,H_kv", [("bf16", 128, 4, 4), ("bf16", 128, 14, 2), ("bf16", 64, 8, 2),
                                               ("f32", 64, 3, 3), ("f32", 128, 4, 1), ("bf16", 128, 24, 2)])
@pytest.mark.parametrize("n", [0.0, 1.0, 2.5])
def test_decode_matches_oracle(gpu, oracle, dtype, D, H_q, H_kv, n):
    U = _util()
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(H_q * 100 + D + int(n * 10))
    lens = [0, 1, 63, 257, 5000, 1024]
    B, cap = len(lens), 5003
    G = H_q // H_kv
    _say(f"[decode] dtype={dtype} D={D} H_q={H_q} H_kv={H_kv} n={n} lens={lens}")
    layer = CspLayer(dtype=dtype, H_q=H_q, H_kv=H_kv, D=D, O=1, R=1, sel_group=G, cu_seqlens=[0] + list(range(1, B + 1)),
                     budgets=[cap] * B, n_decode=n, decode_cap=cap)
    mk = (lambda shape: W.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))) if dtype == "bf16" \
        else (lambda shape: rng.standard_normal(shape, dtype=np.float32))
    kc, vc, q = mk((B, H_kv, layer.cache_cap, D)), mk((B, H_kv, layer.cache_cap, D)), mk((B, H_q, D))
    layer.k_cache.copy_(U.to_dev(kc, dtype))
    layer.v_cache.copy_(U.to_dev(vc, dtype))
    kvl = np.array([[l + (h % 2 if l > 1 else 0) for h in range(H_kv)] for l in lens], np.int32)   # per-head lengths
    layer.kv_len.copy_(torch.from_numpy(kvl))
    out = layer.decode(U.to_dev(q, dtype)).cpu().numpy()
    torch.cuda.synchronize()
    for b in range(B):
        for hq in range(H_q):
            hk = hq // G
            T = int(kvl[b, hk])
            ref = oracle.decode(oracle.to_f64(q[b, hq], dtype), oracle.to_f64(kc[b, hk, :T], dtype),
                                oracle.to_f64(vc[b, hk, :T], dtype), n)
            U.assert_decode_close(out[b, hq], ref, f"decode b{b} h{hq} T{T}")


def test_decode_large_logits_shift_law(gpu, oracle):
    """Logits around +40 and around -40: n must be scaled with the running
    maximum, not added to a max-shifted sum."""
    U = _util()
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(77)
    D, T = 64, 700
    for shift in (40.0, -40.0):
        q = rng.standard_normal((1, 1, D)).astype(np.float32)
        kc = rng.standard_normal((1, 1, T, D)).astype(np.float32) * 0.3
        kc += shift * math.sqrt(D) * q[0, 0] / float(q[0, 0] @ q[0, 0])      # adds `shift` to every logit
        vc = rng.standard_normal((1, 1, T, D)).astype(np.float32)
        layer = CspLayer(dtype="f32", H_q=1, H_kv=1, D=D, O=1, R=1, cu_seqlens=[0, 1], budgets=[T], n_decode=1.0,
                         decode_cap=T - 1)
        layer.k_cache.copy_(torch.from_numpy(kc))
        layer.v_cache.copy_(torch.from_numpy(vc))
        layer.kv_len.fill_(T)
        out = layer.decode(torch.from_numpy(q).to(gpu)).cpu().numpy()
        ref = oracle.decode(q[0, 0], kc[0, 0], vc[0, 0], 1.0)
        U.assert_decode_close(out[0, 0], ref, f"shift {shift}")


def test_append_then_decode(gpu, oracle):
    U = _util()
    case = W.make_case("app", dtype="bf16", H_q=4, H_kv=2, D=128, O=8, R=8, sel_group=2,
                       layouts=[[(0, 64), (1, 128), (0, 40)], [(1, 300), (0, 30)]], budgets=[100, 330], seed=4,
                       decode_steps=3)
    dc = U.DeviceCase(case, decode_cap=2)          # capacity for 2 of the 3 appends
    lay = dc.layer
    lay.prune(dc.q_win, dc.k, dc.v, dc.modality)
    torch.cuda.synchronize()
    base = lay.kv_len.cpu().numpy().copy()
    dk, dv = U.to_dev(case.dec_k, "bf16"), U.to_dev(case.dec_v, "bf16")
    for t in range(3):
        lay.append(dk[t], dv[t])
    torch.cuda.synchronize()
    kvl = lay.kv_len.cpu().numpy()
    cap = lay.cache_cap
    np.testing.assert_array_equal(kvl, np.minimum(base + 3, cap))        # a full slab is left unchanged
    kc = U.from_dev_bits(lay.k_cache, "bf16")
    for b in range(2):
        for h in range(2):
            for t in range(min(3, cap - int(base[b, h]))):
                np.testing.assert_array_equal(kc[b, h, base[b, h] + t], case.dec_k[t, b, h])


@pytest.mark.parametrize("dtype,D,H_q,H_kv", [("bf16", 128, 4, 4), ("bf16", 128, 14, 2), ("f32", 64, 6, 3)])
def test_decode_step_equals_append_then_attend(gpu, oracle, dtype, D, H_q, H_kv):
    """The fused call must leave the same cache and kv_len as csp_append_kv and return what
    csp_decode_attn returns afterwards (and what the oracle says), also when a slab is full."""
    U = _util()
    from paper_2412_04652_amd.runner import CspLayer
    rng = np.random.default_rng(D + H_q)
    lens = [0, 5, 300, 1027, 1030]
    B, G = len(lens), H_q // H_kv
    mk = (lambda shape: W.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))) if dtype == "bf16" \
        else (lambda shape: rng.standard_normal(shape, dtype=np.float32))
    lays = [CspLayer(dtype=dtype, H_q=H_q, H_kv=H_kv, D=D, O=1, R=1, sel_group=G, cu_seqlens=list(range(B + 1)),
                     budgets=[1029] * B, decode_cap=1029) for _ in range(3)]
    cap = lays[0].cache_cap                     # 1030: the last sequence's slabs are full
    kc, vc = mk((B, H_kv, cap, D)), mk((B, H_kv, cap, D))
    for lay in lays:
        lay.k_cache.copy_(U.to_dev(kc, dtype)); lay.v_cache.copy_(U.to_dev(vc, dtype))
        lay.kv_len.copy_(torch.tensor(lens, dtype=torch.int32)[:, None].expand(B, H_kv))
    for step in range(3):
        q, kn, vn = mk((B, H_q, D)), mk((B, H_kv, D)), mk((B, H_kv, D))
        dq, dk, dv = U.to_dev(q, dtype), U.to_dev(kn, dtype), U.to_dev(vn, dtype)
        out_f = lays[0].decode_step(dq, dk, dv).clone()
        lays[1].append(dk, dv)
        out_r = lays[1].decode(dq)
        lays[2].decode_step_phase(1, dq, dk, dv)           # the two launches issued one by one
        out_p = lays[2].decode_step_phase(2, dq, dk, dv)
        torch.cuda.synchronize()
        assert torch.equal(out_p, out_f) and torch.equal(lays[2].kv_len, lays[0].kv_len)
        assert torch.equal(lays[2].k_cache.view(torch.uint8), lays[0].k_cache.view(torch.uint8))
        assert torch.equal(lays[0].kv_len, lays[1].kv_len)
        assert torch.equal(lays[0].k_cache.view(torch.uint8), lays[1].k_cache.view(torch.uint8))
        assert torch.equal(lays[0].v_cache.view(torch.uint8), lays[1].v_cache.view(torch.uint8))
        assert torch.equal(out_f, out_r)         # same kernel, same order of operations
        kvl = lays[0].kv_len.cpu().numpy()
        kch, vch = U.from_dev_bits(lays[0].k_cache, dtype), U.from_dev_bits(lays[0].v_cache, dtype)
        for b in range(B):
            assert kvl[b, 0] == min(lens[b] + step + 1, cap)
            for hq in range(0, H_q, max(1, H_q // 3)):
                hk, T = hq // G, int(kvl[b, hq // G])
                ref = oracle.decode(oracle.to_f64(q[b, hq], dtype), oracle.to_f64(kch[b, hk, :T], dtype),
                                    oracle.to_f64(vch[b, hk, :T], dtype), 1.0)
                U.assert_decode_close(out_f[b, hq].cpu().numpy(), ref, f"decode_step step{step} b{b} h{hq}")


# ---------------------------------------------------------------------------
# end to end: score -> select -> compact -> append/decode
# ---------------------------------------------------------------------------
def _end_to_end(U, oracle, case, heads_to_check, decode_steps):
    dc = U.DeviceCase(case, decode_cap=decode_steps)
    lay = dc.layer
    lay.prune(dc.q_win, dc.k, dc.v, dc.modality)
    torch.cuda.synchronize()
    g_self, g_cross = lay.score_self.cpu().numpy(), lay.score_cross.cpu().numpy()
    idx, cnt = lay.kept_idx.cpu().numpy(), lay.kept_cnt.cpu().numpy()
    kc, vc = U.from_dev_bits(lay.k_cache, case.dtype), U.from_dev_bits(lay.v_cache, case.dtype)
    G = case.H_q // case.H_kv
    kv_per_sel = case.sel_group // G
    n_diff = 0
    refs = {}
    for b, s in heads_to_check:
        lo, hi = int(case.cu_seqlens[b]), int(case.cu_seqlens[b + 1])
        L, T = hi - lo, int(case.budget_T[b])
        res = oracle.prune_group(case, b, s)
        n = int(cnt[b, s, 0])
        assert n == res["counts"]["kept"] == min(T, L)
        if L > T:
            P = L - case.R
            U.assert_scores_close(g_self[s, lo:lo + P], res["a_self"][:P], f"{case.name} b{b} s{s} self")
            U.assert_scores_close(g_cross[s, lo:lo + P], res["a_cross"][:P], f"{case.name} b{b} s{s} cross")
            assert cnt[b, s, 1:3].tolist() == [res["counts"]["K_s"], res["counts"]["K_c"]]
        n_diff += U.assert_kept_equivalent(idx[b, s, :n], res["idx"], res["a_self"], res["a_cross"],
                                           case.modality[lo:hi], L, case.R if L > T else 0, f"{case.name} b{b} s{s}")
        # gathered rows: bit-exact given the GPU's own indices
        for hk in range(s * kv_per_sel, (s + 1) * kv_per_sel):
            np.testing.assert_array_equal(kc[b, hk, :n], oracle.gather(case.k[hk, lo:hi], idx[b, s, :n]))
            np.testing.assert_array_equal(vc[b, hk, :n], oracle.gather(case.v[hk, lo:hi], idx[b, s, :n]))
        refs[(b, s)] = idx[b, s, :n].copy()
    # decode loop over the pruned cache the GPU built (append, then attend)
    dq = U.to_dev(case.dec_q, case.dtype)
    dk, dv = U.to_dev(case.dec_k, case.dtype), U.to_dev(case.dec_v, case.dtype)
    for t in range(decode_steps):
        if t % 2:                      # alternate the fused and the two-call form
            out = lay.decode_step(dq[t], dk[t], dv[t]).cpu().numpy()
        else:
            lay.append(dk[t], dv[t])
            out = lay.decode(dq[t]).cpu().numpy()
        for b, s in heads_to_check:
            lo, hi = int(case.cu_seqlens[b]), int(case.cu_seqlens[b + 1])
            for hq in range(s * case.sel_group, (s + 1) * case.sel_group):
                hk = hq // G
                keys = np.concatenate([case.k[hk, lo:hi][refs[(b, s)]], case.dec_k[: t + 1, b, hk]])
                vals = np.concatenate([case.v[hk, lo:hi][refs[(b, s)]], case.dec_v[: t + 1, b, hk]])
                ref = oracle.decode(oracle.to_f64(case.dec_q[t, b, hq], case.dtype), oracle.to_f64(keys, case.dtype),
                                    oracle.to_f64(vals, case.dtype), case.n_decode)
                U.assert_decode_close(out[b, hq], ref, f"{case.name} step{t} b{b} h{hq}")
    return n_diff


def test_end_to_end_tiny_config(gpu, oracle):
    U = _util()
    case = W.case_tiny(0)
    _say("[e2e] tiny config, all 8 heads, 4 decode steps")
    _end_to_end(U, oracle, case, [(0, h) for h in range(8)], 4)


def test_end_to_end_7b_4k_config(gpu, oracle):
    U = _util()
    case = W.case_7b_4k(0, decode_steps=16)
    _say("[e2e] 7B 4k config, all 32 heads, 16 decode steps")
    nd = _end_to_end(U, oracle, case, [(0, h) for h in range(32)], 16)
    _say(f"[e2e] 7b_4k keys differing near the threshold: {nd}")
    assert nd <= 32          # a handful of near-threshold swaps at most


def test_end_to_end_gqa_ragged(gpu, oracle):
    U = _util()
    case = W.case_gqa_ragged(0, B=3, decode_steps=2, max_len=4096)
    _say(f"[e2e] GQA ragged lens={np.diff(case.cu_seqlens).tolist()}")
    _end_to_end(U, oracle, case, [(b, s) for b in range(3) for s in (0, 3)], 2)


def test_end_to_end_mixed_window_counts(gpu, oracle):
    """A window with both modalities: both regions cover every prefix key, the
    masks overlap and the kept count is data dependent."""
    U = _util()
    case = W.make_case("mixed", dtype="bf16", H_q=2, H_kv=2, D=128, O=32, R=32,
                       layouts=[[(0, 300), (1, 600), (0, 20), (1, 12), (0, 4), (1, 4)]], budgets=[400], seed=6)
    dc = U.DeviceCase(case)
    dc.layer.prune(dc.q_win, dc.k, dc.v, dc.modality)
    torch.cuda.synchronize()
    cnt = dc.layer.kept_cnt.cpu().numpy()
    for h in range(2):
        res = oracle.prune_group(case, 0, h)
        assert cnt[0, h, 1:3].tolist() == [res["counts"]["K_s"], res["counts"]["K_c"]] == [184, 184]
        assert int(cnt[0, h, 0]) == 400 - int(cnt[0, h, 3])
        n = int(cnt[0, h, 0])
        idx = dc.layer.kept_idx[0, h].cpu().numpy()
        assert (idx[n:] == -1).all()
        # the kept set is the union of the two top-K sets: a key kept by one side only must score within the
        # tolerance of one of the two thresholds (so the count may differ from the oracle's by such keys only)
        a_s, a_c = oracle.group_scores(case, 0, h)
        U.assert_kept_equivalent_mixed(idx[:n], res["idx"], a_s, a_c, 184, 184, 940, 32, f"mixed window h{h}")
        assert int(dc.layer.kv_len[0, h]) == n


EDGE_CASES = {
    # name: make_case keyword overrides (base: bf16, 2 heads, D=128, O=R=8)
    "len_9": dict(layouts=[[(1, 3), (0, 6)]], budgets=[6], O=4, R=2),
    "len_32_exact_tile": dict(layouts=[[(0, 10), (1, 14), (0, 8)]], budgets=[20]),
    "len_33_one_past_a_tile": dict(layouts=[[(0, 10), (1, 15), (0, 8)]], budgets=[20]),
    "one_head": dict(H_q=1, H_kv=1, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[100]),
    "d64_window_128": dict(D=64, O=128, R=128, layouts=[[(0, 100), (1, 500), (0, 200)]], budgets=[400]),
    "f32_d128": dict(dtype="f32", layouts=[[(0, 90), (1, 200), (0, 43)]], budgets=[150]),
    "only_recent_kept": dict(layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[8]),
    "all_cross": dict(cross_ratio=1.0, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[108]),
    "all_self": dict(cross_ratio=0.0, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[108]),
    "ratio_0p9": dict(cross_ratio=0.9, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[108]),
    "text_spills_into_visual": dict(layouts=[[(0, 5), (1, 400), (0, 12)]], budgets=[300]),
    "visual_spills_into_text": dict(layouts=[[(0, 300), (1, 7), (0, 100)]], budgets=[300]),
    "no_visual_tokens": dict(layouts=[[(0, 300)]], budgets=[100]),
    "n_score_1": dict(n_score=1.0, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[100]),
    "one_index_set_per_layer": dict(H_q=4, H_kv=4, sel_group=4, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[100]),
    "identity_and_pruned_in_one_batch": dict(layouts=[[(0, 40), (1, 50), (0, 20)], [(0, 200), (1, 300), (0, 50)], [(0, 64)],
                                                      [(1, 90), (0, 38)]], budgets=[110, 200, 100, 128]),
    "n_decode_0": dict(n_decode=0.0, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[100]),
    "n_decode_3": dict(n_decode=3.0, layouts=[[(0, 100), (1, 150), (0, 30)]], budgets=[100]),
}


@pytest.mark.parametrize("name", list(EDGE_CASES))
def test_end_to_end_edge_cases(gpu, oracle, name):
    U = _util()
    kw = dict(dtype="bf16", H_q=2, H_kv=2, D=128, O=8, R=8, seed=21, decode_steps=2)
    kw.update(EDGE_CASES[name])
    case = W.make_case(name, **kw)
    _say(f"[e2e-edge] {name} lens={np.diff(case.cu_seqlens).tolist()} budgets={case.budget_T.tolist()}")
    H_sel = case.H_q // case.sel_group
    _end_to_end(U, oracle, case, [(b, s) for b in range(case.B) for s in range(H_sel)], 2)


@pytest.mark.parametrize("dtype,L", [("bf16", 1500), ("f32", 700), ("bf16", 5000)])
def test_all_scores_tie_lower_index_wins(gpu, oracle, dtype, L):
    """Zero queries: every logit is 0, so all prefix keys of a modality carry the same score (the
    same sum of 1/(visible keys) over the window rows) and the selection is decided by the tie rule
    alone: the lowest indices of each region, exactly as in the oracle."""
    U = _util()
    n_vis = L // 2
    case = W.make_case("ties", dtype=dtype, H_q=2, H_kv=2, D=64, O=16, R=16,
                       layouts=[[(0, 100), (1, n_vis), (0, L - 100 - n_vis)]], budgets=[L // 3], seed=3)
    case.q_win[...] = 0
    dc = U.DeviceCase(case)
    dc.layer.prune(dc.q_win, dc.k, dc.v, dc.modality)
    torch.cuda.synchronize()
    g_self = dc.layer.score_self.cpu().numpy()
    g_cross = dc.layer.score_cross.cpu().numpy()
    P = L - 16
    mod = case.modality
    for h in range(2):
        # identical bits within each region: the tie is exact on the GPU too
        assert len(np.unique(g_self[h, :P][mod[:P] == 0])) == 1 and len(np.unique(g_cross[h, :P][mod[:P] == 1])) == 1
        res = oracle.prune_group(case, 0, h)
        n = int(dc.layer.kept_cnt[0, h, 0])
        np.testing.assert_array_equal(dc.layer.kept_idx[0, h, :n].cpu().numpy(), res["idx"])
        K_s, K_c = res["counts"]["K_s"], res["counts"]["K_c"]
        text, vis = np.flatnonzero(mod[:P] == 0), np.flatnonzero(mod[:P] == 1)
        expect = np.sort(np.concatenate([text[:K_s], vis[:K_c], np.arange(P, L)]))
        np.testing.assert_array_equal(res["idx"], expect)


@pytest.mark.parametrize("dtype,scale", [("bf16", 8.0), ("f32", 16.0), ("bf16", 0.03125)])
def test_sharp_and_flat_softmax_end_to_end(gpu, oracle, dtype, scale):
    """Queries scaled by a power of two (exact in both storage types): logits with a standard deviation
    of about 8 or 16 (rows close to one-hot, most weights far below the fp32 normal range of the
    sums) and of about 0.03 (rows close to uniform, scores nearly tied)."""
    U = _util()
    case = W.make_case("sharp", dtype=dtype, H_q=4, H_kv=2, D=128, O=32, R=32, sel_group=2,
                       layouts=[[(0, 300), (1, 1400), (0, 500)], [(1, 900), (0, 140)]], budgets=[700, 300], seed=17,
                       decode_steps=2)
    if dtype == "bf16":
        for name in ("q_win", "dec_q"):
            a = getattr(case, name)
            a[...] = W.f32_to_bf16_bits(W.bf16_bits_to_f32(a) * np.float32(scale))
    else:
        case.q_win *= np.float32(scale)
        case.dec_q *= np.float32(scale)
    _end_to_end(U, oracle, case, [(b, s) for b in range(2) for s in range(2)], 2)


def test_compact_token_major_input(gpu, oracle):
    """K and V stored [tokens, H_kv, D]: same pruned cache as from the head-major layout."""
    U = _util()
    from paper_2412_04652_amd.runner import CspLayer
    case = W.make_case("tm", dtype="bf16", H_q=4, H_kv=4, D=128, O=16, R=16,
                       layouts=[[(0, 100), (1, 300), (0, 60)], [(1, 200), (0, 77)]], budgets=[200, 100], seed=5)
    dc = U.DeviceCase(case)
    dc.layer.prune(dc.q_win, dc.k, dc.v, dc.modality)
    k_tm, v_tm = dc.k.permute(1, 0, 2).contiguous(), dc.v.permute(1, 0, 2).contiguous()
    lay = CspLayer(dtype="bf16", H_q=4, H_kv=4, D=128, O=16, R=16, cu_seqlens=case.cu_seqlens.tolist(),
                   budgets=case.budget_T.tolist(), k_strides=(4 * 128, 128), v_strides=(4 * 128, 128))
    lay.prune(dc.q_win, k_tm, v_tm, dc.modality)
    torch.cuda.synchronize()
    assert torch.equal(lay.kept_idx, dc.layer.kept_idx) and torch.equal(lay.kv_len, dc.layer.kv_len)
    for b in range(2):
        n = int(lay.kv_len[b, 0])
        assert torch.equal(lay.k_cache[b, :, :n].view(torch.int16), dc.layer.k_cache[b, :, :n].view(torch.int16))
        assert torch.equal(lay.v_cache[b, :, :n].view(torch.int16), dc.layer.v_cache[b, :, :n].view(torch.int16))


def test_full_budget_identity_and_full_attention(gpu, oracle):
    """T >= L: pruning is the identity and, with n = 0, decode is textbook
    attention over the whole cache."""
    U = _util()
    case = W.make_case("ident", dtype="bf16", H_q=2, H_kv=2, D=128, O=16, R=16, n_decode=0.0,
                       layouts=[[(0, 100), (1, 200), (0, 50)]], budgets=[350], seed=8, decode_steps=1)
    dc = U.DeviceCase(case)
    lay = dc.layer
    lay.prune(dc.q_win, dc.k, dc.v, dc.modality)
    out = lay.decode(U.to_dev(case.dec_q[0], "bf16")).cpu().numpy()
    assert lay.kept_idx[0, 0].cpu().tolist() == list(range(350))
    kc = U.from_dev_bits(lay.k_cache, "bf16")
    np.testing.assert_array_equal(kc[0, 1, :350], case.k[1])
    kf = torch.tensor(W.bf16_bits_to_f32(case.k)).double()
    vf = torch.tensor(W.bf16_bits_to_f32(case.v)).double()
    qf = torch.tensor(W.bf16_bits_to_f32(case.dec_q[0, 0])).double()
    ref = torch.nn.functional.scaled_dot_product_attention(qf[:, None, :], kf, vf)[:, 0].numpy()
    U.assert_decode_close(out[0], ref, "full attention")


def test_determinism(gpu):
    U = _util()
    case = W.case_7b_4k(3, decode_steps=0)
    dc = U.DeviceCase(case)
    dc.layer.prune(dc.q_win, dc.k, dc.v, dc.modality)
    a = (dc.layer.score_self.clone(), dc.layer.kept_idx.clone(), dc.layer.k_cache.clone())
    dc.layer.prune(dc.q_win, dc.k, dc.v, dc.modality)
    torch.cuda.synchronize()
    assert torch.equal(a[0], dc.layer.score_self) and torch.equal(a[1], dc.layer.kept_idx)
    assert torch.equal(a[2].view(torch.int16), dc.layer.k_cache.view(torch.int16))


def test_probe_stream_copies_and_reads(gpu):
    """The measurement aid behind bench.py's read and copy ceilings: a copy is exact for sizes that are
    whole blocks, ragged, and smaller than one block, and touches nothing behind the end; a read-only
    pass leaves its XOR of the data in the sink."""
    import paper_2412_04652_amd as pkg
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev); g.manual_seed(5)
    for nbytes in (16, 4096, 16384 * 7, 16384 * 1024 + 16 * 37, (1 << 26) + 48):
        src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=dev, generator=g)
        whole = torch.full((nbytes + 256,), 0xA5, dtype=torch.uint8, device=dev)
        sink = torch.zeros(4096, dtype=torch.uint8, device=dev)
        pkg.csp_probe_stream(src, whole[:nbytes], sink)
        torch.cuda.synchronize()
        assert torch.equal(whole[:nbytes], src), nbytes
        assert bool((whole[nbytes:] == 0xA5).all()), nbytes
        assert not sink.any()
        pkg.csp_probe_stream(src, None, sink)
        torch.cuda.synchronize()
        words = src.view(torch.int32)
        x = int(np.bitwise_xor.reduce(words.cpu().numpy().view(np.uint32)))
        got = int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)))
        assert got == x, nbytes


def test_guard_bands_notice_a_stray_write(gpu, oracle):
    """The guard bands that every GPU test puts around a layer's buffers (tests/conftest.py): a byte
    written just outside a buffer (here by the test itself, inside its own allocation) is reported."""
    U = _util()
    case = _score_case("guards")
    dc = U.DeviceCase(case)
    dc.layer.prune(dc.q_win, dc.k, dc.v, dc.modality)
    torch.cuda.synchronize()
    live = list(U._LIVE)
    assert {name for name, _, _ in live} >= {"score_self", "score_cross", "kept_idx", "kept_cnt", "k_cache", "v_cache", "ws_score"}
    U.check_guards()                      # intact after a pruning pass (and the list is cleared)
    name, whole, n = next(x for x in live if x[0] == "kept_idx")
    U._LIVE.append((name, whole, n))
    whole[U.GUARD + n] = 0                # first byte behind the buffer
    with pytest.raises(AssertionError, match="behind the buffer"):
        U.check_guards()
    U._LIVE.append((name, whole, n))
    whole[U.GUARD + n] = U.CANARY
    whole[U.GUARD - 1] = 0                # last byte in front of it
    with pytest.raises(AssertionError, match="in front of the buffer"):
        U.check_guards()
