"""Pins for the CPU oracle: what the paper and the mathematics fix, computed
independently of the oracle's own code (CPU only, no GPU needed).

The paper prints no worked example (see tests/golden/README.md), so the pins
are: an independent numpy brute force that materialises the attention map and
its four explicit blocks A^st, A^sv, A^ct, A^cv (Eq. "cross-self"); exact
rational examples; closed forms of the n-softmax (Eq. "n-softmax") and of the
sharpness shift (Eq. "softmax change"); identity / count / nesting invariants
of the top-K masks (Eq. "top-K") and of Algorithm 1's early-out.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import csp_workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


# ---------------------------------------------------------------------------
# independent brute force (numpy, raw exponentials exactly as the equations
# are printed: no max subtraction, full O x L matrix, explicit blocks)
# ---------------------------------------------------------------------------
def brute_scores(q, k, mod, R, n_score=0.0):
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    O, D = q.shape
    L = k.shape[0]
    S = q @ k.T / math.sqrt(D)
    pos = np.arange(L - O, L)
    visible = np.arange(L)[None, :] <= pos[:, None]
    E = np.where(visible, np.exp(S), 0.0)
    A = E / (n_score + E.sum(axis=1, keepdims=True))
    P = L - R
    Ap = A[:, :P]
    qm, km = mod[L - O:], mod[:P]
    tq, vq, tk, vk = qm == 0, qm == 1, km == 0, km == 1
    A_st = Ap[np.ix_(tq, tk)]      # text query,   text key
    A_sv = Ap[np.ix_(vq, vk)]      # visual query, visual key
    A_ct = Ap[np.ix_(vq, tk)]      # visual query, text key
    A_cv = Ap[np.ix_(tq, vk)]      # text query,   visual key
    a_s = np.zeros(L)
    a_c = np.zeros(L)
    a_s[np.flatnonzero(tk)] = A_st.sum(axis=0)
    a_s[np.flatnonzero(vk)] = A_sv.sum(axis=0)
    a_c[np.flatnonzero(tk)] = A_ct.sum(axis=0)
    a_c[np.flatnonzero(vk)] = A_cv.sum(axis=0)
    return a_s, a_c, A


def brute_select(a_s, a_c, mod, O, R, T, ratio, combine="union"):
    L = len(mod)
    if L <= T:
        return np.arange(L)
    P = L - R
    has = [bool((mod[L - O:] == 0).any()), bool((mod[L - O:] == 1).any())]
    km = mod[:P]
    cand_s = np.flatnonzero(np.array([has[m] for m in km]))
    cand_c = np.flatnonzero(np.array([has[1 - m] for m in km]))
    K_sel = T - R
    K_c = int(math.floor(ratio * K_sel))
    K_s = K_sel - K_c
    if K_s > len(cand_s):
        K_c += K_s - len(cand_s)
        K_s = len(cand_s)
    if K_c > len(cand_c):
        K_s += K_c - len(cand_c)
        K_c = len(cand_c)
    top_s = cand_s[np.argsort(-a_s[cand_s], kind="stable")[:K_s]]
    top_c = cand_c[np.argsort(-a_c[cand_c], kind="stable")[:K_c]]
    if combine == "union":
        sel = set(top_s.tolist()) | set(top_c.tolist())
    else:
        sel = set(top_s.tolist()) & set(top_c.tolist())
    return np.array(sorted(sel | set(range(P, L))), dtype=np.int64)


def rand_mod(rng, L, O, mixed_window):
    mod = (rng.random(L) < 0.5).astype(np.uint8)
    if not mixed_window:
        mod[L - O:] = 0
    return mod


# ---------------------------------------------------------------------------
# P12 brute force on random tiny cases (mixed windows too)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(12))
def test_scores_match_brute_force_tiny(oracle, seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(8, 65))
    O = int(rng.integers(1, min(L, 9)))
    R = int(rng.integers(0, min(L, 9)))
    D = int(rng.choice([4, 8, 16]))
    n_score = float(rng.choice([0.0, 1.0, 0.3]))
    mod = rand_mod(rng, L, O, mixed_window=bool(seed % 2))
    q = rng.standard_normal((O, D))
    k = rng.standard_normal((L, D))
    a_s, a_c = oracle.head_scores(q, k, mod, R, n_score)
    b_s, b_c, _ = brute_scores(q, k, mod, R, n_score)
    np.testing.assert_allclose(a_s, b_s, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(a_c, b_c, rtol=1e-12, atol=1e-15)
    # last R entries are never written
    assert not a_s[L - R:].any() and not a_c[L - R:].any()


@pytest.mark.parametrize("seed", range(12))
def test_select_matches_brute_force_tiny(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(10, 65))
    O = int(rng.integers(1, 9))
    R = int(rng.integers(0, 9))
    T = int(rng.integers(R, L + 3))
    ratio = float(rng.choice([0.0, 0.1, 0.5, 0.9, 1.0]))
    mod = rand_mod(rng, L, O, mixed_window=bool(seed % 3 == 0))
    a_s = rng.random(L)
    a_c = rng.random(L)
    for combine in ("union", "and"):
        idx, cnt = oracle.select(a_s, a_c, mod, O, R, T, ratio, combine)
        ref = brute_select(a_s, a_c, mod, O, R, T, ratio, combine)
        np.testing.assert_array_equal(idx, ref)
        assert cnt["kept"] == len(ref)


def test_tiny_config_against_brute_force(oracle):
    """The tiny benchmark configuration, all 8 heads, scores and kept sets."""
    case = W.case_tiny(seed=0)
    mod = case.modality
    for h in range(case.H_q):
        q = case.q_win[0, h].astype(np.float64)
        k = case.k[h].astype(np.float64)
        res = oracle.prune_group(case, 0, h)
        b_s, b_c, A = brute_scores(q, k, mod, case.R, 0.0)
        np.testing.assert_allclose(res["a_self"], b_s, rtol=1e-11, atol=1e-16)
        np.testing.assert_allclose(res["a_cross"], b_c, rtol=1e-11, atol=1e-16)
        ref = brute_select(b_s, b_c, mod, case.O, case.R, 256, 0.5)
        np.testing.assert_array_equal(res["idx"], ref)
        assert res["counts"] == {"kept": 256, "K_s": 112, "K_c": 112, "both": 0}
        # P1: rows sum to one, total column mass over ALL keys = O
        np.testing.assert_allclose(A.sum(axis=1), 1.0, rtol=1e-12)
        # per-modality kept counts equal their budgets
        pref = res["idx"][res["idx"] < 512 - 32]
        assert int((mod[pref] == 0).sum()) == 112 and int((mod[pref] == 1).sum()) == 112


# ---------------------------------------------------------------------------
# exact rational example: D = 1, q = 1, k_j = ln c_j  =>  A_ij = c_j / sum c
# ---------------------------------------------------------------------------
def test_exact_rational_example(oracle):
    c = [3, 1, 4, 1, 5, 9, 2, 6]                  # weights of 8 keys
    mod = np.array([0, 1, 1, 0, 1, 0, 0, 0], np.uint8)
    L, O, R = 8, 2, 1
    q = np.ones((O, 1))
    k = np.log(np.array(c, np.float64))[:, None]
    for n in (0, 1):
        a_s, a_c, rs = oracle.head_scores(q, k, mod, R, float(n), True, want_row_sum=True)
        # window rows: positions 6 (sees c[0..6]) and 7 (sees all); both text
        den6 = Fraction(n) + sum(Fraction(x) for x in c[:7])
        den7 = Fraction(n) + sum(Fraction(x) for x in c[:8])
        for j in range(L - R):
            w = Fraction(c[j]) / den6 + Fraction(c[j]) / den7
            exp_s, exp_c = (w, 0) if mod[j] == 0 else (0, w)
            assert a_s[j] == pytest.approx(float(exp_s), rel=1e-13, abs=1e-300)
            assert a_c[j] == pytest.approx(float(exp_c), rel=1e-13, abs=1e-300)
        assert rs[0] == pytest.approx(float(1 - Fraction(n) / den6), rel=1e-13)   # P2
        assert rs[1] == pytest.approx(float(1 - Fraction(n) / den7), rel=1e-13)
    # selection on these exact scores: T=5, R=1 -> K_sel 4 -> 2 text, 2 visual.
    # text prefix keys 0,3,5,6 weights 3,1,9,2 -> {5,0}; visual 1,2,4 weights 1,4,5 -> {4,2}
    a_s, a_c = oracle.head_scores(q, k, mod, R, 0.0)
    idx, cnt = oracle.select(a_s, a_c, mod, O, R, 5, 0.5)
    assert idx.tolist() == [0, 2, 4, 5, 7]
    assert (cnt["K_s"], cnt["K_c"]) == (2, 2)


def test_visual_window_swaps_regions(oracle):
    """With an all-visual window the intra-modality region is visual->visual
    and the inter-modality region is visual->text (blocks A^sv and A^ct)."""
    rng = np.random.default_rng(5)
    L, O, R, D = 40, 4, 4, 8
    mod = rand_mod(rng, L, O, False)
    mod[L - O:] = 1
    q, k = rng.standard_normal((O, D)), rng.standard_normal((L, D))
    a_s, a_c = oracle.head_scores(q, k, mod, R)
    pre = np.arange(L - R)
    assert not a_s[pre][mod[pre] == 0].any() and not a_c[pre][mod[pre] == 1].any()
    b_s, b_c, _ = brute_scores(q, k, mod, R)
    np.testing.assert_allclose(a_s, b_s, rtol=1e-12)
    np.testing.assert_allclose(a_c, b_c, rtol=1e-12)


# ---------------------------------------------------------------------------
# P1/P2 row sums, non-causal switch, scale d = head dim
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n_score", [0.0, 1.0, 2.5])
def test_row_sums_closed_form(oracle, n_score):
    rng = np.random.default_rng(7)
    L, O, R, D = 96, 16, 0, 32
    mod = rand_mod(rng, L, O, True)
    q, k = rng.standard_normal((O, D)), rng.standard_normal((L, D))
    a_s, a_c, rs = oracle.head_scores(q, k, mod, R, n_score, want_row_sum=True)
    S = q @ k.T / math.sqrt(D)
    for i in range(O):
        e = np.exp(S[i, : L - O + i + 1]).sum()
        assert rs[i] == pytest.approx(e / (n_score + e), rel=1e-12)
    # R = 0: all the mass of every row lands in the two score vectors
    assert (a_s + a_c).sum() == pytest.approx(rs.sum(), rel=1e-12)


def test_scale_is_sqrt_head_dim(oracle):
    """One key with q.k = D and one with q.k = 0: weight of the first is
    e^{sqrt D} / (1 + e^{sqrt D})."""
    D = 16
    q = np.ones((1, D))
    k = np.stack([np.ones(D), np.zeros(D), np.zeros(D)])
    mod = np.zeros(3, np.uint8)
    a_s, _ = oracle.head_scores(q, k, mod, 0, 0.0, causal=False)
    e = math.exp(math.sqrt(D))
    assert a_s[0] == pytest.approx(e / (e + 2), rel=1e-13)


# ---------------------------------------------------------------------------
# P3 n-softmax == softmax with one extra key of logit ln(n) and zero value;
# for n = 1 this is a zero key and a zero value handed to torch's SDPA.
# ---------------------------------------------------------------------------
def test_decode_equals_library_attention_with_virtual_zero_key(oracle):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    T, D = 77, 32
    q, kc, vc = rng.standard_normal(D), rng.standard_normal((T, D)), rng.standard_normal((T, D))
    out = oracle.decode(q, kc, vc, n=1.0)
    kk = torch.tensor(np.vstack([kc, np.zeros((1, D))]))[None, None]
    vv = torch.tensor(np.vstack([vc, np.zeros((1, D))]))[None, None]
    ref = torch.nn.functional.scaled_dot_product_attention(torch.tensor(q)[None, None, None], kk, vv)
    np.testing.assert_allclose(out, ref[0, 0, 0].numpy(), rtol=1e-10, atol=1e-12)
    # n = 0 is textbook attention
    out0 = oracle.decode(q, kc, vc, n=0.0)
    ref0 = torch.nn.functional.scaled_dot_product_attention(
        torch.tensor(q)[None, None, None], torch.tensor(kc)[None, None], torch.tensor(vc)[None, None])
    np.testing.assert_allclose(out0, ref0[0, 0, 0].numpy(), rtol=1e-10, atol=1e-12)


# P4 shift law: adding c to every logit equals dividing n by e^c.  Realised by
# a constant extra coordinate: q' = [q, sqrt(D+1)*c'], k' = [k, 1].
def test_nsoftmax_shift_law(oracle):
    rng = np.random.default_rng(13)
    T, D, n, c = 50, 15, 1.0, 3.7
    q, kc, vc = rng.standard_normal(D), rng.standard_normal((T, D)), rng.standard_normal((T, D))
    s = math.sqrt(D + 1)
    # logits of the widened problem: (q.k + s*c)/s... build so logits are old*sqrt(D)/s + c
    q2 = np.concatenate([q, [c * s]])
    k2 = np.hstack([kc, np.ones((T, 1))])
    out_shift, p_shift = oracle.decode(q2, k2, np.hstack([vc, np.zeros((T, 1))]), n=n, want_p=True)
    # same logits without the shift, n scaled by e^{-c}
    q3 = np.concatenate([q, [0.0]])
    out_ref, p_ref = oracle.decode(q3, k2, np.hstack([vc, np.zeros((T, 1))]), n=n * math.exp(-c), want_p=True)
    np.testing.assert_allclose(p_shift, p_ref, rtol=1e-11)
    np.testing.assert_allclose(out_shift, out_ref, rtol=1e-10, atol=1e-13)
    # large shift: a bare n added after max-subtraction would give weights summing to ~1/2
    q4 = np.concatenate([q, [40.0 * s]])
    _, p_big = oracle.decode(q4, k2, np.hstack([vc, np.zeros((T, 1))]), n=1.0, want_p=True)
    logits = (kc @ q) / s + 40.0
    e = np.exp(logits - logits.max())
    assert p_big.sum() == pytest.approx(e.sum() / (math.exp(-logits.max()) + e.sum()), rel=1e-12)
    assert p_big.sum() > 0.999999


# P5/P6 sharpness shift: with n = mass of the pruned keys the n-softmax
# weights on the kept keys equal the un-pruned softmax weights; ordering of
# un-pruned <= n-softmax (n <= pruned mass) <= plain softmax after pruning.
def test_nsoftmax_undoes_sharpness_shift(oracle):
    rng = np.random.default_rng(17)
    L, D = 120, 16
    q, k, v = rng.standard_normal(D), rng.standard_normal((L, D)), rng.standard_normal((L, D))
    keep = np.sort(rng.choice(L, size=40, replace=False))
    drop = np.setdiff1d(np.arange(L), keep)
    logits = k @ q / math.sqrt(D)
    full = np.exp(logits) / np.exp(logits).sum()
    pruned_mass = np.exp(logits[drop]).sum()
    out, p = oracle.decode(q, k[keep], v[keep], n=pruned_mass, want_p=True)
    np.testing.assert_allclose(p, full[keep], rtol=1e-12)
    np.testing.assert_allclose(out, (full[keep, None] * v[keep]).sum(0), rtol=1e-10, atol=1e-13)
    _, p_plain = oracle.decode(q, k[keep], v[keep], n=0.0, want_p=True)
    _, p_half = oracle.decode(q, k[keep], v[keep], n=0.5 * pruned_mass, want_p=True)
    assert (full[keep] < p_half).all() and (p_half < p_plain).all()
    assert p_plain.sum() == pytest.approx(1.0, rel=1e-13)


def test_decode_empty_cache_is_zero(oracle):
    out = oracle.decode(np.ones(8), np.zeros((0, 8)), np.zeros((0, 8)), n=1.0)
    assert not out.any()


# ---------------------------------------------------------------------------
# P7 / early-out of Algorithm 1: budget >= length is the identity
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("T_minus_L", [0, 1, 50])
def test_full_budget_is_identity(oracle, T_minus_L):
    rng = np.random.default_rng(19)
    L, O, R = 64, 8, 8
    mod = rand_mod(rng, L, O, False)
    idx, cnt = oracle.select(rng.random(L), rng.random(L), mod, O, R, L + T_minus_L, 0.5)
    assert idx.tolist() == list(range(L)) and cnt["kept"] == L


def test_budget_one_below_length_drops_exactly_one(oracle):
    """T = L-1 through the spill rule: everything but the single worst
    candidate of the side that keeps fewer than it has."""
    rng = np.random.default_rng(23)
    L, O, R = 64, 8, 8
    mod = rand_mod(rng, L, O, False)
    a_s, a_c = rng.random(L), rng.random(L)
    idx, cnt = oracle.select(a_s, a_c, mod, O, R, L - 1, 0.5)
    assert cnt["kept"] == L - 1 and len(set(idx.tolist())) == L - 1


# ---------------------------------------------------------------------------
# P8 Q = 0: all logits zero, A_ij = 1/(n + p_i + 1); all prefix scores equal
# within a modality, so ties decide: lowest indices are kept
# ---------------------------------------------------------------------------
def test_zero_queries_closed_form_and_tie_rule(oracle):
    case = W.case_tiny(0)
    L, O, R = 512, 32, 32
    mod = case.modality
    for n in (0.0, 1.0):
        a_s, a_c = oracle.head_scores(np.zeros((O, 64)), case.k[0].astype(np.float64), mod, R, n)
        w = sum(1.0 / (n + (L - O + i) + 1) for i in range(O))
        pre = np.arange(L - R)
        np.testing.assert_allclose(a_s[pre][mod[pre] == 0], w, rtol=1e-13)
        np.testing.assert_allclose(a_c[pre][mod[pre] == 1], w, rtol=1e-13)
        assert not a_s[pre][mod[pre] == 1].any() and not a_c[pre][mod[pre] == 0].any()
    idx, cnt = oracle.select(a_s, a_c, mod, O, R, 256, 0.5)
    text = np.flatnonzero(mod[: L - R] == 0)[:112]
    vis = np.flatnonzero(mod[: L - R] == 1)[:112]
    expect = sorted(text.tolist() + vis.tolist() + list(range(L - R, L)))
    assert idx.tolist() == expect


# ---------------------------------------------------------------------------
# P9 planted keys: keys aligned with the mean query dominate
# ---------------------------------------------------------------------------
def test_planted_keys_are_selected(oracle):
    rng = np.random.default_rng(29)
    case = W.case_tiny(1)
    L, O, R, T = 512, 32, 32, 256
    mod = case.modality
    q = case.q_win[0, 0].astype(np.float64) + 2.0       # common direction so q-bar is not ~0
    k = case.k[0].astype(np.float64).copy()
    pre_t = np.flatnonzero(mod[: L - R] == 0)
    pre_v = np.flatnonzero(mod[: L - R] == 1)
    planted = np.concatenate([rng.choice(pre_t, 112, replace=False), rng.choice(pre_v, 112, replace=False)])
    k[planted] = 3.0 * q.mean(axis=0)
    a_s, a_c = oracle.head_scores(q, k, mod, R)
    idx, _ = oracle.select(a_s, a_c, mod, O, R, T, 0.5)
    assert set(idx[idx < L - R].tolist()) == set(planted.tolist())


# ---------------------------------------------------------------------------
# P10 / P11 counts, uniqueness, order, recent keys, nesting, permutation
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("ratio", [0.0, 0.1, 0.5, 0.9, 1.0])
def test_counts_and_order_invariants(oracle, ratio):
    case = W.case_tiny(2)
    res = None
    L, R, O = 512, 32, 32
    mod = case.modality
    a_s, a_c = oracle.group_scores(case, 0, 3)
    prev = None
    for T in (32, 33, 100, 256, 400, 511):
        idx, cnt = oracle.select(a_s, a_c, mod, O, R, T, ratio)
        assert len(idx) == T == cnt["kept"]
        assert (np.diff(idx) > 0).all()
        assert idx[-R:].tolist() == list(range(L - R, L))
        pre = idx[idx < L - R]
        assert int((mod[pre] == 0).sum()) == cnt["K_s"] and int((mod[pre] == 1).sum()) == cnt["K_c"]
        assert cnt["K_s"] + cnt["K_c"] == T - R
        if prev is not None and ratio in (0.0, 1.0):
            assert set(prev.tolist()) <= set(idx.tolist())     # nesting at a fixed split side
        prev = idx


def test_nesting_when_both_shares_grow(oracle):
    case = W.case_tiny(3)
    a_s, a_c = oracle.group_scores(case, 0, 0)
    small, c1 = oracle.select(a_s, a_c, case.modality, 32, 32, 132, 0.5)
    large, c2 = oracle.select(a_s, a_c, case.modality, 32, 32, 232, 0.5)
    assert c1["K_s"] <= c2["K_s"] and c1["K_c"] <= c2["K_c"]
    assert set(small.tolist()) <= set(large.tolist())


def test_permuting_prefix_keys_permutes_the_result(oracle):
    rng = np.random.default_rng(31)
    L, O, R, D, T = 80, 8, 8, 16, 40
    mod = rand_mod(rng, L, O, False)
    q, k = rng.standard_normal((O, D)), rng.standard_normal((L, D))
    perm = np.arange(L)
    perm[: L - R] = rng.permutation(L - R)
    a_s, a_c = oracle.head_scores(q, k, mod, R)
    b_s, b_c = oracle.head_scores(q, k[perm], mod[perm], R)
    np.testing.assert_allclose(b_s, a_s[perm], rtol=1e-12)
    np.testing.assert_allclose(b_c, a_c[perm], rtol=1e-12)
    i1, _ = oracle.select(a_s, a_c, mod, O, R, T, 0.5)
    i2, _ = oracle.select(b_s, b_c, mod[perm], O, R, T, 0.5)
    assert set(perm[i2].tolist()) == set(i1.tolist())


def test_intersection_reading_is_empty_for_a_text_window(oracle):
    """Documents why the printed AND is read as a union: with an all-text
    window the two masks live on disjoint keys."""
    case = W.case_tiny(0)
    res_u = oracle.prune_group(case, 0, 0, combine="union")
    res_a = oracle.prune_group(case, 0, 0, combine="and")
    assert res_u["counts"]["both"] == 0
    assert res_a["idx"].tolist() == list(range(512 - 32, 512))


def test_mixed_window_masks_overlap(oracle):
    """A window with both modalities makes both regions cover every prefix key;
    the masks overlap and fewer than T keys are kept (the paper's remark that
    overlap saves budget)."""
    rng = np.random.default_rng(37)
    L, O, R, D, T = 128, 16, 16, 16, 80
    mod = rand_mod(rng, L, O, True)
    assert mod[L - O:].min() == 0 and mod[L - O:].max() == 1
    q, k = rng.standard_normal((O, D)), rng.standard_normal((L, D))
    a_s, a_c = oracle.head_scores(q, k, mod, R)
    idx, cnt = oracle.select(a_s, a_c, mod, O, R, T, 0.5)
    assert cnt["K_s"] == 32 and cnt["K_c"] == 32
    assert cnt["kept"] == T - cnt["both"] and len(idx) == cnt["kept"]
    ref = brute_select(a_s, a_c, mod, O, R, T, 0.5)
    np.testing.assert_array_equal(idx, ref)


# ---------------------------------------------------------------------------
# budget rule: hand-worked table in tests/golden/budget_examples.txt
# ---------------------------------------------------------------------------
def test_budget_rule_golden(oracle):
    rows = 0
    with open(os.path.join(HERE, "golden", "budget_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, L, R, T, ratio, nt, nv, ks, kc = line.split()
            got = oracle.budget(int(T), int(R), float(ratio), int(nt), int(nv))
            assert got == (int(ks), int(kc)), name
            rows += 1
    assert rows >= 10
    with pytest.raises(ValueError):
        oracle.budget(3, 4, 0.5, 10, 10)


def test_group_sum_over_heads(oracle):
    """Selection group: scores are summed over the group's query heads."""
    case = W.make_case("g", dtype="f32", H_q=4, H_kv=2, D=16, O=8, R=8,
                       layouts=[[(0, 20), (1, 30), (0, 14)]], budgets=[32], seed=3, sel_group=2)
    a_s, a_c = oracle.group_scores(case, 0, 1)
    ref_s = np.zeros(64)
    ref_c = np.zeros(64)
    for hq in (2, 3):
        s, c, _ = brute_scores(case.q_win[0, hq], case.k[1], case.modality, 8)
        ref_s += s
        ref_c += c
    np.testing.assert_allclose(a_s, ref_s, rtol=1e-12)
    np.testing.assert_allclose(a_c, ref_c, rtol=1e-12)


def test_gather_is_a_bit_copy(oracle):
    rng = np.random.default_rng(41)
    rows = rng.integers(0, 65536, size=(50, 16), dtype=np.uint16)
    idx = np.sort(rng.choice(50, 20, replace=False)).astype(np.int32)
    np.testing.assert_array_equal(oracle.gather(rows, idx), rows[idx])


def test_batch_drivers_equal_single_calls(oracle):
    rng = np.random.default_rng(43)
    P, L, O, R, D = 5, 48, 8, 8, 16
    q, k = rng.standard_normal((P, O, D)), rng.standard_normal((P, L, D))
    mod = np.stack([rand_mod(rng, L, O, False) for _ in range(P)])
    bs, bc = oracle.scores_batch(q, k, mod, R)
    for p in range(P):
        s, c = oracle.head_scores(q[p], k[p], mod[p], R)
        np.testing.assert_array_equal(bs[p], s)
        np.testing.assert_array_equal(bc[p], c)
    kc, vc, qq = rng.standard_normal((P, 30, D)), rng.standard_normal((P, 30, D)), rng.standard_normal((P, D))
    ob = oracle.decode_batch(qq, kc, vc, 1.0)
    for p in range(P):
        np.testing.assert_array_equal(ob[p], oracle.decode(qq[p], kc[p], vc[p], 1.0))
