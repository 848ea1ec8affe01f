"""Pins for the oracle's re-pruning step (the generation loop of Algorithm 1), CPU only.

The oracle works in cache coordinates: after every pruning the kept rows are renumbered, and
window row i sees cache rows t <= L-O+i.  The independent check below never renumbers anything:
it keeps every key ever seen with an `alive` flag, places the window queries at their absolute
positions, materialises the attention map over the whole timeline with raw exponentials (dead
and future keys get weight zero, the n of the n-softmax is added to every row sum), and ranks
the alive keys.  With R >= O (every key of the window's own positions is still cached) both
formulations describe the same attention map, so the kept absolute positions must agree after
every pruning of a whole generation loop."""
import math

import numpy as np
import pytest


def brute_prune_absolute(q_hist, K_all, mod_all, alive, n_seen, O, R, T, ratio, n_score):
    """q_hist[-O:] are the queries of absolute positions n_seen-O .. n_seen-1.  Returns the new alive mask."""
    D = K_all.shape[1]
    live = np.flatnonzero(alive[:n_seen])
    if len(live) <= T:
        return alive.copy()
    qpos = np.arange(n_seen - O, n_seen)
    S = q_hist[-O:] @ K_all[:n_seen].T / math.sqrt(D)
    see = alive[None, :n_seen] & (np.arange(n_seen)[None, :] <= qpos[:, None])
    E = np.where(see, np.exp(S), 0.0)
    A = E / (n_score + E.sum(axis=1, keepdims=True))
    rank, recent = live[:-R], live[-R:]
    qm = mod_all[qpos]
    score_self = np.array([A[qm == mod_all[j], j].sum() for j in rank])
    score_cross = np.array([A[qm != mod_all[j], j].sum() for j in rank])
    has = [bool((qm == 0).any()), bool((qm == 1).any())]
    cand_s = np.array([has[mod_all[j]] for j in rank])
    cand_c = np.array([has[1 - mod_all[j]] for j in rank])
    K_sel = T - R
    K_c = int(math.floor(ratio * K_sel))
    K_s = K_sel - K_c
    if K_s > cand_s.sum():
        K_c += K_s - int(cand_s.sum()); K_s = int(cand_s.sum())
    if K_c > cand_c.sum():
        K_s += K_c - int(cand_c.sum()); K_c = int(cand_c.sum())
    K_s = min(K_s, int(cand_s.sum()))
    ps, pc = np.flatnonzero(cand_s), np.flatnonzero(cand_c)
    top_s = rank[ps[np.argsort(-score_self[ps], kind="stable")[:K_s]]]
    top_c = rank[pc[np.argsort(-score_cross[pc], kind="stable")[:K_c]]]
    new = np.zeros_like(alive)
    new[top_s] = True
    new[top_c] = True
    new[recent] = True
    return new


@pytest.mark.parametrize("seed,O,R,T,period,mixed", [
    (0, 4, 4, 16, 1, False),    # the loop read literally: one key leaves per step
    (1, 4, 6, 18, 3, False),
    (2, 5, 5, 20, 7, False),    # more steps than the window between prunings
    (3, 4, 4, 14, 2, True),     # the prefill window holds visual queries
    (4, 3, 8, 20, 5, True),
    (5, 6, 6, 13, 4, False),
])
def test_generation_loop_matches_absolute_position_brute_force(oracle, seed, O, R, T, period, mixed):
    rng = np.random.default_rng(seed)
    D, L0, steps, ratio, n_score = 4, 36, 17, 0.4, (1.0 if seed % 2 else 0.0)
    N = L0 + steps
    K_all = rng.standard_normal((N, D))
    mod_all = np.zeros(N, dtype=np.uint8)
    mod_all[:L0] = rng.random(L0) < 0.55
    if not mixed:
        mod_all[L0 - O:L0] = 0
    else:
        mod_all[L0 - O:L0 - O + 2] = 1
    q_hist = rng.standard_normal((O, D))          # queries of positions L0-O .. L0-1
    alive = np.zeros(N, dtype=bool)
    alive[:L0] = True

    # prefill pruning, both ways
    alive = brute_prune_absolute(q_hist, K_all, mod_all, alive, L0, O, R, T, ratio, n_score)
    a_s, a_c = oracle.head_scores(q_hist, K_all[:L0], mod_all[:L0], R, n_score, True)
    idx, _ = oracle.select(a_s, a_c, mod_all[:L0], O, R, T, ratio)
    origin = idx.astype(np.int64)                  # absolute position of every cache row
    cache_k, cache_m = oracle.gather(K_all[:L0], idx), mod_all[:L0][idx]
    np.testing.assert_array_equal(origin, np.flatnonzero(alive))

    n_prunings = 0
    for t in range(steps):
        pos = L0 + t
        q_hist = np.concatenate([q_hist, rng.standard_normal((1, D))])
        alive[pos] = True
        cache_k = np.concatenate([cache_k, K_all[pos:pos + 1]])
        cache_m = np.concatenate([cache_m, [0]]).astype(np.uint8)
        origin = np.concatenate([origin, [pos]])
        if (t + 1) % period:
            continue
        alive = brute_prune_absolute(q_hist, K_all, mod_all, alive, pos + 1, O, R, T, ratio, n_score)
        res = oracle.reprune_group([q_hist[-O:]], [cache_k], cache_m, O, R, T, ratio, n_score)
        cache_k, cache_m = oracle.gather(cache_k, res["idx"]), cache_m[res["idx"]]
        origin = origin[res["idx"]]
        n_prunings += 1
        np.testing.assert_array_equal(origin, np.flatnonzero(alive), err_msg=f"after step {t}")
        assert len(origin) <= T and (np.diff(origin) > 0).all()
        assert origin[-R:].tolist() == list(range(pos + 1 - R, pos + 1))   # R >= steps since the last pruning or not: the last R alive keys
    assert n_prunings >= 2


def test_reprune_within_budget_keeps_everything(oracle):
    rng = np.random.default_rng(9)
    k = rng.standard_normal((12, 4))
    res = oracle.reprune_group([rng.standard_normal((3, 4))], [k], np.zeros(12, np.uint8), 3, 3, 12)
    assert res["idx"].tolist() == list(range(12)) and res["counts"]["kept"] == 12


def test_reprune_sums_the_heads_of_a_group(oracle):
    rng = np.random.default_rng(10)
    L, O, D = 30, 4, 8
    mod = (rng.random(L) < 0.5).astype(np.uint8); mod[-O:] = 0
    qs = [rng.standard_normal((O, D)) for _ in range(3)]
    ks = [rng.standard_normal((L, D)) for _ in range(3)]
    res = oracle.reprune_group(qs, ks, mod, O, 4, 15)
    a = sum(oracle.head_scores(q, k, mod, 4)[0] for q, k in zip(qs, ks))
    np.testing.assert_allclose(res["a_self"], a, rtol=1e-14)
