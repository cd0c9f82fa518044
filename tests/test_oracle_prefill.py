"""Pins for the oracle's merge-first prefill pass (Sec. 3.3.2, last sentence; App. B.4): brute force on tiny
caches, the group rule on hand-made link forests, Theorem 2 (the pass is lossless for the query whose scores
it uses), vote and mass conservation, exact duplicates (Lemma 4's zero-error case), and the order of the
policy (merge first, then the eviction strategy)."""
import math

import numpy as np
import pytest

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W


def _brute_near(k, T):
    n = k.shape[0]
    near = [-1] * n
    for i in range(1, n):
        best, arg = -math.inf, -1
        for j in range(i):
            dot = sum(float(a) * float(b) for a, b in zip(k[i], k[j]))
            u = dot / math.sqrt(sum(float(a) ** 2 for a in k[i])) / math.sqrt(sum(float(a) ** 2 for a in k[j]))
            if u > best:                                   # strict: the first maximiser stays
                best, arg = u, j
        if best > T:
            near[i] = arg
    return near


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_nearest_earlier_key_brute_force(seed):
    g = np.random.default_rng(seed)
    centres = g.standard_normal((5, 6))
    k = centres[g.integers(0, 5, size=40)] + 0.25 * g.standard_normal((40, 6))
    k[17] = k[3]                                           # an exact duplicate: similarity 1 with slot 3
    k[23] = 2.0 * k[3]                                     # and a scaled one: cosine ties, the lowest index wins
    for T in (0.8, 0.5, -2.0):
        near, sim = O.prefill_nearest_earlier(k, 40, T)
        assert near.tolist() == pytest.approx(_brute_near(k, T))
        assert near[0] == -1 and np.isneginf(sim[0])
        assert (near < np.arange(40)).all()
    near, sim = O.prefill_nearest_earlier(k, 40, 0.8)
    assert near[17] == 3 and near[23] == 3 and sim[17] == pytest.approx(1.0, abs=1e-12)
    # the threshold is strict
    near_at, _ = O.prefill_nearest_earlier(k, 40, float(sim[30]))
    assert near_at[30] == -1
    # only the live prefix takes part
    short, _ = O.prefill_nearest_earlier(k, 10, 0.8)
    assert short.shape == (10,) and short.tolist() == near[:10].tolist()


def test_groups_on_hand_made_forests():
    # a chain 0 <- 1 <- 2 <- 3 <- 4: every other slot is absorbed by its predecessor
    roots, absorbed, tgt = O.prefill_groups([-1, 0, 1, 2, 3])
    assert roots.tolist() == [0, 2, 4] and absorbed.tolist() == [1, 3] and tgt.tolist() == [0, 1]
    # a star: all link to slot 0
    roots, absorbed, tgt = O.prefill_groups([-1, 0, 0, 0])
    assert roots.tolist() == [0] and absorbed.tolist() == [1, 2, 3] and tgt.tolist() == [0, 0, 0]
    # a tree of depth two: 1 and 2 link to 0, 3 and 4 link to 1 (absorbed, so they stay), 5 links to 3
    roots, absorbed, tgt = O.prefill_groups([-1, 0, 0, 1, 1, 3])
    assert roots.tolist() == [0, 3, 4] and absorbed.tolist() == [1, 2, 5] and tgt.tolist() == [0, 0, 1]
    # no links: nothing merges
    roots, absorbed, tgt = O.prefill_groups([-1, -1, -1])
    assert roots.tolist() == [0, 1, 2] and absorbed.size == 0
    # two separate trees
    roots, absorbed, tgt = O.prefill_groups([-1, -1, 1, 0, 2])
    assert roots.tolist() == [0, 1, 4] and absorbed.tolist() == [2, 3] and tgt.tolist() == [1, 0]


def _cache_with_scores(w, seed, alpha, n_window):
    K, V = W.make_cache(w, seed)
    c = O.Cache(w.batch, w.n_kv_heads, w.context, w.head_dim)
    c.k[:], c.v[:], c.votes[:], c.len[:] = K, V, 1, w.context
    for t in range(n_window):
        q = W.make_query(w, seed, -n_window + t).astype(np.float64)
        O.observe(c, O.attend(c, q, w.scale)[2], alpha)
    return c


@pytest.mark.parametrize("threshold", [0.8, 0.3])
def test_merge_first_is_lossless_for_the_scoring_query_and_conserves_votes(threshold):
    """alpha = 0: the scores are the last query's, so by Theorem 2 attention for that (group-mean) query is
    unchanged by the pass, for groups of any size; votes and the mass sum p s_hat are conserved."""
    w = W.CONFIGS["long_32k"].scaled(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=32, context=300)   # mixture keys: many links
    c = _cache_with_scores(w, 3, 0.0, 1)
    q = W.make_query(w, 3, -1).astype(np.float64)
    before, lse_b, _ = O.attend(c, q, w.scale)
    mass_b = [np.sum(c.votes[0, h, :300] * np.exp(O.log_s_hat(c.log_S[0, h, :300], c.n_obs[0, h, :300], 0.0))) for h in range(2)]
    trace = O.prefill_merge_first(c, 0.0, threshold)
    after, lse_a, _ = O.attend(c, q, w.scale)
    np.testing.assert_allclose(after, before, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(lse_a, lse_b, rtol=1e-11)
    for h in range(2):
        n = int(c.len[0, h])
        near, roots = trace[h]
        assert n == roots.shape[0] < 300                   # something merged
        assert c.votes[0, h, :n].sum() == 300
        mass_a = np.sum(c.votes[0, h, :n] * np.exp(O.log_s_hat(c.log_S[0, h, :n], c.n_obs[0, h, :n], 0.0)))
        np.testing.assert_allclose(mass_a, mass_b[h], rtol=1e-11)
        # every absorbed slot's similarity to its receiving slot exceeded the threshold (groups are stars)
        assert (near[near >= 0] < np.flatnonzero(near >= 0)).all()


def test_exact_duplicates_collapse_with_zero_error_at_any_query():
    """Lemma 4's case: identical (k, v) pairs merge into one slot carrying their votes, and attention is
    unchanged for EVERY query, not only the scoring one."""
    g = np.random.default_rng(5)
    d, n = 16, 12
    base_k, base_v = g.standard_normal((4, d)), g.standard_normal((4, d))
    which = np.array([0, 1, 0, 2, 1, 0, 3, 2, 0, 1, 3, 3])
    c = O.Cache(1, 1, n, d)
    c.k[0, 0], c.v[0, 0], c.votes[0, 0], c.len[0, 0] = base_k[which], base_v[which], 1, n
    q0 = g.standard_normal((1, 1, d))
    O.observe(c, O.attend(c, q0, 0.25)[2], 0.0)
    q_other = g.standard_normal((1, 1, d)) * 2
    before = O.attend(c, q_other, 0.25)[0]
    O.prefill_merge_first(c, 0.0, 0.999)
    assert int(c.len[0, 0]) == 4
    assert sorted(c.votes[0, 0, :4].tolist()) == sorted(np.bincount(which).tolist())
    np.testing.assert_allclose(c.k[0, 0, :4], base_k[[0, 1, 2, 3]], rtol=1e-12)      # first occurrences, in order
    np.testing.assert_allclose(O.attend(c, q_other, 0.25)[0], before, rtol=1e-10, atol=1e-12)


def test_policy_order_merge_first_then_the_eviction_strategy():
    """Merge first, then the eviction strategy on the shorter cache (App. B.4): the pass shortens the cache
    without dropping a vote, the usual event then brings it to the budget, and votes + dropped still account
    for every prompt token; the evict-first path on the same input obeys the same conservation."""
    w = W.CONFIGS["long_32k"].scaled(batch=1, n_q_heads=4, n_kv_heads=1, head_dim=32, context=400, ratio=0.1)
    alpha, T = 0.9, 0.8
    a = _cache_with_scores(w, 2, alpha, 8)
    b = _cache_with_scores(w, 2, alpha, 8)
    O.prefill_merge_first(a, alpha, T)
    n1 = int(a.len[0, 0])
    assert w.budget < n1 < 400 and a.votes[0, 0, :n1].sum() == 400 and a.dropped[0, 0] == 0
    assert (a.votes[0, 0, :n1] >= 1).all() and (a.votes[0, 0, :n1] > 1).any()
    O.compress(a, w.budget, w.n_sink, w.n_recent, alpha, T)
    O.compress(b, w.budget, w.n_sink, w.n_recent, alpha, T)
    assert int(a.len[0, 0]) == w.budget == int(b.len[0, 0])
    assert a.votes[0, 0, : w.budget].sum() + a.dropped[0, 0] == 400
    assert b.votes[0, 0, : w.budget].sum() + b.dropped[0, 0] == 400
