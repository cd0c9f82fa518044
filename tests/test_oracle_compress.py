"""Pins for the oracle's selection, matching and ZIP-Merging (Alg. 1, Eq. 7, Thm 1-3, Lemma 4)."""
import itertools
import math

import numpy as np
import pytest
import torch
from scipy.optimize import brentq
from scipy.spatial.distance import cdist

from oracle import keepkv_oracle as O


def _sdpa_votes(q, k, v, votes, scale):
    """Textbook attention on the cache with every slot physically repeated `votes` times."""
    kd, vd = np.repeat(k, votes, axis=0), np.repeat(v, votes, axis=0)
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(kd)[None], torch.from_numpy(vd)[None], scale=scale)
    return out[0].numpy()


# ----------------------------------------------------------------------------- select
def _brute_select(key, length, budget, n_sink, n_recent):
    prot = set(range(n_sink)) | set(range(length - n_recent, length))
    cand = [i for i in range(length) if i not in prot]
    kept = set()
    for _ in range(budget - len(prot)):              # repeatedly take the best remaining slot
        best = None
        for i in cand:
            if i in kept:
                continue
            if best is None or key[i] > key[best]:   # strict: the lower index wins ties
                best = i
        kept.add(best)
    keep = sorted(prot | kept)
    return keep, [i for i in range(length) if i not in set(keep)]


@pytest.mark.parametrize("seed", range(4))
def test_select_brute_force_with_ties(seed):
    g = np.random.default_rng(seed)
    length, budget, n_sink, n_recent, alpha = 61, 20, 4, 9, 0.9
    n_obs = g.integers(1, 8, size=length)
    votes = g.integers(1, 4, size=length)
    log_S = np.round(g.standard_normal(length) * 2, 1)           # coarse values -> many exact ties
    n_obs[10:30], votes[10:30] = 3, 1
    log_S[10:30:2] = log_S.max() + 1.0                           # ten exactly tied top candidates, seven places left:
    keep, evict = O.select(log_S, n_obs, votes, length, budget, n_sink, n_recent, alpha)   # the boundary cuts the tie
    key = [math.log(votes[i]) + log_S[i] - math.log(1 - alpha ** n_obs[i]) for i in range(length)]
    bk, be = _brute_select(key, length, budget, n_sink, n_recent)
    assert keep.tolist() == bk and evict.tolist() == be
    assert len(keep) == budget and len(evict) == length - budget


def test_select_all_equal_keeps_lowest_indices_and_noop_under_budget():
    length = 40
    keep, evict = O.select(np.zeros(length), np.ones(length, dtype=int), np.ones(length, dtype=int),
                           length, 16, 4, 8, 0.9)
    assert keep.tolist() == list(range(0, 8)) + list(range(32, 40))
    keep, evict = O.select(np.zeros(length), np.ones(length, dtype=int), np.ones(length, dtype=int),
                           10, 16, 4, 8, 0.9)
    assert keep.tolist() == list(range(10)) and evict.size == 0


def test_select_votes_weight_the_mass():
    # slot 5 has a lower EMA score but 8 votes: ln 8 + (-1) > 0 + 0.5
    log_S = np.array([0, 0, 0.5, 0.4, 0.3, -1.0, 0.2, 0, 0, 0.0])
    votes = np.ones(10, dtype=int); votes[5] = 8
    keep, _ = O.select(log_S, np.full(10, 50), votes, 10, 5, 2, 2, 0.5)
    assert keep.tolist() == [0, 1, 5, 8, 9]


@pytest.mark.parametrize("seed", range(3))
def test_select_by_key_brute_force_ties_nan_and_infinities(seed):
    g = np.random.default_rng(100 + seed)
    length, budget, n_sink, n_recent = 57, 19, 3, 7
    rank = np.round(g.standard_normal(length), 1)
    rank[g.integers(0, length, 6)] = np.nan
    rank[g.integers(0, length, 3)] = -np.inf
    rank[g.integers(0, length, 2)] = np.inf
    keep, evict = O.select_by_key(rank, length, budget, n_sink, n_recent)
    key = [(-math.inf if math.isnan(x) else x) for x in rank]
    bk, be = _brute_select(key, length, budget, n_sink, n_recent)
    assert keep.tolist() == bk and evict.tolist() == be


def test_select_by_key_accumulated_attention_policy_differs_from_ema_mass():
    # a cumulative-attention ranking (sum of past attention probabilities) and the EMA mass
    # disagree on a slot that was heavy long ago: the accumulated sum keeps it, the EMA drops it
    steps, length = 40, 12
    probs = np.full((steps, length), 1.0 / length)
    probs[:10, 5] = 0.9                                          # slot 5: heavy only in the first steps
    probs[30:, 7] = 0.5                                          # slot 7: heavy recently
    acc = probs.sum(0)
    keep_acc, _ = O.select_by_key(acc, length, 5, 2, 2)
    log_S, n_obs = np.full(length, -np.inf), np.zeros(length, dtype=np.int64)
    for t in range(steps):
        log_S, n_obs = O.score_update(log_S, n_obs, np.log(probs[t]), length, 0.5)
    keep_ema, _ = O.select(log_S, n_obs, np.ones(length, dtype=int), length, 5, 2, 2, 0.5)
    assert keep_acc.tolist() == [0, 1, 5, 10, 11] and keep_ema.tolist() == [0, 1, 7, 10, 11]


# ----------------------------------------------------------------------------- match
@pytest.mark.parametrize("exact", [False, True])
def test_match_brute_force_cosine(exact):
    g = np.random.default_rng(5)
    k = g.standard_normal((50, 8))
    if exact:                                                     # bf16-like coarse values
        k = np.round(k * 8) / 8
    keep = np.sort(g.choice(50, 12, replace=False))
    evict = np.setdiff1d(np.arange(50), keep)
    tgt, sim = O.match(k, keep, evict, 0.35, exact_any_order=exact)
    U = 1.0 - cdist(k[evict], k[keep], metric="cosine")           # library cosine similarity
    for j in range(len(evict)):
        best = max(range(len(keep)), key=lambda c: (U[j, c], -c))
        assert abs(sim[j] - U[j, best]) < 1e-12
        assert tgt[j] == (best if U[j, best] > 0.35 else -1)
    assert (tgt >= 0).any() and (tgt < 0).any()


def test_match_ties_go_to_lowest_retained_position_and_threshold_is_strict():
    g = np.random.default_rng(6)
    k = g.standard_normal((10, 16))
    k[7] = k[2]                   # duplicate retained keys: 2 and 7
    k[9] = 3.0 * k[2]             # evicted, cos = 1 with both
    k[8] = -k[4]                  # evicted, cos = -1 with 4
    keep, evict = np.array([1, 2, 4, 7]), np.array([8, 9])
    tgt, sim = O.match(k, keep, evict, 0.8)
    assert tgt[1] == 1 and abs(sim[1] - 1) < 1e-15
    # strictness: threshold equal to the achieved similarity rejects
    tgt2, _ = O.match(k, keep, evict, float(sim[1]))
    assert tgt2[1] == -1
    # merge-everything threshold accepts even the worst match
    tgt3, _ = O.match(k, keep, evict, -2.0)
    assert (tgt3 >= 0).all()
    # a zero key matches nothing
    k[8] = 0
    assert O.match(k, keep, evict, -2.0)[0][0] == -1


# ----------------------------------------------------------------------------- merge
def _setup(seed, S=30, d=12, nk=9, alpha=0.0, G=1, n_steps=1, vote_hi=4):
    g = np.random.default_rng(seed)
    k, v = g.standard_normal((S, d)), g.standard_normal((S, d))
    votes = g.integers(1, vote_hi, size=S)
    scale = 1 / math.sqrt(d)
    log_S, n_obs = np.full(S, -np.inf), np.zeros(S, dtype=np.int64)
    q = None
    for _ in range(n_steps):
        q = g.standard_normal((G, d)) * 2
        _, _, ml = O.decode_attn(q, k, v, votes, S, scale)
        log_S, n_obs = O.score_update(log_S, n_obs, ml, S, alpha)
    keep = np.sort(g.choice(S, nk, replace=False))
    evict = np.setdiff1d(np.arange(S), keep)
    target = g.integers(-1, nk, size=len(evict))                  # arbitrary many-to-one map
    return dict(k=k, v=v, votes=votes, log_S=log_S, n_obs=n_obs, keep=keep, evict=evict,
                target=target, q=q, scale=scale, alpha=alpha)


def _apply(s):
    return O.merge(s["k"], s["v"], s["votes"], s["log_S"], s["n_obs"], s["keep"], s["evict"],
                   s["target"], s["alpha"])


@pytest.mark.parametrize("seed", range(5))
def test_theorem2_single_step_lossless(seed):
    """With s_hat = s (alpha = 0) the step-t output is unchanged by the merge (Thm 2), against
    textbook attention over the physically duplicated un-merged cache minus dropped slots."""
    s = _setup(seed)
    r = _apply(s)
    assert not r.guarded.any()
    live = np.concatenate([s["keep"], s["evict"][s["target"] >= 0]])
    before = _sdpa_votes(s["q"], s["k"][live], s["v"][live], s["votes"][live], s["scale"])
    after = _sdpa_votes(s["q"], r.k, r.v, r.votes, s["scale"])
    np.testing.assert_allclose(after, before, rtol=1e-10, atol=1e-12)
    # the two sums of App. A.3 hold group by group: sum p s v = p_r s_r v_r, sum p s = p_r s_r
    sc = np.exp(s["scale"] * s["k"] @ s["q"][0])
    for j, c in enumerate(s["keep"]):
        grp = [c] + s["evict"][s["target"] == j].tolist()
        s_r = math.exp(s["scale"] * r.k[j] @ s["q"][0])
        np.testing.assert_allclose(r.votes[j] * s_r, (s["votes"][grp] * sc[grp]).sum(), rtol=1e-10)
        np.testing.assert_allclose(r.votes[j] * s_r * r.v[j], (s["votes"][grp] * sc[grp]) @ s["v"][grp], rtol=1e-9, atol=1e-12)
        assert r.votes[j] == s["votes"][grp].sum()
    assert r.dropped == s["votes"][s["evict"][s["target"] < 0]].sum()


def test_pairwise_equation7():
    """|group| = 2 reproduces Eq. 7 evaluated term by term with scalar arithmetic."""
    s = _setup(10, S=2, nk=1)
    s["keep"], s["evict"], s["target"] = np.array([1]), np.array([0]), np.array([0])
    r = _apply(s)
    pe, pc = int(s["votes"][0]), int(s["votes"][1])
    se = math.exp(s["scale"] * float(s["k"][0] @ s["q"][0]))
    sc = math.exp(s["scale"] * float(s["k"][1] @ s["q"][0]))
    we, wc = pe * se, pc * sc
    kr = (we * s["k"][0] + wc * s["k"][1]) * math.log((we + wc) / (pe + pc)) / (we * math.log(se) + wc * math.log(sc))
    vr = (we * s["v"][0] + wc * s["v"][1]) / (we + wc)
    np.testing.assert_allclose(r.k[0], kr, rtol=1e-12)
    np.testing.assert_allclose(r.v[0], vr, rtol=1e-12)
    assert r.votes[0] == pe + pc


def test_closed_forms_equal_scores_and_unit_score():
    d = 4
    ke, kc = np.array([1.0, 2, 3, 4]), np.array([-1.0, 0, 5, 2])
    ve, vc = np.array([1.0, 0, 0, 0]), np.array([0.0, 1, 0, 0])
    k, v = np.stack([ke, kc]), np.stack([ve, vc])
    one = np.array([1, 1])
    # equal scores e^a: the merged key and value are the plain means, votes 2, ln s_hat_r = a
    r = O.merge(k, v, one, np.array([0.7, 0.7]), one, [1], [0], [0], 0.0)
    np.testing.assert_allclose(r.k[0], (ke + kc) / 2, rtol=1e-14)
    np.testing.assert_allclose(r.v[0], (ve + vc) / 2, rtol=1e-14)
    assert r.votes[0] == 2 and abs(r.log_S[0] - 0.7) < 1e-14
    # s_e = 1, s_c = e: k_r = (k_e + e k_c) ln((1 + e)/2) / e ; v_r = (v_e + e v_c)/(1 + e)
    r = O.merge(k, v, one, np.array([0.0, 1.0]), one, [1], [0], [0], 0.0)
    e = math.e
    np.testing.assert_allclose(r.k[0], (ke + e * kc) * math.log((1 + e) / 2) / e, rtol=1e-14)
    np.testing.assert_allclose(r.v[0], (ve + e * vc) / (1 + e), rtol=1e-14)
    # unequal votes 3 and 1, s_e = e^2, s_c = e^-1
    r = O.merge(k, v, np.array([3, 1]), np.array([2.0, -1.0]), one, [1], [0], [0], 0.0)
    we, wc = 3 * e ** 2, e ** -1
    np.testing.assert_allclose(r.k[0], (we * ke + wc * kc) * math.log((we + wc) / 4) / (2 * we - wc), rtol=1e-13)
    assert r.votes[0] == 4


@pytest.mark.parametrize("alpha,n_steps", [(0.9, 5), (0.5, 3)])
def test_mass_conservation_with_ema_scores(alpha, n_steps):
    """p_r s_hat_r = sum p_i s_hat_i (App. A.4), read back through the stored ln S and n."""
    s = _setup(20, alpha=alpha, n_steps=n_steps)
    r = _apply(s)
    sh = np.exp(O.log_s_hat(s["log_S"], s["n_obs"], alpha))
    sh_r = np.exp(O.log_s_hat(r.log_S, r.n_obs, alpha))
    for j, c in enumerate(s["keep"]):
        grp = [c] + s["evict"][s["target"] == j].tolist()
        np.testing.assert_allclose(r.votes[j] * sh_r[j], (s["votes"][grp] * sh[grp]).sum(), rtol=1e-11)
        w = s["votes"][grp] * sh[grp]
        np.testing.assert_allclose(r.v[j], w @ s["v"][grp] / w.sum(), rtol=1e-10, atol=1e-13)
        # key direction is the weighted mean; its length obeys ln(W/P) <= sum w ln s / W
        kbar = w @ s["k"][grp] / w.sum()
        if len(grp) > 1:
            L, ell = math.log(w.sum() / s["votes"][grp].sum()), (w * np.log(sh[grp])).sum() / w.sum()
            assert L <= ell + 1e-12
            np.testing.assert_allclose(r.k[j], kbar * L / ell, rtol=1e-10)
    assert r.votes.sum() + r.dropped == s["votes"].sum()


def test_gqa_lossless_for_the_group_mean_query():
    s = _setup(30, G=4)
    r = _apply(s)
    qbar = s["q"].mean(0, keepdims=True)
    live = np.concatenate([s["keep"], s["evict"][s["target"] >= 0]])
    before = _sdpa_votes(qbar, s["k"][live], s["v"][live], s["votes"][live], s["scale"])
    after = _sdpa_votes(qbar, r.k, r.v, r.votes, s["scale"])
    np.testing.assert_allclose(after, before, rtol=1e-10, atol=1e-12)


def test_lemma4_identical_members_zero_perturbation_at_any_later_query():
    g = np.random.default_rng(40)
    S, d = 12, 8
    k, v = g.standard_normal((S, d)), g.standard_normal((S, d))
    k[[3, 5, 9]], v[[3, 5, 9]] = k[3], v[3]                       # three identical pairs
    votes = g.integers(1, 4, size=S)
    log_S = g.standard_normal(S); log_S[[5, 9]] = log_S[3]; n = np.full(S, 4)
    keep = np.array([0, 1, 2, 3, 4, 6, 7, 8, 10, 11]); evict = np.array([5, 9])
    r = O.merge(k, v, votes, log_S, n, keep, evict, np.array([3, 3]), 0.9)
    np.testing.assert_allclose(r.k[3], k[3], rtol=1e-13)
    np.testing.assert_allclose(r.v[3], v[3], rtol=1e-13)
    assert r.votes[3] == votes[[3, 5, 9]].sum()
    q2 = g.standard_normal((2, d)) * 3                            # any other query
    np.testing.assert_allclose(_sdpa_votes(q2, r.k, r.v, r.votes, 0.4),
                               _sdpa_votes(q2, k, v, votes, 0.4), rtol=1e-10, atol=1e-12)


def test_theorem1_convex_merge_sags():
    """Negative control: a convex combination (Eq. 5) lowers the merged slot's attention share."""
    s = _setup(50)
    sc = np.exp(s["scale"] * s["k"] @ s["q"][0])
    e, c = 0, 1
    for w_e in (0.2, 0.5, 0.8):
        k_r = w_e * s["k"][e] + (1 - w_e) * s["k"][c]
        s_r = math.exp(s["scale"] * k_r @ s["q"][0])
        rest = sc[2:].sum()
        assert s_r / (rest + s_r) < (sc[e] + sc[c]) / sc.sum()


@pytest.mark.parametrize("seed", range(6))
def test_theorem3_bound_at_a_later_step(seed):
    """Theta_{t'} < 2 eps (1+eps) gamma / (1-eps)^2 with eps over the merged members and the
    merged slot, gamma over value distances to the members (Thm 3), one group merged."""
    g = np.random.default_rng(100 + seed)
    S, d = 20, 8
    k, v = g.standard_normal((S, d)) * 0.5, g.standard_normal((S, d))
    votes = g.integers(1, 3, size=S)
    scale = 1 / math.sqrt(d)
    q = g.standard_normal((1, d)) * 2
    _, _, ml = O.decode_attn(q, k, v, votes, S, scale)
    keep = np.arange(1, S) if seed % 2 else np.arange(2, S)
    evict = np.setdiff1d(np.arange(S), keep)
    r = O.merge(k, v, votes, ml, np.ones(S, dtype=int), keep, evict, np.zeros(len(evict), dtype=int), 0.0)
    grp = [int(keep[0])] + evict.tolist()
    q2 = q + g.standard_normal((1, d)) * 0.15                     # the next step's query
    o_full = _sdpa_votes(q2, k, v, votes, scale)
    o_merged = _sdpa_votes(q2, r.k, r.v, r.votes, scale)
    theta = np.linalg.norm(o_full - o_merged)
    s2 = np.exp(scale * k @ q2[0]); s_hat = np.exp(ml)
    ratios = [s_hat[i] / s2[i] for i in grp]
    ratios.append(math.exp(r.log_S[0]) / math.exp(scale * r.k[0] @ q2[0]))
    eps = max(abs(1 - x) for x in ratios)
    gamma = max(np.linalg.norm(v[j] - v[i]) for i in range(S) for j in grp)
    assert eps < 1 and theta > 0
    assert theta < O.perturbation_bound(eps, gamma)


def test_guard_and_unobserved_members():
    d = 3
    k = np.array([[1.0, 0, 0], [0, 1.0, 0], [0, 0, 2.0]]); v = k.copy()
    one = np.ones(3, dtype=int)
    # weights e^{+a}, e^{-b} chosen so that sum w ln s = 0: a e^a = b e^-b
    a = 0.2
    b = brentq(lambda x: x * math.exp(-x) - a * math.exp(a), 0.0, 1.0, xtol=1e-15)
    r = O.merge(k, v, one, np.array([a, -b, 0.0]), one, [0, 2], [1], [0], 0.0)
    assert r.guarded[0] and not r.guarded[1]
    w = np.array([math.exp(a), math.exp(-b)])
    np.testing.assert_allclose(r.k[0], (w[0] * k[0] + w[1] * k[1]) / w.sum(), rtol=1e-13)
    # an unobserved member contributes votes but no weight
    r = O.merge(k, v, one, np.array([0.5, -np.inf, 0.0]), np.array([2, 0, 2]), [0, 2], [1], [0], 0.9)
    np.testing.assert_allclose(r.v[0], v[0]); assert r.votes[0] == 2
    np.testing.assert_allclose(r.k[0], k[0] * math.log(math.exp(0.5 - math.log(1 - 0.81)) / 2) / (0.5 - math.log(1 - 0.81)), rtol=1e-13)


def test_unobserved_retained_slot_takes_its_observed_members_score():
    """Reading R12 for a retained slot that was never observed (n = 0, weight 0) absorbing an observed member:
    the merged slot is all the member's key direction and value, carries both votes, and its score obeys the
    mass identity p_r s_hat_r = sum p s_hat (App. A.4) with the observation count raised to 1."""
    alpha = 0.9
    k = np.array([[1.0, 2.0], [3.0, -1.0], [0.5, 0.5]]); v = np.array([[1.0, 0.0], [0.0, 4.0], [2.0, 2.0]])
    votes = np.array([2, 3, 1])
    n_obs = np.array([0, 5, 4])                                   # slot 0 (retained) unobserved, slot 1 (member) observed
    E1 = 0.7                                                      # ln s_hat of the member
    log_S = np.array([-np.inf, E1 + math.log(1 - alpha ** 5), 0.1])
    r = O.merge(k, v, votes, log_S, n_obs, [0, 2], [1], [0], alpha)
    assert r.votes[0] == 5 and r.n_obs[0] == 1 and not r.guarded[0]
    np.testing.assert_allclose(r.v[0], v[1], rtol=1e-14)          # the only member with weight
    L = math.log(3 * math.exp(E1) / 5)                            # ln(sum p s_hat / sum p)
    np.testing.assert_allclose(r.k[0], k[1] * (L / E1), rtol=1e-13)
    np.testing.assert_allclose(r.log_S[0], L + math.log(1 - alpha ** 1), rtol=1e-13)
    np.testing.assert_allclose(5 * math.exp(r.log_S[0] - math.log(1 - alpha)), 3 * math.exp(E1), rtol=1e-13)
    # the untouched retained slot is a copy
    assert r.votes[1] == 1 and r.n_obs[1] == 4 and r.log_S[1] == 0.1


def test_perturbation_bound_values():
    """Theorem 3's right-hand side 2 eps (1 + eps) gamma / (1 - eps)^2 at values worked by hand."""
    assert O.perturbation_bound(0.5, 1.0) == pytest.approx(6.0, rel=1e-15)          # 2 * .5 * 1.5 / .25
    assert O.perturbation_bound(0.0, 3.0) == 0.0
    assert O.perturbation_bound(0.1, 2.0) == pytest.approx(2 * 0.1 * 1.1 * 2.0 / 0.81, rel=1e-15)
    assert O.perturbation_bound(0.2, 1.0) == pytest.approx(0.75, rel=1e-15)         # .4 * 1.2 / .64
    assert O.perturbation_bound(0.5, 2.0) == 2 * O.perturbation_bound(0.5, 1.0)      # linear in gamma
