"""The paper's qualitative claims, reproduced with the oracle and the comparison baselines:
eviction (Eq. 4) and convex merging (Eq. 5, Theorem 1) perturb the current step, the
vote-carrying merge does not (Theorem 2)."""
import numpy as np
import pytest

from oracle import baselines as B
from oracle import keepkv_oracle as O


def _case(seed, n=48, d=16, budget=12):
    g = np.random.default_rng(seed)
    k = g.standard_normal((n, d))
    k[n // 2:] = k[: n - n // 2] + 0.2 * g.standard_normal((n - n // 2, d))     # near-duplicate keys
    v = g.standard_normal((n, d))
    q = g.standard_normal((1, d)) * 1.5
    scale = d ** -0.5
    votes = np.ones(n, dtype=np.int64)
    logit = scale * (k @ q[0])
    log_S, n_obs = O.score_update(np.full(n, -np.inf), np.zeros(n, dtype=np.int64), logit, n, 0.0)
    keep, ev = O.select(log_S, n_obs, votes, n, budget, 2, 4, 0.0)
    tgt, _ = O.match(k, keep, ev, -2.0)                                          # every evicted slot merges
    return dict(k=k, v=v, q=q, scale=scale, votes=votes, log_S=log_S, n_obs=n_obs, keep=keep, ev=ev, tgt=tgt,
                logit=logit)


def _attend(q, k, v, votes, scale):
    out, _, _ = O.decode_attn(q, k, v, votes, k.shape[0], scale)
    return out


def test_eviction_closed_form_equation4():
    c = _case(0)
    n = c["k"].shape[0]
    o = _attend(c["q"], c["k"], c["v"], c["votes"], c["scale"])[0]
    a = np.exp(c["logit"] - c["logit"].max())
    a /= a.sum()
    for e in (3, 17, n - 1):
        rest = np.array([i for i in range(n) if i != e])
        k2, v2 = B.evict(c["k"], c["v"], rest)
        o2 = _attend(c["q"], k2, v2, np.ones(n - 1, dtype=np.int64), c["scale"])[0]
        np.testing.assert_allclose(o2, B.evicted_output(o, a[e], c["v"][e]), rtol=1e-12, atol=1e-14)
        assert np.linalg.norm(o2 - o) > 0


@pytest.mark.parametrize("scheme", ["similarity", "gaussian", "uniform"])
@pytest.mark.parametrize("seed", range(3))
def test_theorem1_attention_sag_for_every_weighting_and_group_size(scheme, seed):
    c = _case(seed)
    k2, v2 = B.convex_merge(c["k"], c["v"], c["keep"], c["ev"], c["tgt"], scheme, sigma=2.0)
    s = np.exp(c["logit"])
    s2 = np.exp(c["scale"] * (k2 @ c["q"][0]))
    A, A2 = s / s.sum(), s2 / s2.sum()
    merged = 0
    for r, slot in enumerate(c["keep"]):
        members = c["ev"][c["tgt"] == r]
        if members.size == 0:
            continue
        merged += 1
        # the merged slot's score is below the largest member's, hence below their sum
        assert s2[r] <= max(s[slot], s[members].max()) * (1 + 1e-12)
        before = s[slot] + s[members].sum()
        rest = s2.sum() - s2[r]
        assert s2[r] / (rest + s2[r]) < before / (rest + before)
    assert merged >= 3
    assert A2.sum() == pytest.approx(1.0) and A.sum() == pytest.approx(1.0)
    assert s2.sum() < s.sum()                                    # total unnormalised mass shrinks: the "sag"


@pytest.mark.parametrize("seed", range(3))
def test_current_step_perturbation_ordering(seed):
    """Same retained set and merge targets for all three: only the vote-carrying merge is lossless."""
    c = _case(seed)
    o = _attend(c["q"], c["k"], c["v"], c["votes"], c["scale"])[0]
    ke, ve = B.evict(c["k"], c["v"], c["keep"])
    o_ev = _attend(c["q"], ke, ve, np.ones(len(c["keep"]), dtype=np.int64), c["scale"])[0]
    errs = {"evict": np.linalg.norm(o_ev - o)}
    for scheme in ("similarity", "gaussian", "uniform"):
        kc, vc = B.convex_merge(c["k"], c["v"], c["keep"], c["ev"], c["tgt"], scheme, sigma=2.0)
        errs[scheme] = np.linalg.norm(_attend(c["q"], kc, vc, np.ones(len(c["keep"]), dtype=np.int64), c["scale"])[0] - o)
    r = O.merge(c["k"], c["v"], c["votes"], c["log_S"], c["n_obs"], c["keep"], c["ev"], c["tgt"], 0.0)
    errs["keepkv"] = np.linalg.norm(_attend(c["q"], r.k, r.v, r.votes, c["scale"])[0] - o)
    assert errs["keepkv"] < 1e-12 * max(1.0, np.linalg.norm(o))
    assert all(errs[m] > 1e-4 for m in ("evict", "similarity", "gaussian", "uniform"))


def test_convex_weights_are_the_stated_softmaxes():
    g = np.random.default_rng(5)
    km, kc = g.standard_normal((4, 8)), g.standard_normal(8)
    km[0] = kc
    w = B.convex_weights(km, kc, "similarity")
    cos = [float(km[i] @ kc / (np.linalg.norm(km[i]) * np.linalg.norm(kc))) for i in range(4)]
    assert w == pytest.approx(np.exp(cos) / np.exp(cos).sum()) and w.argmax() == 0
    w = B.convex_weights(km, kc, "gaussian", sigma=0.7)
    z = [float(np.exp(-np.sum((km[i] - kc) ** 2) / (2 * 0.49))) for i in range(4)]
    assert w == pytest.approx(np.array(z) / sum(z)) and w.argmax() == 0
    assert B.convex_weights(km, kc, "uniform") == pytest.approx([0.25] * 4)
