"""Pins for the oracle's vote-weighted attention (Eq. 3, Eq. 6) and EMA scores (Eq. 8)."""
import math

import numpy as np
import pytest
import torch

from oracle import keepkv_oracle as O


def _rand(seed, S=37, G=3, d=16):
    g = np.random.default_rng(seed)
    return g.standard_normal((G, d)), g.standard_normal((S, d)), g.standard_normal((S, d))


def _sdpa(q, k, v, scale):
    """Library softmax attention (torch CPU, float64): the textbook definition of Eq. 3."""
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None], scale=scale)
    return out[0].numpy()


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_unit_votes_is_textbook_softmax(seed):
    q, k, v = _rand(seed)
    scale = 1 / math.sqrt(q.shape[1])
    o, lse, ml = O.decode_attn(q, k, v, np.ones(len(k), dtype=np.int64), len(k), scale)
    np.testing.assert_allclose(o, _sdpa(q, k, v, scale), rtol=1e-12, atol=1e-13)
    # lse is ln sum_i exp(logit_i); mean_logit is the logit of the mean query
    ref_lse = torch.logsumexp(torch.from_numpy(q @ k.T * scale), dim=1).numpy()
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-12)
    np.testing.assert_allclose(ml, scale * (k @ q.mean(0)), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("seed", [3, 4])
def test_votes_equal_physical_duplication(seed):
    """A slot with p votes acts as p identical independent copies (Sec. 3.3.1)."""
    q, k, v = _rand(seed)
    g = np.random.default_rng(seed + 100)
    votes = g.integers(1, 6, size=len(k))
    scale = 0.3
    o, lse, _ = O.decode_attn(q, k, v, votes, len(k), scale)
    kd, vd = np.repeat(k, votes, axis=0), np.repeat(v, votes, axis=0)
    np.testing.assert_allclose(o, _sdpa(q, kd, vd, scale), rtol=1e-11, atol=1e-13)
    o1, lse1, _ = O.decode_attn(q, kd, vd, np.ones(len(kd), dtype=np.int64), len(kd), scale)
    np.testing.assert_allclose(lse, lse1, rtol=1e-12)


def test_live_prefix_only_and_empty():
    q, k, v = _rand(5)
    votes = np.ones(len(k), dtype=np.int64)
    k2, v2 = k.copy(), v.copy()
    k2[20:], v2[20:] = np.nan, np.nan            # dead slots must never be read
    o, _, ml = O.decode_attn(q, k2, v2, votes, 20, 0.25)
    np.testing.assert_allclose(o, _sdpa(q, k[:20], v[:20], 0.25), rtol=1e-12)
    assert ml.shape == (20,)
    o0, lse0, ml0 = O.decode_attn(q, k, v, votes, 0, 0.25)
    assert (o0 == 0).all() and np.isneginf(lse0).all() and ml0.size == 0


def test_eviction_identity():
    """Eq. 4 / App. A.1: o' = (o - sum_j A_j v_j) / (1 - sum_j A_j) when slots j are dropped."""
    q, k, v = _rand(6, S=50, G=1)
    ones = np.ones(50, dtype=np.int64)
    o, lse, _ = O.decode_attn(q, k, v, ones, 50, 0.25)
    drop = np.array([3, 17, 18, 40])
    A = np.exp(0.25 * (k @ q[0]) - lse[0])
    assert abs(A.sum() - 1) < 1e-12
    keep = np.setdiff1d(np.arange(50), drop)
    o_ev, _, _ = O.decode_attn(q, k[keep], v[keep], ones, len(keep), 0.25)
    np.testing.assert_allclose(o_ev[0], (o[0] - A[drop] @ v[drop]) / (1 - A[drop].sum()), rtol=1e-11)


def test_large_logits_do_not_overflow():
    q, k, v = _rand(7)
    o, lse, _ = O.decode_attn(q * 400, k, v, np.ones(len(k), dtype=np.int64), len(k), 1.0)
    assert np.isfinite(o).all() and np.isfinite(lse).all()


# ----------------------------------------------------------------------------- Eq. 8
@pytest.mark.parametrize("alpha", [0.5, 0.9, 0.99])
def test_ema_closed_form(alpha):
    """S after n updates from 0 is sum_k (1-alpha) alpha^(n-k) s_k; s_hat divides by 1-alpha^n."""
    g = np.random.default_rng(11)
    n, S = 9, 13
    x = g.standard_normal((n, S)) * 3
    log_S, n_obs = np.full(S, -np.inf), np.zeros(S, dtype=np.int64)
    for t in range(n):
        log_S, n_obs = O.score_update(log_S, n_obs, x[t], S, alpha)
    wts = (1 - alpha) * alpha ** np.arange(n - 1, -1, -1)
    direct = (wts[:, None] * np.exp(x)).sum(0)
    np.testing.assert_allclose(np.exp(log_S), direct, rtol=1e-12)
    np.testing.assert_allclose(np.exp(O.log_s_hat(log_S, n_obs, alpha)), direct / (1 - alpha ** n), rtol=1e-12)
    assert (n_obs == n).all()


def test_ema_constant_input_is_unbiased_and_alpha_zero_tracks_last():
    S = 5
    x = np.linspace(-2, 2, S)
    log_S, n_obs = np.full(S, -np.inf), np.zeros(S, dtype=np.int64)
    for t in range(1, 7):
        log_S, n_obs = O.score_update(log_S, n_obs, x, S, 0.8)
        np.testing.assert_allclose(O.log_s_hat(log_S, n_obs, 0.8), x, rtol=0, atol=1e-13)
    g = np.random.default_rng(0)
    for t in range(3):
        y = g.standard_normal(S)
        log_S, n_obs = O.score_update(log_S, n_obs, y, S, 0.0)
        np.testing.assert_array_equal(O.log_s_hat(log_S, n_obs, 0.0), y)


def test_ema_only_live_slots_and_unobserved_is_zero_score():
    log_S, n_obs = np.full(6, -np.inf), np.zeros(6, dtype=np.int64)
    log_S, n_obs = O.score_update(log_S, n_obs, np.zeros(6), 4, 0.9)
    assert (n_obs == [1, 1, 1, 1, 0, 0]).all()
    assert np.isneginf(O.log_s_hat(log_S, n_obs, 0.9)[4:]).all()
    # staggered births: a slot born later has its own count
    log_S, n_obs = O.score_update(log_S, n_obs, np.ones(6), 6, 0.9)
    sh = O.log_s_hat(log_S, n_obs, 0.9)
    np.testing.assert_allclose(sh[4:], 1.0, atol=1e-13)
    np.testing.assert_allclose(np.exp(sh[0]), (0.9 * 0.1 * 1 + 0.1 * math.e) / (1 - 0.81), rtol=1e-12)


# ----------------------------------------------------------------------------- window form of Eq. 8
def _window_case(seed, W=7, G=2, d=8, n=23, cap=30):
    g = np.random.default_rng(seed)
    return g.standard_normal((W, G, d)), g.standard_normal((cap, d)), n, cap, d ** -0.5


@pytest.mark.parametrize("alpha", [0.0, 0.5, 0.9])
@pytest.mark.parametrize("first_pos", [-1, 15, 22, 3])
def test_window_score_equals_one_update_per_query(alpha, first_pos):
    """The window sum of Eq. 8 (t = L) is what the per-step recursion (t > L) builds query by query,
    also on top of an earlier state and with a causal window."""
    q, k, n, cap, scale = _window_case(0)
    W = q.shape[0]
    g = np.random.default_rng(1)
    for start in ("empty", "observed"):
        if start == "empty":
            log_S, n_obs = np.full(cap, -np.inf), np.zeros(cap, dtype=np.int64)
        else:
            log_S, n_obs = g.standard_normal(cap), g.integers(1, 5, cap)
        want_S, want_n = log_S.copy(), n_obs.copy()
        for j in range(W):
            vis = n if first_pos < 0 else max(0, min(n, first_pos + j + 1))
            logit = np.array([np.mean([scale * q[j, h] @ k[i] for h in range(q.shape[1])]) for i in range(n)])
            want_S, want_n = O.score_update(want_S, want_n, logit, vis, alpha)
        got_S, got_n = O.window_score(log_S, n_obs, q, k, n, scale, alpha, first_pos)
        np.testing.assert_allclose(got_S, want_S, rtol=1e-12, atol=1e-12)
        assert np.array_equal(got_n, want_n)
        assert np.array_equal(got_S[n:], log_S[n:]) and np.array_equal(got_n[n:], n_obs[n:])


def test_window_score_closed_forms():
    q, k, n, cap, scale = _window_case(2)
    W = q.shape[0]
    # identical queries: every observation has the same score, so the corrected EMA returns it
    q_same = np.repeat(q[:1], W, axis=0)
    S, nn = O.window_score(np.full(cap, -np.inf), np.zeros(cap, dtype=np.int64), q_same, k, n, scale, 0.8)
    x = scale * (q_same[0] @ k[:n].T).mean(0)
    np.testing.assert_allclose(O.log_s_hat(S, nn, 0.8)[:n], x, rtol=1e-12, atol=1e-12)
    assert (nn[:n] == W).all() and (nn[n:] == 0).all() and np.isinf(S[n:]).all()
    # alpha = 0 keeps the last query's score only
    S0, _ = O.window_score(np.full(cap, -np.inf), np.zeros(cap, dtype=np.int64), q, k, n, scale, 0.0)
    np.testing.assert_allclose(S0[:n], scale * (q[-1] @ k[:n].T).mean(0), rtol=1e-12)
    # causal window: slot i is seen by the queries at positions >= i; the weights are the stated powers
    first = n - W
    Sc, nc = O.window_score(np.full(cap, -np.inf), np.zeros(cap, dtype=np.int64), q, k, n, scale, 0.5, first)
    assert nc[:n].tolist() == [W] * (first + 1) + list(range(W - 1, 0, -1))
    i = n - 2                                                     # seen by the last two queries
    s = [math.exp(np.mean([scale * q[j, h] @ k[i] for h in range(q.shape[1])])) for j in (W - 2, W - 1)]
    assert math.exp(Sc[i]) == pytest.approx(0.5 * 0.5 * s[0] + 0.5 * s[1], rel=1e-12)
