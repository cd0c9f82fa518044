"""Pins for the oracle's decode loop: ordering (App. C.2), vote conservation, Thm 2 and Thm 3
across compression events on small instances of the synthetic workloads."""
import copy
import math

import numpy as np
import pytest

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W


def _prefill(w, seed, alpha):
    K, V = W.make_cache(w, seed)
    c = O.Cache(w.batch, w.n_kv_heads, w.capacity, w.head_dim)
    c.k[:, :, : w.context], c.v[:, :, : w.context] = K, V
    c.votes[:, :, : w.context] = 1
    c.len[:] = w.context
    for t in range(w.window):                       # observation window over the full cache
        q = W.make_query(w, seed, -w.window + t).astype(np.float64)
        _, _, logits = O.attend(c, q, w.scale)
        O.observe(c, logits, alpha)
    return c


@pytest.mark.parametrize("threshold", [0.8, -2.0])
def test_tiny_loop_conserves_votes(threshold):
    w = W.CONFIGS["tiny"]
    alpha = w.alpha
    c = _prefill(w, 0, alpha)
    assert (c.n_obs[:, :, : w.context] == w.window).all()
    O.compress(c, w.budget, w.n_sink, w.n_recent, alpha, threshold)
    assert (c.len == w.budget).all()
    tokens = w.context
    events = 1
    for t in range(w.steps):
        k_t, v_t = W.make_token(w, 0, t)
        c.append(k_t, v_t); tokens += 1
        q = W.make_query(w, 0, t).astype(np.float64)
        o, _, logits = O.attend(c, q, w.scale)
        O.observe(c, logits, alpha)
        assert np.isfinite(o).all()
        if (c.len == w.budget + w.period).all():
            O.compress(c, w.budget, w.n_sink, w.n_recent, alpha, threshold); events += 1
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                n = int(c.len[b, h])
                assert c.votes[b, h, :n].sum() + c.dropped[b, h] == tokens
                assert (c.votes[b, h, :n] >= 1).all() and (c.n_obs[b, h, :n] >= 1).all()
    assert events == 1 + w.steps // w.period
    if threshold < -1:
        assert (c.dropped == 0).all()
    else:
        assert (c.dropped > 0).all()                # i.i.d. Gaussian keys rarely exceed cos 0.8


def test_loop_event_is_lossless_for_the_current_query_when_alpha_is_zero():
    """App. C.2: re-running step t on the compressed cache reproduces step t's output (Thm 2)."""
    w = W.CONFIGS["tiny"].scaled(context=128, window=1, steps=8, period=4)
    c = _prefill(w, 1, 0.0)
    q = W.make_query(w, 1, -1).astype(np.float64)
    before, lse_b, _ = O.attend(c, q, w.scale)
    O.compress(c, w.budget, w.n_sink, w.n_recent, 0.0, -2.0)
    after, lse_a, _ = O.attend(c, q, w.scale)
    np.testing.assert_allclose(after, before, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(lse_a, lse_b, rtol=1e-11)
    for t in range(w.steps):
        c.append(*W.make_token(w, 1, t))
        q = W.make_query(w, 1, t).astype(np.float64)
        before, lse_b, logits = O.attend(c, q, w.scale)
        O.observe(c, logits, 0.0)
        if (c.len == w.budget + w.period).all():
            O.compress(c, w.budget, w.n_sink, w.n_recent, 0.0, -2.0)
            after, lse_a, _ = O.attend(c, q, w.scale)
            np.testing.assert_allclose(after, before, rtol=1e-9, atol=1e-12)
            np.testing.assert_allclose(lse_a, lse_b, rtol=1e-11)


def test_theorem3_across_events_on_a_small_stress_instance():
    """Between events the deviation from the un-merged cache stays under Thm 3's bound
    (eps over all merged members and merged slots of the event, frozen s_hat; all groups)."""
    w = W.CONFIGS["stress"].scaled(batch=1, n_q_heads=2, n_kv_heads=2, head_dim=16, context=96,
                                   ratio=0.25, period=4, steps=16, window=4)
    alpha, seed = 0.5, 3
    g = np.random.default_rng(9)
    base = g.standard_normal((1, 2, 16)) * 2

    def query(t):                                    # slowly drifting query: scores are predictable
        return base + 0.05 * np.random.default_rng(1000 + t).standard_normal(base.shape)

    K, V = W.make_cache(w, seed)
    c = O.Cache(1, 2, w.capacity + w.steps, 16)     # room for the un-merged shadow copy to grow
    c.k[:, :, :96], c.v[:, :, :96], c.votes[:, :, :96], c.len[:] = K, V, 1, 96
    for t in range(w.window):
        O.observe(c, O.attend(c, query(-10 + t), w.scale)[2], alpha)
    shadow = None
    checked = 0
    prev = (K[:, :, -1], V[:, :, -1])
    for t in range(-1, w.steps):
        if t >= 0:
            prev = W.make_token(w, seed, t, prev=prev)
            c.append(*prev)
            q = query(t)
            o_m, _, logits = O.attend(c, q, w.scale)
            if shadow is not None:
                pre, trace, shat = shadow
                pre.append(*prev)
                o_f, _, _ = O.attend(pre, q, w.scale)
                for h in range(2):
                    keep, evict, tgt = trace[h]
                    mem = np.concatenate([evict, keep[np.unique(tgt)]])
                    n_pre, n_post = int(pre.len[0, h]), int(c.len[0, h])
                    s_now = np.exp(w.scale * pre.k[0, h, :n_pre] @ q[0, h])
                    ratios = list(np.exp(shat["pre"][h][mem]) / s_now[mem])
                    s_post = np.exp(w.scale * c.k[0, h, :n_post] @ q[0, h])
                    ratios += list(np.exp(shat["post"][h][np.unique(tgt)]) / s_post[np.unique(tgt)])
                    eps = max(abs(1 - r) for r in ratios)
                    vv = pre.v[0, h, :n_pre]
                    gamma = max(np.linalg.norm(vv - vv[j], axis=1).max() for j in mem)
                    theta = np.linalg.norm(o_f[0, h] - o_m[0, h])
                    if eps < 1:
                        assert theta < O.perturbation_bound(eps, gamma)
                        checked += 1
            O.observe(c, logits, alpha)
        if t == -1 or (c.len == w.budget + w.period).all():
            pre = copy.deepcopy(c)
            shat_pre = [O.log_s_hat(c.log_S[0, h], c.n_obs[0, h], alpha) for h in range(2)]
            trace = O.compress(c, w.budget, w.n_sink, w.n_recent, alpha, -2.0)
            shat_post = [O.log_s_hat(c.log_S[0, h], c.n_obs[0, h], alpha) for h in range(2)]
            shadow = (pre, trace, {"pre": shat_pre, "post": shat_post})
    assert checked >= 16


def test_theorem3_on_a_stress_recipe_instance_reports_the_vacuous_fraction(capsys):
    """The stress configuration's own recipe at reduced batch and context: Mistral-7B-like head layout
    (grouped-query attention 4 : 1, head dim 128), AR(1) keys and values (rho = 0.98) continued by the decode
    tokens, the workload's peaked queries, an event every 16 steps, merge-all (T = -2).  For every event and
    every later step until the next event, per query head: theta = |o_unmerged - o_merged| against Thm 3's bound
    with eps taken over all merged members and merged slots (s_hat frozen at merge time, from the group-mean
    query; s from the head's own query) and gamma over the value distances to members.  The bound is checked
    whenever eps < 1; the fraction of (event, step, head) triples with eps >= 1, where it says nothing, is
    reported (with grouped queries the EMA of the group-mean query predicts a single head's score poorly)."""
    w = W.CONFIGS["stress"].scaled(batch=1, n_q_heads=8, n_kv_heads=2, context=640, ratio=0.1, steps=48, window=8)
    assert w.head_dim == 128 and w.group == 4 and w.period == 16 and w.key_model == "ar1"
    alpha, seed, T = 0.9, 5, -2.0
    H, G = w.n_kv_heads, w.group
    K, V = W.make_cache(w, seed)
    c = O.Cache(1, H, w.capacity + w.steps, w.head_dim)
    c.k[:, :, : w.context], c.v[:, :, : w.context], c.votes[:, :, : w.context], c.len[:] = K, V, 1, w.context
    for t in range(w.window):
        O.observe(c, O.attend(c, W.make_query(w, seed, -w.window + t).astype(np.float64), w.scale)[2], alpha)
    shadow, prev = None, (K[:, :, -1], V[:, :, -1])
    checked = vacuous = 0
    worst = 0.0
    for t in range(-1, w.steps):
        if t >= 0:
            prev = W.make_token(w, seed, t, prev=prev)
            c.append(*prev)
            q = W.make_query(w, seed, t).astype(np.float64)
            o_m, _, logits = O.attend(c, q, w.scale)
            if shadow is not None:
                pre, trace, shat = shadow
                pre.append(*prev)
                o_f, _, _ = O.attend(pre, q, w.scale)
                for h in range(H):
                    keep, evict, tgt = trace[h]
                    targets = np.unique(tgt[tgt >= 0])
                    mem = np.concatenate([evict[tgt >= 0], keep[targets]])
                    n_pre, n_post = int(pre.len[0, h]), int(c.len[0, h])
                    vv = pre.v[0, h, :n_pre]
                    gamma = max(np.linalg.norm(vv - vv[j], axis=1).max() for j in mem)
                    for g_ in range(G):
                        qh = q[0, h * G + g_]
                        s_pre = w.scale * pre.k[0, h, :n_pre] @ qh           # ln s of the head's own query
                        s_post = w.scale * c.k[0, h, :n_post] @ qh
                        dev = np.concatenate([shat["pre"][h][mem] - s_pre[mem], shat["post"][h][targets] - s_post[targets]])
                        eps = float(np.abs(1.0 - np.exp(dev)).max())
                        theta = float(np.linalg.norm(o_f[0, h * G + g_] - o_m[0, h * G + g_]))
                        if eps < 1.0:
                            bound = O.perturbation_bound(eps, gamma)
                            assert theta < bound, (t, h, g_, theta, bound, eps)
                            worst = max(worst, theta / bound)
                            checked += 1
                        else:
                            vacuous += 1
            O.observe(c, logits, alpha)
        if t == -1 or (c.len == w.budget + w.period).all():
            pre = copy.deepcopy(c)
            shat_pre = [O.log_s_hat(c.log_S[0, h], c.n_obs[0, h], alpha) for h in range(H)]
            trace = O.compress(c, w.budget, w.n_sink, w.n_recent, alpha, T)
            shat_post = [O.log_s_hat(c.log_S[0, h], c.n_obs[0, h], alpha) for h in range(H)]
            shadow = (pre, trace, {"pre": shat_pre, "post": shat_post})
    total = checked + vacuous
    assert total == w.steps * H * G
    with capsys.disabled():
        print(f"\n[Thm 3, stress recipe] {total} (event, step, head) triples: bound vacuous (eps >= 1) in "
              f"{vacuous} ({vacuous / total:.1%}); checked {checked}, largest theta / bound {worst:.3g}")
