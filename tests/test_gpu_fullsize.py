"""GPU parity at the benchmark's full sizes and launch configuration: the Llama-3-8B-shaped
workload (batch 8, context 8192 -> 820 slots) and the long-context / wide-group / stress shapes.
Sampled (batch, kv head) units are compared with the oracle element by element; properties that
hold at any size (vote conservation, index lists being a partition) are checked on every unit."""
import numpy as np
import pytest
import torch

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _unit_cache(c, b, h):
    """Oracle-side copy of one (batch, kv head) unit of a GPU cache."""
    cap, D = c.capacity, c.k.shape[-1]
    o = O.Cache(1, 1, cap, D)
    o.k[0, 0], o.v[0, 0] = U.to_host(c.k[b, h]), U.to_host(c.v[b, h])
    o.votes[0, 0], o.n_obs[0, 0] = c.votes[b, h].cpu().numpy(), U.n_obs(c)[b, h].cpu().numpy()
    o.log_S[0, 0] = c.log_s[b, h].cpu().numpy().astype(np.float64)
    o.len[0, 0] = int(c.len[b, h].item())
    return o


def _run(w, seed, n_window, n_steps, threshold, sample):
    kk = U.kk()
    alpha, T = U.f32(w.alpha), U.f32(threshold)
    B, H, G, D, N, Bud, P = w.batch, w.n_kv_heads, w.group, w.head_dim, w.context, w.budget, w.period
    K, V = W.make_cache(w, seed)
    lay, big = U.new_cache(w, capacity=N, K=K, V=V)
    del K, V
    ws = kk.new_workspace(lay, N, Bud)
    out = torch.zeros(B, w.n_q_heads, D, dtype=lay.torch_dtype, device="cuda")
    logits = torch.zeros(B, H, N, dtype=torch.float32, device="cuda")

    # observation passes over the full cache; the last one is checked on the sampled units
    for t in range(n_window):
        q = W.make_query(w, seed, t - n_window)
        if t == n_window - 1:
            pre = {u: _unit_cache(big, *u) for u in sample}
        kk.decode_attn(lay, big, U.to_device(q, w.dtype), out, logits, None, ws)
        kk.score(lay, big, logits, alpha)
    torch.cuda.synchronize()
    got = U.to_host(out)
    for (b, h), oc in pre.items():
        o_ref, _, lg = O.attend(oc, q[b:b + 1, h * G:(h + 1) * G].astype(np.float64), w.scale)
        err = U.storage_err_rows(got[b, h * G:(h + 1) * G], o_ref[0], w.dtype)
        assert err.max() <= TOL, ("window attention", b, h, err.max())
        np.testing.assert_allclose(logits[b, h].cpu().numpy(), lg[0, 0], rtol=2e-3, atol=2e-3)

    # first compression event, full size
    keep = torch.zeros(B, H, Bud, dtype=torch.int32, device="cuda")
    evict = torch.zeros(B, H, N - Bud, dtype=torch.int32, device="cuda")
    match = torch.zeros(B, H, N - Bud, dtype=torch.int32, device="cuda")
    n_ev = torch.zeros(B, H, dtype=torch.int32, device="cuda")
    dropped = torch.zeros(B, H, dtype=torch.int64, device="cuda")
    lay2, small = U.new_cache(w, capacity=Bud + P)
    pre = {u: _unit_cache(big, *u) for u in sample}
    kk.select(lay, big, Bud, w.n_sink, w.n_recent, alpha, keep, evict, n_ev, ws)
    kk.match(lay, big, Bud, keep, evict, n_ev, T, match, None, ws)
    kk.merge(lay, big, small, Bud, keep, evict, n_ev, match, alpha, dropped, ws)
    torch.cuda.synchronize()
    keep_h, evict_h, match_h = keep.cpu().numpy(), evict.cpu().numpy(), match.cpu().numpy()
    # any-size properties on every unit
    assert (n_ev.cpu().numpy() == N - Bud).all() and (small.len.cpu().numpy() == Bud).all()
    both = np.concatenate([keep_h, evict_h], axis=2)
    assert (np.sort(both, axis=2) == np.arange(N)[None, None]).all()            # a partition of the slots
    assert (np.diff(keep_h, axis=2) > 0).all() and (np.diff(evict_h, axis=2) > 0).all()
    assert ((match_h >= -1) & (match_h < Bud)).all()
    total = small.votes[:, :, :Bud].sum(dim=2).cpu().numpy() + dropped.cpu().numpy()
    assert (total == N).all()
    # sampled units against the oracle, stage by stage
    for (b, h), oc in pre.items():
        rk, re = O.select(oc.log_S[0, 0], oc.n_obs[0, 0], oc.votes[0, 0], N, Bud, w.n_sink, w.n_recent, alpha)
        np.testing.assert_array_equal(keep_h[b, h], rk)
        np.testing.assert_array_equal(evict_h[b, h], re)
        tgt, _ = O.match(oc.k[0, 0], rk, re, T, exact_any_order=(w.dtype == "bf16"))
        np.testing.assert_array_equal(match_h[b, h], tgt)
        res = O.merge(oc.k[0, 0], oc.v[0, 0], oc.votes[0, 0], oc.log_S[0, 0], oc.n_obs[0, 0], rk, re, tgt, alpha)
        np.testing.assert_array_equal(small.votes[b, h, :Bud].cpu().numpy(), res.votes)
        assert dropped[b, h].item() == res.dropped
        ev_ = U.storage_err_rows(U.to_host(small.v[b, h, :Bud]), res.v, w.dtype)
        ek = U.storage_err_rows(U.to_host(small.k[b, h, :Bud]), res.k, w.dtype)
        well = ~(np.abs(res.ell_bar) < 4 * O.ELL_GUARD)
        assert ev_.max() <= TOL and ek[well].max(initial=0) <= TOL, (b, h, ev_.max(), ek[well].max(initial=0))

    # decode steps with the fused kernel up to and including the next event's inputs
    prev = None
    for t in range(n_steps):
        k_t, v_t = W.make_token(w, seed, t, prev=prev)
        prev = (k_t, v_t) if w.key_model == "ar1" else None
        q = W.make_query(w, seed, t)
        if t == n_steps - 1:
            pre = {u: _unit_cache(small, *u) for u in sample}
        kk.decode_step(lay, small, U.to_device(q, w.dtype), U.to_device(k_t, w.dtype), U.to_device(v_t, w.dtype),
                       out, None, alpha, None, ws)
    torch.cuda.synchronize()
    assert (small.len.cpu().numpy() == Bud + n_steps).all()
    got = U.to_host(out)
    for (b, h), oc in pre.items():
        oc.append(k_t[b:b + 1, h:h + 1], v_t[b:b + 1, h:h + 1])
        o_ref, _, lg = O.attend(oc, q[b:b + 1, h * G:(h + 1) * G].astype(np.float64), w.scale)
        O.observe(oc, lg, alpha)
        err = U.storage_err_rows(got[b, h * G:(h + 1) * G], o_ref[0], w.dtype)
        assert err.max() <= TOL, ("decode step", b, h, err.max())
        n = Bud + n_steps
        np.testing.assert_allclose(small.log_s[b, h, :n].cpu().numpy(), oc.log_S[0, 0, :n], rtol=2e-3, atol=2e-3)
        np.testing.assert_array_equal(U.n_obs(small)[b, h, :n].cpu().numpy(), oc.n_obs[0, 0, :n])


def test_llama3_8b_full_size_first_event_and_decode():
    w = W.CONFIGS["llama3_8b"]
    _run(w, 0, n_window=3, n_steps=w.period, threshold=w.threshold, sample=[(0, 0), (3, 5), (7, 7)])


def test_llama3_8b_20_percent_budget_merge_all():
    w = W.CONFIGS["llama3_8b_20"].scaled(batch=2)
    _run(w, 1, n_window=2, n_steps=8, threshold=-2.0, sample=[(0, 1), (1, 6)])


def test_long_context_32k_full_size():
    w = W.CONFIGS["long_32k"]
    _run(w, 0, n_window=2, n_steps=16, threshold=w.threshold, sample=[(0, 0), (0, 7)])


def test_llama3_70b_group_of_8_reduced_batch():
    w = W.CONFIGS["llama3_70b"].scaled(batch=4)
    _run(w, 0, n_window=2, n_steps=8, threshold=w.threshold, sample=[(0, 0), (3, 4)])


def test_stress_shape_reduced_batch():
    w = W.CONFIGS["stress"].scaled(batch=2)
    _run(w, 0, n_window=2, n_steps=w.period, threshold=-2.0, sample=[(0, 2), (1, 7)])


def test_odd_head_count_with_uneven_passes():
    """9 heads (not a multiple of the 8 XCDs) with 31 blocks of evicted rows each: the first event's match
    workgroups take one or two passes, the last one ragged; the sampled heads sit at both ends."""
    w = W.CONFIGS["stress"].scaled(batch=3, n_q_heads=6, n_kv_heads=3)
    _run(w, 2, n_window=2, n_steps=4, threshold=0.5, sample=[(0, 0), (2, 2)])


@pytest.mark.parametrize("cfg,kw,window,causal", [
    ("llama3_8b", {}, 32, False),
    ("llama3_8b", {}, 32, True),
    ("long_32k", {}, 32, True),
    ("llama3_70b", {"batch": 16}, 16, False),
])
def test_window_scores_full_size(cfg, kw, window, causal):
    """keepkv_score_window at the benchmark's sizes and launch configuration; sampled units against the oracle,
    observation counts on every unit."""
    kk = U.kk()
    w = W.CONFIGS[cfg].scaled(**kw)
    alpha, seed = U.f32(w.alpha), 2
    B, H, G, N = w.batch, w.n_kv_heads, w.group, w.context
    K, V = W.make_cache(w, seed)
    lay, c = U.new_cache(w, capacity=N, K=K, V=V)
    del K, V
    q = np.stack([W.make_query(w, seed, t - window) for t in range(window)], axis=2)
    first_pos = N - window if causal else -1
    kk.score_window(lay, c, U.to_device(q, w.dtype), window, alpha, first_pos)
    torch.cuda.synchronize()
    n_obs = U.n_obs(c).cpu().numpy()
    want_n = np.full(N, window) if not causal else window - np.maximum(0, np.arange(N) - first_pos)
    assert (n_obs == want_n[None, None, :]).all()
    empty_S, empty_n = np.full(N, -np.inf), np.zeros(N, dtype=np.int64)
    for (b, h) in [(0, 0), (B - 1, H - 1), (B // 2, 3)]:
        kh = U.to_host(c.k[b, h])
        ref_S, _ = O.window_score(empty_S, empty_n, q[b, h * G:(h + 1) * G].transpose(1, 0, 2), kh, N,
                                  U.f32(w.scale), alpha, first_pos)
        np.testing.assert_allclose(c.log_s[b, h].cpu().numpy(), ref_S, rtol=1e-5, atol=2e-4, err_msg=f"unit {(b, h)}")
