"""GPU parity: keepkv_decode_attn, keepkv_score, keepkv_append against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

TOL = 2e-3   # relative error of attention outputs (per output vector), as the task states


def _case(name, **kw):
    return W.CONFIGS[name].scaled(**kw)


CASES = [
    ("tiny_f32", _case("tiny")),
    ("bf16_g4", _case("llama3_8b", batch=2, context=1000)),
    ("bf16_g8", _case("llama3_70b", batch=2, context=700)),
    ("bf16_d64_g2", _case("llama3_8b", batch=1, n_q_heads=8, n_kv_heads=4, head_dim=64, context=333)),
    ("f32_d128_g1", _case("tiny", batch=2, n_q_heads=2, n_kv_heads=2, head_dim=128, context=257)),
    ("bf16_mixture", _case("long_32k", batch=1, context=4100)),
    ("bf16_g1", _case("llama3_8b", batch=1, n_q_heads=8, n_kv_heads=8, context=555)),
    ("bf16_d64_g8", _case("llama3_8b", batch=2, n_q_heads=32, n_kv_heads=4, head_dim=64, context=300)),
    ("bf16_many_heads", _case("llama3_8b", batch=40, context=300)),     # 320 heads: the 4-wavefront workgroups
]


def test_cases_cover_both_workgroup_sizes_of_the_matrix_core_kernel():
    """The decode plan picks 8 wavefronts per workgroup for few heads and 4 for many; the parity cases above
    run under both (and under one and several splits)."""
    kk = U.kk()
    plans = {name: kk.decode_plan(U.layout_of(w), w.context) for name, w in CASES if w.dtype == "bf16"}
    assert plans["bf16_g4"][2] == 8 and plans["bf16_many_heads"][2] == 4, plans
    assert {p[2] for p in plans.values()} == {4, 8}
    assert any(p[0] == 1 for p in plans.values()) and any(p[0] > 1 for p in plans.values()), plans


@pytest.mark.parametrize("hint", [False, True], ids=["wait_for_len", "len_hint"])
@pytest.mark.parametrize("name,w", CASES, ids=[c[0] for c in CASES])
def test_decode_attn_matches_oracle(name, w, hint):
    kk = U.kk()
    K, V = W.make_cache(w, 0)
    g = np.random.default_rng(1)
    B, H, N = w.batch, w.n_kv_heads, w.context
    votes = g.integers(1, 9, size=(B, H, N)).astype(np.int32)
    lens = g.integers(1, N + 1, size=(B, H)).astype(np.int32)
    lens.flat[0] = N                      # one full head
    if lens.size > 1:
        lens.flat[1] = 0                  # one empty head
    if lens.size > 2:
        lens.flat[2] = 1
    lay, c = U.new_cache(w, capacity=N, K=K, V=V, votes=votes, lens=lens)
    if hint:
        c.len_hint = int(lens.max())            # rows below the hint may be fetched but must not matter
    # poison dead slots: they must never be read (or, below a hint, never influence a result)
    for b in range(B):
        for h in range(H):
            c.k[b, h, lens[b, h]:] = float("nan")
            c.v[b, h, lens[b, h]:] = float("nan")
    q = W.make_query(w, 0, 0)
    qd = U.to_device(q, w.dtype)
    out = torch.full_like(qd, 7.0)
    logits = torch.full((B, H, N), -123.0, dtype=torch.float32, device="cuda")
    lse = torch.zeros(B, w.n_q_heads, dtype=torch.float32, device="cuda")
    ws = U.workspace(lay, N, max(1, N // 10))
    kk.decode_attn(lay, c, qd, out, logits, lse, ws)
    torch.cuda.synchronize()
    oc = U.download(c)
    o_ref, lse_ref, lg_ref = O.attend(oc, q.astype(np.float64), w.scale)
    o_ref = W.round_storage(o_ref, w.dtype)
    got = U.to_host(out)
    err = U.rel_err_rows(got, o_ref)
    assert err.max() <= TOL, (name, err.max())
    lg = logits.cpu().numpy()
    G = w.group
    for b in range(B):
        for h in range(H):
            n = lens[b, h]
            np.testing.assert_allclose(lg[b, h, :n], lg_ref[b, h, :n], rtol=2e-3, atol=2e-3)
            assert (lg[b, h, n:] == -123.0).all()          # untouched beyond the live prefix
            if n == 0:
                assert (got[b, h * G:(h + 1) * G] == 0).all()
                assert np.isneginf(lse.cpu().numpy()[b, h * G:(h + 1) * G]).all()
    live = np.repeat(lens > 0, G, axis=1)
    np.testing.assert_allclose(lse.cpu().numpy()[live], lse_ref[live], rtol=1e-4, atol=2e-3)


@pytest.mark.parametrize("alpha", [0.0, 0.9])
def test_score_and_append_match_oracle(alpha):
    kk = U.kk()
    w = _case("llama3_8b", batch=2, context=300)
    alpha = U.f32(alpha)
    K, V = W.make_cache(w, 2)
    lay, c = U.new_cache(w, capacity=w.context + 8, K=K, V=V)
    oc = U.download(c)
    ws = U.workspace(lay, c.capacity, 64)
    logits = torch.zeros(w.batch, w.n_kv_heads, c.capacity, dtype=torch.float32, device="cuda")
    out = torch.zeros(w.batch, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    overflow = torch.zeros(1, dtype=torch.int32, device="cuda")
    for t in range(6):
        k_t, v_t = W.make_token(w, 2, t)
        kk.append(lay, c, U.to_device(k_t, w.dtype), U.to_device(v_t, w.dtype), overflow)
        oc.append(k_t, v_t)
        q = W.make_query(w, 2, t)
        kk.decode_attn(lay, c, U.to_device(q, w.dtype), out, logits, None, ws)
        kk.score(lay, c, logits, alpha)
        torch.cuda.synchronize()
        # stage-wise: the oracle consumes the GPU's logits, so only the EMA arithmetic is compared
        O.observe(oc, logits.cpu().numpy().astype(np.float64), alpha)
        n = w.context + t + 1
        assert (c.len.cpu().numpy() == n).all() and (oc.len == n).all()
        np.testing.assert_array_equal(U.n_obs(c).cpu().numpy()[:, :, :n], oc.n_obs[:, :, :n])
        np.testing.assert_allclose(c.log_s.cpu().numpy()[:, :, :n], oc.log_S[:, :, :n], rtol=1e-5, atol=1e-5)
        np.testing.assert_array_equal(U.to_host(c.k)[:, :, :n], oc.k[:, :, :n].astype(np.float32))
        np.testing.assert_array_equal(c.votes.cpu().numpy()[:, :, :n], oc.votes[:, :, :n])
        # keep the oracle's state on the GPU's f32 values for the next step
        oc.log_S[:] = c.log_s.cpu().numpy()
    assert overflow.item() == 0
    for t in range(4):                                     # run into the capacity limit
        kk.append(lay, c, U.to_device(k_t, w.dtype), U.to_device(v_t, w.dtype), overflow)
    torch.cuda.synchronize()
    assert overflow.item() == 1 and (c.len.cpu().numpy() == c.capacity).all()


@pytest.mark.parametrize("hint", [False, True], ids=["wait_for_len", "len_hint"])
@pytest.mark.parametrize("name,w", [CASES[0], CASES[1], CASES[2], CASES[3], CASES[6], CASES[7], CASES[8]],
                         ids=[CASES[i][0] for i in (0, 1, 2, 3, 6, 7, 8)])
def test_decode_step_equals_append_attend_score(name, w, hint):
    """The fused single-kernel step against the oracle's append -> attention -> EMA update."""
    kk = U.kk()
    alpha = U.f32(0.9)
    K, V = W.make_cache(w, 5)
    B, H, N = w.batch, w.n_kv_heads, w.context
    g = np.random.default_rng(2)
    lens = g.integers(1, N + 1, size=(B, H)).astype(np.int32)
    lens.flat[0] = N + 6                       # will hit the capacity limit during the run
    if lens.size > 1:
        lens.flat[1] = 0                       # starts empty
    cap = N + 8
    Kp = np.concatenate([K, K[:, :, :8]], axis=2)
    Vp = np.concatenate([V, V[:, :, :8]], axis=2)
    votes = g.integers(1, 5, size=(B, H, cap)).astype(np.int32)
    lay, c = U.new_cache(w, capacity=cap, K=Kp, V=Vp, votes=votes, lens=lens)
    c.log_s[:] = torch.from_numpy(g.standard_normal((B, H, cap)).astype(np.float32)).cuda()
    U.set_n_obs(c, g.integers(1, 9, size=(B, H, cap)).astype(np.int32))
    ws = U.workspace(lay, cap, max(1, N // 10))
    out = torch.zeros(B, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    logits = torch.zeros(B, H, cap, dtype=torch.float32, device="cuda")
    overflow = torch.zeros(1, dtype=torch.int32, device="cuda")
    oc = U.download(c)
    for b in range(B):                         # dead slots hold garbage that must never matter
        for h in range(H):
            c.k[b, h, lens[b, h]:] = float("nan")
            c.v[b, h, lens[b, h]:] = float("nan")
    for t in range(4):
        if hint:
            c.len_hint = int(min(cap, lens.max() + t))   # bound on len before this step's append
        k_t, v_t = W.make_token(w, 5, t)
        q = W.make_query(w, 5, t)
        kk.decode_step(lay, c, U.to_device(q, w.dtype), U.to_device(k_t, w.dtype), U.to_device(v_t, w.dtype), out,
                       logits if t % 2 == 0 else None, alpha, overflow, ws)
        torch.cuda.synchronize()
        for b in range(B):                     # oracle: append where there is room
            for h in range(H):
                i = int(oc.len[b, h])
                if i < cap:
                    oc.k[b, h, i], oc.v[b, h, i] = k_t[b, h], v_t[b, h]
                    oc.votes[b, h, i], oc.log_S[b, h, i], oc.n_obs[b, h, i] = 1, -np.inf, 0
                    oc.len[b, h] = i + 1
        o_ref, _, lg_ref = O.attend(oc, q.astype(np.float64), w.scale)
        O.observe(oc, lg_ref, alpha)
        np.testing.assert_array_equal(c.len.cpu().numpy(), oc.len)
        err = U.storage_err_rows(U.to_host(out), o_ref, w.dtype)
        assert err.max() <= TOL, (name, t, err.max())
        for b in range(B):
            for h in range(H):
                n = int(oc.len[b, h])
                np.testing.assert_array_equal(U.n_obs(c)[b, h, :n].cpu().numpy(), oc.n_obs[b, h, :n])
                np.testing.assert_array_equal(c.votes[b, h, :n].cpu().numpy(), oc.votes[b, h, :n])
                np.testing.assert_allclose(c.log_s[b, h, :n].cpu().numpy(), oc.log_S[b, h, :n], rtol=2e-3, atol=2e-3)
                np.testing.assert_array_equal(U.to_host(c.k)[b, h, :n], oc.k[b, h, :n].astype(np.float32))
                np.testing.assert_array_equal(U.to_host(c.v)[b, h, :n], oc.v[b, h, :n].astype(np.float32))
                if t % 2 == 0:
                    np.testing.assert_allclose(logits[b, h, :n].cpu().numpy(), lg_ref[b, h, :n], rtol=2e-3, atol=2e-3)
        oc.log_S[:] = c.log_s.cpu().numpy()    # continue from the GPU's f32 state
    assert overflow.item() == 1                # the head that started at N + 6 ran out of room
    assert c.len.cpu().numpy().flat[0] == cap


@pytest.mark.parametrize("name,w", [CASES[1], CASES[2], CASES[0]], ids=[CASES[i][0] for i in (1, 2, 0)])
def test_decode_extreme_values(name, w):
    """Logits of magnitude ~1e2..1e3 (no overflow: the running maximum carries them), votes up to a million,
    one slot dominating a head, a head whose slots all tie."""
    kk = U.kk()
    K, V = W.make_cache(w, 4)
    g = np.random.default_rng(9)
    B, H, N, G = w.batch, w.n_kv_heads, w.context, w.group
    votes = g.integers(1, 1_000_000, size=(B, H, N)).astype(np.int32)
    votes[0, 0] = 1
    K[0, 0] = K[0, 0, :1]                                   # identical keys: every slot ties
    q = W.round_storage(W.make_query(w, 4, 0) * 40.0, w.dtype)
    lay, c = U.new_cache(w, capacity=N, K=K, V=V, votes=votes)
    qd = U.to_device(q, w.dtype)
    out = torch.zeros_like(qd)
    logits = torch.zeros(B, H, N, dtype=torch.float32, device="cuda")
    lse = torch.zeros(B, w.n_q_heads, dtype=torch.float32, device="cuda")
    ws = U.workspace(lay, N, max(1, N // 10))
    kk.decode_attn(lay, c, qd, out, logits, lse, ws)
    torch.cuda.synchronize()
    oc = U.download(c)
    o_ref, lse_ref, lg_ref = O.attend(oc, q.astype(np.float64), w.scale)
    assert np.abs(lg_ref).max() > 100.0
    got = U.to_host(out)
    assert np.isfinite(got).all()
    err = U.storage_err_rows(got, o_ref, w.dtype)
    assert err.max() <= TOL, (name, err.max())
    np.testing.assert_allclose(logits.cpu().numpy(), lg_ref, rtol=2e-3, atol=2e-3)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=1e-4, atol=2e-3)
