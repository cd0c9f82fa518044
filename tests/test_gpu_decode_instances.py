"""GPU parity of every decode kernel instance the benchmark configurations launch at full size.

The matrix-core decode kernel is compiled per (head dim, group size, step / attention only, single tile per
wavefront / tile loop, 4 / 8 wavefronts).  Which instance runs is decided by the host plan from batch, heads and
capacity, so small parity shapes do not reach what the full-size shapes launch.  Here
  * every benchmark configuration runs `keepkv_decode_step` at its full batch on a steady-state cache
    (capacity = budget + period, ragged lengths) under the plan the library chooses, and sampled
    (batch, kv head) units are compared with the oracle element by element (Eq. 6, Eq. 8);
  * every instance at head dim 128 is forced through the per-call plan overrides of `keepkv_cache` on a
    shape small enough to compare all units.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
TOL = 2e-3
HEAD = 64 * 1024 + 256       # control words at the head of a workspace (keepkv.h)


def _workspace_for(lay, cap, per):
    """Workspace for a decode call with `per` slots per split forced (size rule of keepkv.h)."""
    kk = U.kk()
    ns = -(-cap // per)
    need = HEAD + lay.batch * lay.n_q_heads * ns * (lay.head_dim + 2) * 4 + 256
    ws = torch.empty(max(need, kk.workspace_bytes(lay, cap, max(1, cap // 2))), dtype=torch.uint8, device="cuda")
    kk.workspace_init(ws)
    return ws


def _steady_state(w, cap, seed, lens):
    """A cache of `cap` slots per head with random votes, EMA state and the given lengths."""
    g = np.random.default_rng(seed)
    B, H = w.batch, w.n_kv_heads
    K, V = W.make_cache(w.scaled(context=cap), seed)
    votes = g.integers(1, 6, size=(B, H, cap)).astype(np.int32)
    lay, c = U.new_cache(w, capacity=cap, K=K, V=V, votes=votes, lens=lens)
    del K, V
    c.log_s[:] = torch.from_numpy(g.standard_normal((B, H, cap)).astype(np.float32)).cuda()
    U.set_n_obs(c, g.integers(1, 40, size=(B, H, cap)).astype(np.int32))
    return lay, c


def _ragged_lens(g, B, H, cap, per, nsplit):
    """Lengths near capacity with the special cases: a head at capacity, an empty head, one slot, heads
    about to cross a 32-slot tile and a split boundary, a head ending exactly on a split boundary."""
    lens = g.integers(max(1, cap - 3 * 64), cap, size=(B, H)).astype(np.int32)
    flat = lens.reshape(-1)
    special = [cap, 0, 1, 32 * ((cap - 40) // 32) - 1, 32 * ((cap - 40) // 32)]
    if nsplit > 1:
        special += [per * (nsplit - 1) - 1, per * (nsplit - 1), per - 2]
    for i, v in enumerate(special[: flat.size]):
        flat[i] = v
    return lens, list(range(min(len(special), flat.size)))


def _check_steps(w, lay, c, ws, sample, n_steps, seed, hint, tag):
    """Run decode steps on the GPU and compare the sampled units with the oracle after every step."""
    kk = U.kk()
    alpha = U.f32(0.9)
    B, H, G, D, cap = w.batch, w.n_kv_heads, w.group, w.head_dim, c.capacity
    out = torch.zeros(B, w.n_q_heads, D, dtype=lay.torch_dtype, device="cuda")
    overflow = torch.zeros(1, dtype=torch.int32, device="cuda")
    bs = torch.tensor([u // H for u in sample], device="cuda")
    hs = torch.tensor([u % H for u in sample], device="cuda")

    def snapshot():
        return dict(k=U.to_host(c.k[bs, hs]), v=U.to_host(c.v[bs, hs]), votes=c.votes[bs, hs].cpu().numpy(),
                    log_s=c.log_s[bs, hs].cpu().numpy(), n_obs=U.n_obs(c)[bs, hs].cpu().numpy(), born=c.born[bs, hs].cpu().numpy(),
                    len=c.len[bs, hs].cpu().numpy())

    lens_max = int(c.len.max().item())
    for t in range(n_steps):
        pre = snapshot()
        c.len_hint = min(cap, lens_max + t) if hint else 0
        k_t, v_t = W.make_token(w, seed, t)
        q = W.make_query(w, seed, t)
        kk.decode_step(lay, c, U.to_device(q, w.dtype), U.to_device(k_t, w.dtype), U.to_device(v_t, w.dtype), out,
                       None, alpha, overflow, ws)
        torch.cuda.synchronize()
        post = snapshot()
        got = U.to_host(out)
        for i, u in enumerate(sample):
            b, h = u // H, u % H
            k, v = pre["k"][i].astype(np.float64), pre["v"][i].astype(np.float64)
            votes, log_S, n_obs = pre["votes"][i].astype(np.int64), pre["log_s"][i].astype(np.float64), pre["n_obs"][i]
            n = int(pre["len"][i])
            if n < cap:                                    # the append of this step
                k[n], v[n], votes[n], log_S[n], n_obs[n] = k_t[b, h], v_t[b, h], 1, -np.inf, 0
                n += 1
            o_ref, _, ml = O.decode_attn(q[b, h * G:(h + 1) * G], k, v, votes, n, w.scale)
            S_ref, n_ref = O.score_update(log_S, n_obs, ml, n, alpha)
            where = (tag, "step", t, "unit", b, h, "len", n)
            assert int(post["len"][i]) == n, where
            err = U.storage_err_rows(got[b, h * G:(h + 1) * G], o_ref, w.dtype)
            assert err.max() <= TOL, (where, float(err.max()))
            np.testing.assert_array_equal(post["n_obs"][i][:n], n_ref[:n], err_msg=str(where))
            np.testing.assert_allclose(post["log_s"][i][:n], S_ref[:n], rtol=2e-3, atol=2e-3, err_msg=str(where))
            np.testing.assert_array_equal(post["votes"][i][:n], votes[:n], err_msg=str(where))
            np.testing.assert_array_equal(post["k"][i][:n], k[:n].astype(np.float32), err_msg=str(where))
            np.testing.assert_array_equal(post["v"][i][:n], v[:n].astype(np.float32), err_msg=str(where))
            # slots beyond the live prefix are untouched
            np.testing.assert_array_equal(post["log_s"][i][n:], pre["log_s"][i][n:], err_msg=str(where))
            np.testing.assert_array_equal(post["born"][i][n:], pre["born"][i][n:], err_msg=str(where))
    return overflow.item()


FULL = ["llama3_8b", "llama3_8b_20", "long_32k", "llama3_70b", "stress"]


@pytest.mark.parametrize("hint", [True, False], ids=["len_hint", "wait_for_len"])
@pytest.mark.parametrize("name", FULL)
def test_decode_step_full_batch_steady_state(name, hint):
    """What bench.py launches per step: the configuration's full batch on a cache of budget + period slots."""
    kk = U.kk()
    w = W.CONFIGS[name]
    cap = w.budget + w.period
    lay = U.layout_of(w)
    nsplit, per, waves = kk.decode_plan(lay, cap)
    print(f"{name}: capacity {cap}, plan {nsplit} x {per} slots, {waves} wavefronts, "
          f"{'single tile' if per <= waves * 32 else 'tile loop'}", flush=True)
    g = np.random.default_rng(11)
    B, H = w.batch, w.n_kv_heads
    lens, special = _ragged_lens(g, B, H, cap, per, nsplit)
    lay, c = _steady_state(w, cap, 11, lens)
    ws = U.workspace(lay, cap, w.budget)
    units = B * H
    sample = sorted(set(special) | set(g.choice(units, size=min(units, 12), replace=False).tolist()))
    ov = _check_steps(w, lay, c, ws, sample, 3, 11, hint, name)
    assert ov == 1                                         # the head that started at capacity


# (wavefronts, slots per split) at capacity 900: single tile per wavefront, two / four tiles, one long split
FORCED = [(8, 256), (8, 448), (8, 928), (4, 128), (4, 256), (4, 448), (4, 928)]


@pytest.mark.parametrize("waves,per", FORCED, ids=[f"w{a}_per{b}" for a, b in FORCED])
@pytest.mark.parametrize("base", ["llama3_8b", "llama3_70b"], ids=["g4", "g8"])
def test_every_d128_instance_step(base, waves, per):
    w = W.CONFIGS[base].scaled(batch=3, context=900)
    cap = 900
    g = np.random.default_rng(waves * 1000 + per)
    B, H = w.batch, w.n_kv_heads
    nsplit = -(-cap // per)
    lens, _ = _ragged_lens(g, B, H, cap, per, nsplit)
    lay, c = _steady_state(w, cap, 13, lens)
    c.plan_wavefronts, c.plan_slots_per_split = waves, per
    ws = _workspace_for(lay, cap, per)
    _check_steps(w, lay, c, ws, list(range(B * H)), 2, 13, hint=(per % 64 == 0), tag=(base, waves, per))


@pytest.mark.parametrize("waves,per", FORCED + [(-1, 256)], ids=[f"w{a}_per{b}" for a, b in FORCED + [(-1, 256)]])
@pytest.mark.parametrize("base", ["llama3_8b", "llama3_70b"], ids=["g4", "g8"])
def test_every_d128_instance_attention_only(base, waves, per):
    """keepkv_decode_attn (no append, no score update) under every forced launch shape, including the
    vector-ALU kernel on a bf16 cache (plan_wavefronts = -1)."""
    kk = U.kk()
    w = W.CONFIGS[base].scaled(batch=3, context=900)
    cap = 900
    g = np.random.default_rng(7 + abs(waves) * 1000 + per)
    B, H, G = w.batch, w.n_kv_heads, w.group
    nsplit = -(-cap // per)
    lens, _ = _ragged_lens(g, B, H, cap, per, nsplit)
    lay, c = _steady_state(w, cap, 17, lens)
    for b, h in itertools.product(range(B), range(H)):     # dead slots must never matter
        c.k[b, h, lens[b, h]:] = float("nan")
        c.v[b, h, lens[b, h]:] = float("nan")
    c.plan_wavefronts, c.plan_slots_per_split = waves, per
    ws = _workspace_for(lay, cap, per)
    q = W.make_query(w, 17, 0)
    qd = U.to_device(q, w.dtype)
    out = torch.full_like(qd, 7.0)
    logits = torch.full((B, H, cap), -123.0, dtype=torch.float32, device="cuda")
    lse = torch.zeros(B, w.n_q_heads, dtype=torch.float32, device="cuda")
    before = (c.log_s.clone(), c.born.clone(), c.len.clone(), c.t_obs.clone())
    kk.decode_attn(lay, c, qd, out, logits, lse, ws)
    torch.cuda.synchronize()
    assert torch.equal(before[0], c.log_s) and torch.equal(before[1], c.born) and torch.equal(before[2], c.len)
    assert torch.equal(before[3], c.t_obs)
    oc = U.download(c)
    oc.k[np.isnan(oc.k)] = 0.0
    oc.v[np.isnan(oc.v)] = 0.0
    o_ref, lse_ref, lg_ref = O.attend(oc, q.astype(np.float64), w.scale)
    got = U.to_host(out)
    err = U.storage_err_rows(got, o_ref, w.dtype)
    assert err.max() <= TOL, (base, waves, per, float(err.max()))
    lg = logits.cpu().numpy()
    for b, h in itertools.product(range(B), range(H)):
        n = lens[b, h]
        np.testing.assert_allclose(lg[b, h, :n], lg_ref[b, h, :n], rtol=2e-3, atol=2e-3)
        assert (lg[b, h, n:] == -123.0).all()
    live = np.repeat(lens > 0, G, axis=1)
    np.testing.assert_allclose(lse.cpu().numpy()[live], lse_ref[live], rtol=1e-4, atol=2e-3)
    assert (got[~live] == 0).all()


def test_full_size_plans_are_among_the_forced_instances():
    """Host arithmetic only: the (wavefronts, single tile / loop) pair every benchmark configuration plans to
    is one of the pairs the forced tests above run at head dim 128, for both group sizes."""
    kk = U.kk()
    forced = {(wv, per <= wv * 32) for wv, per in FORCED}
    assert forced == {(4, True), (4, False), (8, True), (8, False)}
    for name in FULL:
        w = W.CONFIGS[name]
        nsplit, per, waves = kk.decode_plan(U.layout_of(w), w.budget + w.period)
        assert (waves, per <= waves * 32) in forced, (name, nsplit, per, waves)
        assert w.head_dim == 128 and w.group in (4, 8)
