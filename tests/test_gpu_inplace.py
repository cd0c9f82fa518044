"""GPU parity of the in-place steady-state event (keepkv_select_aged -> keepkv_match -> keepkv_merge_inplace):
every stage against the fp64 oracle on the GPU's own state brought into age order, and the whole cache, token by
token, bit for bit against the compacting event (keepkv_select -> keepkv_match -> keepkv_merge) over several
events with decode steps in between."""
import numpy as np
import pytest
import torch

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else (t.view(torch.int32) if t.dtype == torch.float32 else t)


def _age_index(order_h, lens, budget):
    """Per head: the live slots from the oldest token to the newest."""
    B, H = lens.shape
    return [[np.concatenate([order_h[b, h, :min(int(lens[b, h]), budget)],
                             np.arange(budget, max(int(lens[b, h]), budget))]).astype(np.int64)
             for h in range(H)] for b in range(B)]


def _gather(oc, idx, b, h):
    """The head's oracle-side state in age order."""
    i = idx[b][h]
    return oc.k[b, h, i], oc.v[b, h, i], oc.votes[b, h, i], oc.log_S[b, h, i], oc.n_obs[b, h, i]


def _setup(w, seed, dup, lens=None):
    from tests.test_gpu_compress import _observed_cache
    alpha = U.f32(w.alpha)
    lay, c, ws = _observed_cache(w, seed, 2, alpha, dup=dup)
    if lens is not None:
        c.len[:] = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    return lay, c, ws, alpha


def _clone_cache(lay, c):
    kk = U.kk()
    d = kk.Cache(lay, c.capacity)
    for name in ("k", "v", "votes", "log_s", "born", "t_obs", "len"):
        getattr(d, name).copy_(getattr(c, name))
    return d


CASES = [
    ("bf16_g4_T0.5", W.CONFIGS["llama3_8b"].scaled(batch=2, context=820 + 64, ratio=819.5 / 884, period=64), 0.5, None),
    ("bf16_g4_mergeall", W.CONFIGS["llama3_8b"].scaled(batch=1, context=300 + 200, ratio=299.5 / 500, period=200), -2.0, None),
    ("bf16_d64", W.CONFIGS["llama3_8b"].scaled(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, context=100 + 32, ratio=99.5 / 132,
                                              period=32), 0.3, None),
    ("f32_tiny", W.CONFIGS["tiny"].scaled(batch=2, context=52 + 32, ratio=51.5 / 84, period=32), 0.2, None),
    ("bf16_ragged", W.CONFIGS["llama3_8b"].scaled(batch=1, context=200 + 48, ratio=199.5 / 248, period=48), 0.4,
     [[248, 200, 201, 150, 0, 247, 1, 248]]),
    # no evicted slot finds a target: every one is dropped, the retained tokens of the append region still move
    ("bf16_nomatch", W.CONFIGS["llama3_8b"].scaled(batch=1, context=120 + 40, ratio=119.5 / 160, period=40), 2.0, None),
]


@pytest.mark.parametrize("name,w,threshold,lens", CASES, ids=[c[0] for c in CASES])
def test_inplace_event_matches_oracle_and_compacting_event(name, w, threshold, lens):
    kk = U.kk()
    T = U.f32(threshold)
    B, H, Bud, P = w.batch, w.n_kv_heads, w.budget, w.period
    cap = Bud + P
    assert w.context == cap
    lay, cb, ws, alpha = _setup(w, 11, True, lens)       # in place
    ca = _clone_cache(lay, cb)                           # the same state for the compacting path
    lay2, ca2 = U.new_cache(w, capacity=cap)
    order = torch.arange(Bud, dtype=torch.int32, device="cuda").repeat(B, H, 1).contiguous()
    z = lambda *s, dt=torch.int32, fill=-7: torch.full(s, fill, dtype=dt, device="cuda")
    out = torch.zeros(B, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    n_merged_total, n_moved_total = 0, 0
    step = 0
    for event in range(3):
        keep_a, evict_a, nev_a, match_a = z(B, H, Bud), z(B, H, P), z(B, H), z(B, H, P, fill=-9)
        keep_b, evict_b, nev_b, match_b = z(B, H, Bud), z(B, H, P), z(B, H), z(B, H, P, fill=-9)
        drop_a, drop_b = z(B, H, dt=torch.int64, fill=0), z(B, H, dt=torch.int64, fill=0)
        # ---- the GPU's state before the event, in age order, for the oracle
        torch.cuda.synchronize()
        oc = U.download(cb)
        order_h = order.cpu().numpy()
        lens_h = cb.len.cpu().numpy()
        idx = _age_index(order_h, lens_h, Bud)
        # ---- select
        kk.select_aged(lay, cb, order, Bud, w.n_sink, w.n_recent, alpha, keep_b, evict_b, nev_b, ws)
        kk.select(lay, ca, Bud, w.n_sink, w.n_recent, alpha, keep_a, evict_a, nev_a, ws)
        torch.cuda.synchronize()
        keep_h, evict_h, nev_h = keep_b.cpu().numpy(), evict_b.cpu().numpy(), nev_b.cpu().numpy()
        ref = {}
        for b in range(B):
            for h in range(H):
                k_, v_, p_, ls_, n_ = _gather(oc, idx, b, h)
                n = int(lens_h[b, h])
                rk, re = O.select(ls_, n_, p_, n, Bud, w.n_sink, w.n_recent, alpha)
                ref[b, h] = (rk, re)
                assert nev_h[b, h] == len(re)
                np.testing.assert_array_equal(keep_h[b, h, :len(rk)], idx[b][h][rk], err_msg=f"{name} keep {event} {b},{h}")
                assert (keep_h[b, h, len(rk):] == -1).all()
                np.testing.assert_array_equal(evict_h[b, h, :len(re)], idx[b][h][re])
        assert torch.equal(nev_a, nev_b)
        # ---- match (positions in the keep list: the same numbers on both paths)
        kk.match(lay, cb, Bud, keep_b, evict_b, nev_b, T, match_b, None, ws)
        kk.match(lay, ca, Bud, keep_a, evict_a, nev_a, T, match_a, None, ws)
        torch.cuda.synchronize()
        match_h = match_b.cpu().numpy()
        for b in range(B):
            for h in range(H):
                rk, re = ref[b, h]
                tgt, _ = O.match(_gather(oc, idx, b, h)[0], rk, re, T, exact_any_order=(w.dtype == "bf16"))
                np.testing.assert_array_equal(match_h[b, h, :len(re)], tgt, err_msg=f"{name} match {event} {b},{h}")
                np.testing.assert_array_equal(match_a[b, h, :len(re)].cpu().numpy(), tgt)
        # ---- merge
        kk.merge_inplace(lay, cb, order, Bud, keep_b, evict_b, nev_b, match_b, alpha, drop_b)
        kk.merge(lay, ca, ca2, Bud, keep_a, evict_a, nev_a, match_a, alpha, drop_a, ws)
        torch.cuda.synchronize()
        new_order = order.cpu().numpy()
        kb, vb = U.to_host(cb.k), U.to_host(cb.v)
        for b in range(B):
            for h in range(H):
                rk, re = ref[b, h]
                n = int(lens_h[b, h])
                nk = len(rk)
                assert cb.len[b, h].item() == nk and ca2.len[b, h].item() == nk
                if len(re) == 0:                          # nothing evicted: the head is left as it is
                    np.testing.assert_array_equal(new_order[b, h], order_h[b, h])
                    continue
                assert sorted(new_order[b, h].tolist()) == list(range(Bud))        # a permutation of the slots below budget
                k_, v_, p_, ls_, n_ = _gather(oc, idx, b, h)
                tg = match_h[b, h, :len(re)]
                res = O.merge(k_, v_, p_, ls_, n_, rk, re, tg, alpha)
                s = new_order[b, h].astype(np.int64)                               # retained tokens, oldest first
                np.testing.assert_array_equal(cb.votes[b, h].cpu().numpy()[s], res.votes)
                np.testing.assert_array_equal(U.n_obs(cb)[b, h].cpu().numpy()[s], res.n_obs)
                assert drop_b[b, h].item() == res.dropped
                np.testing.assert_allclose(cb.log_s[b, h].cpu().numpy()[s], res.log_S, rtol=2e-6, atol=2e-6)
                ev = U.storage_err_rows(vb[b, h][s], res.v, w.dtype)
                ek = U.storage_err_rows(kb[b, h][s], res.k, w.dtype)
                well = ~(np.abs(res.ell_bar) < 4 * O.ELL_GUARD)
                assert ev.max(initial=0) <= TOL and ek[well].max(initial=0) <= TOL, (name, event, b, h)
                has = np.zeros(nk, dtype=bool)
                has[tg[tg >= 0]] = True
                np.testing.assert_array_equal(kb[b, h][s][~has], k_[rk[~has]].astype(np.float32))   # untouched or moved: exact copies
                n_merged_total += int(has.sum())
                n_moved_total += int((idx[b][h][rk] >= Bud).sum())
                # a retained token below budget that absorbed nothing has not moved
                stay = (idx[b][h][rk] < Bud)
                np.testing.assert_array_equal(s[stay], idx[b][h][rk][stay])
        # ---- the compacting path holds the same tokens in age order, bit for bit
        g = order.long()
        for name_, exact in (("k", True), ("v", True), ("votes", True), ("log_s", True), ("born", True)):
            a = getattr(ca2, name_)[:, :, :Bud]
            bb = getattr(cb, name_)
            gi = g if bb.dim() == 3 else g.unsqueeze(-1).expand(-1, -1, -1, bb.shape[-1])
            got = torch.gather(bb, 2, gi)
            live = (torch.arange(Bud, device="cuda")[None, None] < cb.len.unsqueeze(-1))
            live = live if bb.dim() == 3 else live.unsqueeze(-1)
            assert torch.equal(torch.where(live, _bits(a), torch.zeros_like(_bits(a))),
                               torch.where(live, _bits(got), torch.zeros_like(_bits(got)))), (name, event, name_)
        assert torch.equal(drop_a, drop_b) and torch.equal(ca2.len, cb.len) and torch.equal(ca2.t_obs, cb.t_obs)
        ca, ca2 = ca2, ca
        # ---- a period of decode steps on both
        for _ in range(P if lens is None else P // 2):
            q = U.to_device(W.make_query(w, 11, step), w.dtype)
            kt, vt = (U.to_device(x, w.dtype) for x in W.make_token(w, 11, step))
            kk.decode_step(lay, cb, q, kt, vt, out, None, alpha, None, ws)
            kk.decode_step(lay, ca, q, kt, vt, out, None, alpha, None, ws)
            step += 1
    assert (n_merged_total > 0 or threshold > 1.0) and n_moved_total > 0, "the case exercises no merge or no move"


def test_inplace_refusals():
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=1, context=820 + 300, ratio=819.5 / 1120, period=300)
    lay, c = U.new_cache(w, capacity=1120)
    order = torch.arange(w.budget, dtype=torch.int32, device="cuda").repeat(1, 8, 1).contiguous()
    keep = torch.zeros(1, 8, w.budget, dtype=torch.int32, device="cuda")
    ev = torch.zeros(1, 8, 300, dtype=torch.int32, device="cuda")
    nev = torch.zeros(1, 8, dtype=torch.int32, device="cuda")
    with pytest.raises(kk.KeepKVError) as e:             # more than 256 evictable slots: the compacting merge is the one to use
        kk.merge_inplace(lay, c, order, w.budget, keep, ev, nev, ev, 0.9, None)
    assert e.value.status == kk.ERR_UNSUPPORTED
    with pytest.raises(kk.KeepKVError) as e:
        kk.merge_inplace(lay, c, None, w.budget, keep, ev, nev, ev, 0.9, None)
    assert e.value.status == kk.ERR_INVALID_ARG
    torch.cuda.synchronize()


def test_inplace_event_in_a_graph_replays_like_eager():
    """A decode step and an in-place event captured in one HIP graph and replayed several times, with eager work
    and synchronisation between the replays, leave the cache, the slot list and the index lists as the eager
    sequence does, every time."""
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=2, context=300 + 64, ratio=299.5 / 364, period=64)
    T = U.f32(0.4)
    B, H, Bud, P = w.batch, w.n_kv_heads, w.budget, w.period
    lay, c, ws, alpha = _setup(w, 5, True)
    c.len.fill_(Bud + P - 1)                              # the step below fills the cache
    order = torch.arange(Bud, dtype=torch.int32, device="cuda").flip(0).repeat(B, H, 1).contiguous()   # (any permutation)
    keep = torch.zeros(B, H, Bud, dtype=torch.int32, device="cuda")
    evict, match = (torch.zeros(B, H, P, dtype=torch.int32, device="cuda") for _ in range(2))
    nev = torch.zeros(B, H, dtype=torch.int32, device="cuda")
    drop = torch.zeros(B, H, dtype=torch.int64, device="cuda")
    out = torch.zeros(B, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    q = U.to_device(W.make_query(w, 5, 0), w.dtype)
    kt, vt = (U.to_device(x, w.dtype) for x in W.make_token(w, 5, 0))
    fields = ("k", "v", "votes", "log_s", "born", "t_obs", "len")
    start = {f: getattr(c, f).clone() for f in fields}
    order0 = order.clone()

    def restore():
        for f in fields:
            getattr(c, f).copy_(start[f])
        order.copy_(order0)
        drop.zero_()

    def body():
        kk.decode_step(lay, c, q, kt, vt, out, None, alpha, None, ws)
        kk.select_aged(lay, c, order, Bud, w.n_sink, w.n_recent, alpha, keep, evict, nev, ws)
        kk.match(lay, c, Bud, keep, evict, nev, T, match, None, ws)
        kk.merge_inplace(lay, c, order, Bud, keep, evict, nev, match, alpha, drop)

    def snapshot():
        live = [getattr(c, f)[:, :, :Bud] if getattr(c, f).dim() >= 3 else getattr(c, f) for f in fields]
        return [_bits(x).clone() for x in (out, order, keep, evict, match, nev, drop, *live)]

    body()
    torch.cuda.synchronize()
    ref = snapshot()
    assert (c.len == Bud).all() and int((match >= 0).sum()) > 0
    restore()
    torch.cuda.synchronize()
    graph, stream = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=stream):
        body()
    for rep in range(3):
        restore()
        keep.fill_(-3); match.fill_(-3); out.zero_()       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(snapshot(), ref)):
            assert torch.equal(a, b), (rep, i)


def test_inplace_event_at_full_batch_128():
    """The batch-128 share of the Llama-3-70B shape (1024 heads, 820 + 64 slots): the configuration in which bench.py
    runs its events in place.  Two events with a period of decode steps between them; after each, every head of
    the in-place cache read through its slot list equals the compacting path's cache bit for bit, and sampled
    heads are compared with the oracle stage by stage."""
    from types import SimpleNamespace
    kk = U.kk()
    w = W.CONFIGS["llama3_70b"].scaled(context=820 + 64, ratio=819.5 / 884)
    T = U.f32(w.threshold)
    B, H, Bud, P = w.batch, w.n_kv_heads, w.budget, w.period
    assert (B, H, Bud, P) == (128, 8, 820, 64)
    cap = Bud + P
    lay, cb, ws, alpha = _setup(w, 2, False)
    ca = _clone_cache(lay, cb)
    lay2, ca2 = U.new_cache(w, capacity=cap)
    order = torch.arange(Bud, dtype=torch.int32, device="cuda").repeat(B, H, 1).contiguous()
    z = lambda *s, dt=torch.int32, fill=-7: torch.full(s, fill, dtype=dt, device="cuda")
    out = torch.zeros(B, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    sample = [(0, 0), (37, 5), (127, 7)]
    step = 0
    for event in range(2):
        keep_a, evict_a, nev_a, match_a = z(B, H, Bud), z(B, H, P), z(B, H), z(B, H, P, fill=-9)
        keep_b, evict_b, nev_b, match_b = z(B, H, Bud), z(B, H, P), z(B, H), z(B, H, P, fill=-9)
        drop_a, drop_b = z(B, H, dt=torch.int64, fill=0), z(B, H, dt=torch.int64, fill=0)
        torch.cuda.synchronize()
        before = {}
        for (b, h) in sample:                               # the sampled heads' state before the event, for the oracle
            view = SimpleNamespace(**{f: getattr(cb, f)[b:b + 1, h:h + 1].clone() for f in ("k", "v", "votes", "log_s", "born", "t_obs", "len")})
            before[b, h] = (U.download(view), order[b, h].cpu().numpy().astype(np.int64))
        kk.select_aged(lay, cb, order, Bud, w.n_sink, w.n_recent, alpha, keep_b, evict_b, nev_b, ws)
        kk.match(lay, cb, Bud, keep_b, evict_b, nev_b, T, match_b, None, ws)
        kk.merge_inplace(lay, cb, order, Bud, keep_b, evict_b, nev_b, match_b, alpha, drop_b)
        kk.select(lay, ca, Bud, w.n_sink, w.n_recent, alpha, keep_a, evict_a, nev_a, ws)
        kk.match(lay, ca, Bud, keep_a, evict_a, nev_a, T, match_a, None, ws)
        kk.merge(lay, ca, ca2, Bud, keep_a, evict_a, nev_a, match_a, alpha, drop_a, ws)
        torch.cuda.synchronize()
        assert torch.equal(match_a, match_b) and torch.equal(nev_a, nev_b) and torch.equal(drop_a, drop_b)
        assert (cb.len == Bud).all() and torch.equal(ca2.len, cb.len) and torch.equal(ca2.t_obs, cb.t_obs)
        assert torch.equal(order.sort(dim=-1).values, torch.arange(Bud, dtype=torch.int32, device="cuda").expand(B, H, Bud))
        g = order.long()
        for f in ("k", "v", "votes", "log_s", "born"):
            a, bb = getattr(ca2, f)[:, :, :Bud], getattr(cb, f)
            gi = g if bb.dim() == 3 else g.unsqueeze(-1).expand(-1, -1, -1, bb.shape[-1])
            assert torch.equal(_bits(a), _bits(torch.gather(bb, 2, gi))), (event, f)
        n_merged = 0
        for (b, h) in sample:
            oc, ordr = before[b, h]
            idx = np.concatenate([ordr, np.arange(Bud, cap)])
            k_, v_, p_, ls_, n_ = oc.k[0, 0, idx], oc.v[0, 0, idx], oc.votes[0, 0, idx], oc.log_S[0, 0, idx], oc.n_obs[0, 0, idx]
            rk, re = O.select(ls_, n_, p_, cap, Bud, w.n_sink, w.n_recent, alpha)
            np.testing.assert_array_equal(keep_b[b, h].cpu().numpy(), idx[rk])
            np.testing.assert_array_equal(evict_b[b, h].cpu().numpy(), idx[re])
            tgt, _ = O.match(k_, rk, re, T, exact_any_order=True)
            np.testing.assert_array_equal(match_b[b, h].cpu().numpy(), tgt)
            res = O.merge(k_, v_, p_, ls_, n_, rk, re, tgt, alpha)
            s = order[b, h].cpu().numpy().astype(np.int64)
            np.testing.assert_array_equal(cb.votes[b, h].cpu().numpy()[s], res.votes)
            np.testing.assert_array_equal(U.n_obs(cb)[b, h].cpu().numpy()[s], res.n_obs)
            assert drop_b[b, h].item() == res.dropped
            np.testing.assert_allclose(cb.log_s[b, h].cpu().numpy()[s], res.log_S, rtol=2e-6, atol=2e-6)
            ev = U.storage_err_rows(U.to_host(cb.v[b, h])[s], res.v, w.dtype)
            ek = U.storage_err_rows(U.to_host(cb.k[b, h])[s], res.k, w.dtype)
            well = ~(np.abs(res.ell_bar) < 4 * O.ELL_GUARD)
            assert ev.max(initial=0) <= TOL and ek[well].max(initial=0) <= TOL, (event, b, h)
            n_merged += int((tgt >= 0).sum())
        assert n_merged > 0
        ca, ca2 = ca2, ca
        for _ in range(P):
            q = U.to_device(W.make_query(w, 2, step), w.dtype)
            kt, vt = (U.to_device(x, w.dtype) for x in W.make_token(w, 2, step))
            kk.decode_step(lay, cb, q, kt, vt, out, None, alpha, None, ws)
            kk.decode_step(lay, ca, q, kt, vt, out, None, alpha, None, ws)
            step += 1
