"""GPU parity: keepkv_select, keepkv_match, keepkv_merge, stage by stage against the fp64 oracle
run on the GPU's own upstream state (indices and votes exact, merged K/V within 2e-3)."""
import numpy as np
import pytest
import torch

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _observed_cache(w, seed, n_pass, alpha, capacity=None, dup=False):
    """Cache after n_pass observation passes (decode_attn + score) on the GPU."""
    kk = U.kk()
    K, V = W.make_cache(w, seed)
    if dup:                                    # plant exact duplicates and near-duplicates of keys
        g = np.random.default_rng(seed)
        src = g.integers(0, w.context, size=(w.context // 8,))
        dst = g.integers(0, w.context, size=(w.context // 8,))
        K[:, :, dst] = K[:, :, src]
        K[:, :, dst[::3]] = W.round_storage(K[:, :, dst[::3]] * 1.5, w.dtype)   # same direction, other norm
    lay, c = U.new_cache(w, capacity=capacity or w.context, K=K, V=V)
    ws = U.workspace(lay, c.capacity, w.budget)
    logits = torch.zeros(w.batch, w.n_kv_heads, c.capacity, dtype=torch.float32, device="cuda")
    out = torch.zeros(w.batch, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    for t in range(n_pass):
        kk.decode_attn(lay, c, U.to_device(W.make_query(w, seed, t - n_pass), w.dtype), out, logits, None, ws)
        kk.score(lay, c, logits, alpha)
    torch.cuda.synchronize()
    return lay, c, ws


def _idx_buffers(w, capacity):
    B, H = w.batch, w.n_kv_heads
    keep = torch.full((B, H, w.budget), -7, dtype=torch.int32, device="cuda")
    evict = torch.full((B, H, capacity - w.budget), -7, dtype=torch.int32, device="cuda")
    n_ev = torch.full((B, H), -7, dtype=torch.int32, device="cuda")
    return keep, evict, n_ev


def _run_compress_stagewise(w, lay, c, ws, alpha, threshold, check_merge=True):
    """select -> match -> merge on the GPU; each stage checked against the oracle on GPU inputs."""
    kk = U.kk()
    B, H, cap = w.batch, w.n_kv_heads, c.capacity
    keep, evict, n_ev = _idx_buffers(w, cap)
    oc = U.download(c)
    kk.select(lay, c, w.budget, w.n_sink, w.n_recent, alpha, keep, evict, n_ev, ws)
    torch.cuda.synchronize()
    keep_h, evict_h, n_ev_h = keep.cpu().numpy(), evict.cpu().numpy(), n_ev.cpu().numpy()
    ref_sel = {}
    for b in range(B):
        for h in range(H):
            n = int(oc.len[b, h])
            rk, re = O.select(oc.log_S[b, h], oc.n_obs[b, h], oc.votes[b, h], n, w.budget, w.n_sink, w.n_recent, alpha)
            ref_sel[b, h] = (rk, re)
            assert n_ev_h[b, h] == len(re)
            np.testing.assert_array_equal(keep_h[b, h, :len(rk)], rk)
            assert (keep_h[b, h, len(rk):] == -1).all()
            np.testing.assert_array_equal(evict_h[b, h, :len(re)], re)
            assert (evict_h[b, h, len(re):] == -7).all()

    match = torch.full((B, H, cap - w.budget), -9, dtype=torch.int32, device="cuda")
    sim = torch.full((B, H, cap - w.budget), -9.0, dtype=torch.float32, device="cuda")
    kk.match(lay, c, w.budget, keep, evict, n_ev, threshold, match, sim, ws)
    # without the similarity output, rows whose best value is safely below the threshold skip the f64 re-check:
    # the targets must not depend on it
    match_nosim = torch.full_like(match, -9)
    kk.match(lay, c, w.budget, keep, evict, n_ev, threshold, match_nosim, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(match, match_nosim)
    match_h, sim_h = match.cpu().numpy(), sim.cpu().numpy()
    n_matched = 0
    for b in range(B):
        for h in range(H):
            rk, re = ref_sel[b, h]
            tgt, s = O.match(oc.k[b, h], rk, re, threshold, exact_any_order=(w.dtype == "bf16"))
            np.testing.assert_array_equal(match_h[b, h, :len(re)], tgt)
            assert (match_h[b, h, len(re):] == -9).all()
            if len(re):
                np.testing.assert_allclose(sim_h[b, h, :len(re)], s, rtol=0, atol=1e-4)
            n_matched += int((tgt >= 0).sum())

    if not check_merge:
        return n_matched
    lay2, d = U.new_cache(w, capacity=w.budget + w.period)
    d.k.fill_(float("nan")); d.v.fill_(float("nan"))
    dropped = torch.zeros(B, H, dtype=torch.int64, device="cuda")
    kk.merge(lay, c, d, w.budget, keep, evict, n_ev, match, alpha, dropped, ws)
    torch.cuda.synchronize()
    dk, dv = U.to_host(d.k), U.to_host(d.v)
    worst = 0.0
    for b in range(B):
        for h in range(H):
            rk, re = ref_sel[b, h]
            res = O.merge(oc.k[b, h], oc.v[b, h], oc.votes[b, h], oc.log_S[b, h], oc.n_obs[b, h], rk, re,
                          match_h[b, h, :len(re)], alpha)
            nk = len(rk)
            assert d.len[b, h].item() == nk
            np.testing.assert_array_equal(d.votes[b, h, :nk].cpu().numpy(), res.votes)
            np.testing.assert_array_equal(U.n_obs(d)[b, h, :nk].cpu().numpy(), res.n_obs)
            assert dropped[b, h].item() == res.dropped
            np.testing.assert_allclose(d.log_s[b, h, :nk].cpu().numpy(), res.log_S, rtol=2e-6, atol=2e-6)
            ev = U.storage_err_rows(dv[b, h, :nk], res.v, w.dtype)
            # keys: slots whose scale denominator is near the guard are ill-conditioned (reported, not gated)
            ek = U.storage_err_rows(dk[b, h, :nk], res.k, w.dtype)
            well = ~(np.abs(res.ell_bar) < 4 * O.ELL_GUARD)
            assert ev.max(initial=0) <= TOL, ("v", b, h, ev.max())
            assert ek[well].max(initial=0) <= TOL, ("k", b, h, ek[well].max())
            worst = max(worst, ek[well].max(initial=0), ev.max(initial=0))
            tg = match_h[b, h, :len(re)]
            has_members = np.zeros(nk, dtype=bool)
            has_members[tg[tg >= 0]] = True
            untouched = np.flatnonzero(~has_members)
            # slots that absorbed nothing are bit-exact copies
            np.testing.assert_array_equal(dk[b, h, untouched], oc.k[b, h, rk[untouched]].astype(np.float32))
    return n_matched


CASES = [
    ("tiny_f32", W.CONFIGS["tiny"], 0.8, False),
    ("tiny_f32_mergeall", W.CONFIGS["tiny"], -2.0, True),
    ("bf16_g4", W.CONFIGS["llama3_8b"].scaled(batch=2, context=1500), 0.8, True),
    ("bf16_g4_mergeall", W.CONFIGS["llama3_8b"].scaled(batch=2, context=1500), -2.0, False),
    ("bf16_mixture", W.CONFIGS["long_32k"].scaled(batch=1, context=5000), 0.8, True),
    ("bf16_ar1", W.CONFIGS["stress"].scaled(batch=2, context=3000, ratio=0.1), 0.3, False),
    ("bf16_d64", W.CONFIGS["llama3_8b"].scaled(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, context=777), 0.5, True),
]


@pytest.mark.parametrize("name,w,threshold,dup", CASES, ids=[c[0] for c in CASES])
def test_first_compression_event(name, w, threshold, dup):
    alpha = U.f32(w.alpha)
    lay, c, ws = _observed_cache(w, 0, 3, alpha, dup=dup)
    n = _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(threshold))
    if threshold < -1:
        assert n > 0


def test_ragged_heads_and_under_budget():
    """Heads with different live lengths, some at or under the budget (nothing to evict)."""
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=1, context=600, ratio=0.25)
    alpha = U.f32(0.9)
    lay, c, ws = _observed_cache(w, 3, 2, alpha)
    lens = np.array([[600, 150, 151, 149, 1, 0, 333, 599]], dtype=np.int32)
    c.len[:] = torch.from_numpy(lens).cuda()
    _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(-2.0))


def test_ragged_heads_with_several_match_passes():
    """40 heads (5 per XCD) whose evicted rows range from none to 8 blocks of 512: the first event's match
    workgroups (6 per head) take two passes on the full heads and none or a ragged one on the short ones."""
    w = W.CONFIGS["llama3_8b"].scaled(batch=5, context=4000)
    alpha = U.f32(0.9)
    lay, c, ws = _observed_cache(w, 5, 2, alpha)
    g = np.random.default_rng(5)
    lens = g.choice([4000, 3999, 2100, 913, 401, 400, 37], size=(5, 8)).astype(np.int32)
    lens[0, 0], lens[4, 7] = 4000, 4000
    c.len[:] = torch.from_numpy(lens).cuda()
    _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(0.6))


def test_select_exact_ties_keep_lowest_index():
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=1, context=900)
    alpha = U.f32(0.9)
    lay, c, ws = _observed_cache(w, 4, 1, alpha)
    g = np.random.default_rng(0)
    # coarse scores: thousands of exact ties across the selection boundary
    c.log_s[:] = torch.from_numpy(np.round(g.standard_normal((1, 8, 900)), 1).astype(np.float32)).cuda()
    U.set_n_obs(c, 5)
    c.votes[:] = torch.from_numpy(g.integers(1, 3, size=(1, 8, 900)).astype(np.int32)).cuda()
    _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(0.8), check_merge=False)


@pytest.mark.parametrize("context,budget_ratio", [(900, 0.1), (8192, 0.1), (2500, 0.5)])
def test_select_by_key_matches_oracle_and_feeds_match_and_merge(context, budget_ratio):
    """Caller-supplied ranking (an accumulated-attention heavy-hitter score here): index lists equal
    the oracle's bit for bit, ragged lengths, exact ties, NaN and infinities included, and the lists
    drive keepkv_match / keepkv_merge like those of keepkv_select."""
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=2, context=context, ratio=budget_ratio)
    alpha = U.f32(0.9)
    lay, c, ws = _observed_cache(w, 5, 2, alpha)
    B, H, cap = w.batch, w.n_kv_heads, c.capacity
    g = np.random.default_rng(context)
    lens = g.integers(w.budget + 1, context + 1, size=(B, H)).astype(np.int32)
    lens[0, 0], lens[0, 1], lens[1, 2] = context, w.budget, 3          # full, exactly at budget, nearly empty
    c.len[:] = torch.from_numpy(lens).cuda()
    # accumulated attention probabilities of 6 synthetic steps, coarsened so that many ranks tie
    rank = np.zeros((B, H, cap), dtype=np.float32)
    for t in range(6):
        x = g.standard_normal((B, H, cap)) * 3
        p = np.exp(x - x.max(-1, keepdims=True))
        rank += (p / p.sum(-1, keepdims=True)).astype(np.float32)
    rank = np.round(rank * 2000).astype(np.float32) / 2000
    rank[0, 3, g.integers(0, cap, 40)] = np.nan
    rank[1, 0, g.integers(0, cap, 40)] = -np.inf
    rank[1, 1, g.integers(0, cap, 5)] = np.inf
    keep, evict, n_ev = _idx_buffers(w, cap)
    kk.select_by_key(lay, c, torch.from_numpy(rank).cuda(), w.budget, w.n_sink, w.n_recent, keep, evict, n_ev, ws)
    torch.cuda.synchronize()
    keep_h, evict_h, n_ev_h = keep.cpu().numpy(), evict.cpu().numpy(), n_ev.cpu().numpy()
    for b in range(B):
        for h in range(H):
            n = int(lens[b, h])
            rk, re = O.select_by_key(rank[b, h], n, w.budget, w.n_sink, w.n_recent)
            assert n_ev_h[b, h] == len(re), (b, h)
            assert np.array_equal(keep_h[b, h, :len(rk)], rk), (b, h)
            assert (keep_h[b, h, len(rk):] == -1).all()
            assert np.array_equal(evict_h[b, h, :len(re)], re), (b, h)
    # the lists are ordinary select output: match and merge accept them and conserve the votes
    oc = U.download(c)
    m = torch.full((B, H, cap - w.budget), -7, dtype=torch.int32, device="cuda")
    kk.match(lay, c, w.budget, keep, evict, n_ev, U.f32(-2.0), m, None, ws)
    _, dst = U.new_cache(w, capacity=w.capacity)
    dropped = torch.zeros(B, H, dtype=torch.int64, device="cuda")
    kk.merge(lay, c, dst, w.budget, keep, evict, n_ev, m, alpha, dropped, ws)
    torch.cuda.synchronize()
    od = U.download(dst)
    for b in range(B):
        for h in range(H):
            n = int(lens[b, h])
            assert od.len[b, h] == min(n, w.budget)
            assert od.votes[b, h, :od.len[b, h]].sum() + int(dropped[b, h]) == oc.votes[b, h, :n].sum()


def test_maximum_sizes_and_limits():
    """The largest sizes match / merge accept: 4096 retained slots and 32768 evictable slots in one head."""
    kk = U.kk()
    N, Bud = 4096 + 32768, 4096
    w = W.CONFIGS["llama3_8b"].scaled(batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64, context=N,
                                      ratio=(Bud - 0.5) / N, period=16)
    assert w.budget == Bud and w.context - w.budget == 32768
    alpha = U.f32(w.alpha)
    lay, c, ws = _observed_cache(w, 7, 2, alpha)
    n = _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(0.3))
    assert n > 100                                             # plenty of merges at this threshold
    # one past either limit is refused before anything is launched
    keep = torch.zeros(1, 1, Bud + 1, dtype=torch.int32, device="cuda")
    evict = torch.zeros(1, 1, 40000, dtype=torch.int32, device="cuda")
    n_ev = torch.zeros(1, 1, dtype=torch.int32, device="cuda")
    m = torch.zeros_like(evict)
    lay2, big = U.new_cache(w, capacity=Bud + 1 + 32768)
    ws2 = U.workspace(lay2, big.capacity, Bud + 1)
    with pytest.raises(kk.KeepKVError) as e:
        kk.match(lay2, big, Bud + 1, keep, evict, n_ev, 0.5, m, None, ws2)
    assert e.value.status == kk.ERR_UNSUPPORTED
    lay3, big3 = U.new_cache(w, capacity=Bud + 32769)
    _, dst = U.new_cache(w, capacity=Bud + 16)
    ws3 = U.workspace(lay3, big3.capacity, Bud)
    with pytest.raises(kk.KeepKVError) as e:
        kk.merge(lay3, big3, dst, Bud, keep, evict, n_ev, m, alpha, None, ws3)
    assert e.value.status == kk.ERR_UNSUPPORTED


@pytest.mark.parametrize("alpha", [0.9, 0.0])
def test_degenerate_inputs(alpha):
    """Zero-norm keys (match nothing, are matched by nothing), never-observed slots (weight 0; groups with no
    observed member), log-scores at zero (the key-scale guard of the merge), identical keys (Lemma 4)."""
    w = W.CONFIGS["llama3_8b"].scaled(batch=1, context=700, ratio=0.2)
    alpha = U.f32(alpha)
    lay, c, ws = _observed_cache(w, 11, 2, alpha if alpha > 0 else U.f32(0.5))
    g = np.random.default_rng(3)
    N = w.context
    zero = g.choice(N, 60, replace=False)
    c.k[:, :, zero] = 0                                        # zero-norm keys on retained and evicted slots
    unobs = g.choice(N, 120, replace=False)
    c.log_s[:, :, unobs] = float("-inf")
    U.set_n_obs(c, 0, (slice(None), slice(None), unobs))
    c.log_s[0, 0] = torch.from_numpy((g.standard_normal(N) * 1e-3).astype(np.float32)).cuda()   # ln s_hat ~ 0: guarded
    U.set_n_obs(c, 50, (0, 0))
    c.log_s[0, 1, :] = float("-inf")                           # a head in which nothing was ever observed
    U.set_n_obs(c, 0, (0, 1))
    c.k[0, 2, 100:400] = c.k[0, 2, 100:101]                    # a run of identical keys
    c.votes[0, 3] = torch.from_numpy(g.integers(1, 1000, N).astype(np.int32)).cuda()
    _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(-2.0))
    _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(0.8))


def _digit_pattern_ranks(cap, seed):
    """Sixteen ranking arrays, each aimed at one branch of the radix select: digits in which no two keys
    differ, two heavily repeated values, mixed signs, zeros of both signs and denormals, values that differ
    only in their last mantissa bits, long tie runs across the selection boundary, infinities and NaN."""
    g = np.random.default_rng(seed)
    r = np.zeros((16, cap), dtype=np.float32)
    r[0] = 1.5
    r[1] = np.where(np.arange(cap) % 2 == 0, -2.0, 3.0)
    r[2] = g.standard_normal(cap) * 4
    r[3] = g.choice(np.array([0.0, -0.0, 1e-45, -1e-45, 3e-39, -3e-39, 1e-38], dtype=np.float32), cap)
    r[4] = (np.float32(1.0).view(np.uint32) + g.integers(0, 64, cap).astype(np.uint32)).view(np.float32)
    r[5] = g.integers(0, 16, cap)
    r[6] = -np.inf
    r[6, g.integers(0, cap, 30)] = g.standard_normal(30)
    r[7] = np.nan
    r[7, g.integers(0, cap, cap // 20)] = g.standard_normal(cap // 20)
    r[8] = g.standard_normal(cap)
    r[8, g.integers(0, cap, cap // 2)] = np.inf
    r[9] = np.arange(cap) * 0.25 - 100
    r[10] = -np.arange(cap) * 0.25 + 100
    r[11] = g.standard_normal(cap)
    r[11, cap // 4: cap // 4 + cap // 3] = 0.125                       # one long run of equal values
    r[12] = g.standard_normal(cap) * np.where(g.integers(0, 2, cap) == 0, 1e30, 1e-30)
    r[13] = -7.0
    r[13, cap // 2] = -6.5
    r[14] = np.where(g.integers(0, 2, cap) == 0, np.float32(1.0), np.nextafter(np.float32(1.0), np.float32(2.0)))
    r[15] = g.standard_normal(cap) - 9.0
    return r


@pytest.mark.parametrize("cap,budget,n_sink,n_recent", [
    (900, 90, 4, 16), (900, 20, 4, 16), (8192 + 37, 820, 4, 64), (8192 + 37, 4096, 0, 0), (20000, 700, 4, 64)])
def test_select_by_key_digit_patterns(cap, budget, n_sink, n_recent):
    """Index lists bit for bit those of the oracle for ranking values built to reach every branch of the
    radix select, at capacities with the keys in LDS and in the workspace, full and ragged lengths,
    and with no heavy-hitter positions at all (budget = sinks + recent)."""
    kk = U.kk()
    B, H = 2, 8
    lay = kk.Layout(B, 4 * H, H, 128, kk.BF16, 128 ** -0.5)
    c = kk.Cache(lay, cap)
    ws = kk.new_workspace(lay, cap, budget)
    rank = _digit_pattern_ranks(cap, cap + budget).reshape(B, H, cap)
    g = np.random.default_rng(budget)
    keep = torch.full((B, H, budget), -7, dtype=torch.int32, device="cuda")
    evict = torch.full((B, H, cap - budget), -7, dtype=torch.int32, device="cuda")
    n_ev = torch.full((B, H), -7, dtype=torch.int32, device="cuda")
    for lens in (np.full((B, H), cap, dtype=np.int32),
                 g.integers(budget + 1, cap + 1, size=(B, H)).astype(np.int32)):
        c.len[:] = torch.from_numpy(lens).cuda()
        kk.select_by_key(lay, c, torch.from_numpy(rank).cuda(), budget, n_sink, n_recent, keep, evict, n_ev, ws)
        torch.cuda.synchronize()
        keep_h, evict_h, n_ev_h = keep.cpu().numpy(), evict.cpu().numpy(), n_ev.cpu().numpy()
        for b in range(B):
            for h in range(H):
                n = int(lens[b, h])
                rk, re = O.select_by_key(rank[b, h], n, budget, n_sink, n_recent)
                assert n_ev_h[b, h] == len(re), (b, h)
                assert np.array_equal(keep_h[b, h, :len(rk)], rk), (b, h, n)
                assert np.array_equal(evict_h[b, h, :len(re)], re), (b, h, n)


@pytest.mark.parametrize("alpha", [0.9, 0.999, 0.5])
def test_select_skips_only_logarithms_that_are_zero(alpha):
    """The kernel evaluates ln p and ln(1 - alpha^n) only where they are not exactly zero.  Observation counts
    on both sides of the point where alpha^n drops below half an ulp of 1, slots never observed, and votes
    of one and of more than one, mixed within and across wavefronts: index lists equal the oracle's."""
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=2, context=3000)
    alpha = U.f32(alpha)
    lay, c = U.new_cache(w, capacity=3000)
    ws = U.workspace(lay, c.capacity, w.budget)
    B, H, n = w.batch, w.n_kv_heads, 3000
    g = np.random.default_rng(11)
    edge = int(40.0 / -np.log(alpha))
    n_obs = g.integers(max(1, edge - 40), edge + 40, size=(B, H, n)).astype(np.int32)
    n_obs[:, :, :1000] = (n - np.arange(1000)).astype(np.int32)        # old slots: the term vanishes (alpha 0.9, 0.5)
    n_obs[0, :, 1500:1600] = 0                                         # never observed
    votes = np.ones((B, H, n), dtype=np.int32)
    votes[:, :, 64:128] = g.integers(1, 9, size=(B, H, 64))            # one wavefront's worth with votes
    votes[1, :, ::5] = g.integers(2, 50, size=(H, 600))
    U.set_n_obs(c, n_obs)
    c.votes[:] = torch.from_numpy(votes).cuda()
    c.log_s[:] = torch.from_numpy((g.standard_normal((B, H, n)) * 3 - 8).astype(np.float32)).cuda()
    c.len[:] = n
    _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(0.8), check_merge=False)


def test_merge_groups_short_long_and_mixed():
    """keepkv_merge orders each target's members by counting when every group is short and with a sorting
    network when one is long.  Heads with exact copies of a retained key among the evicted keys (groups of
    one hundred, of a few hundred and of thousands of members) beside heads with ordinary short groups:
    every stage equals the oracle, so both orderings give the same ascending member lists."""
    w = W.CONFIGS["llama3_8b"].scaled(batch=2, context=6000, ratio=0.1)
    alpha = U.f32(0.9)
    K, V = W.make_cache(w, 21)
    g = np.random.default_rng(21)
    B, H, n = w.batch, w.n_kv_heads, w.context
    log_s = (g.standard_normal((B, H, n)) * 0.5 - 6).astype(np.float32)
    log_s[:, :, 100] = 0.0                                  # slot 100 is retained everywhere
    copies = {(0, 1): 100, (0, 2): 256, (0, 3): 257, (0, 5): 400, (1, 0): 3000, (1, 4): 5200}
    for (b, h), m in copies.items():
        K[b, h, 200:200 + m] = K[b, h, 100] * np.where(g.integers(0, 2, m) == 0, 1.0, 2.0)[:, None]
        log_s[b, h, 200:200 + m] = -30.0                    # all of them evicted
    lay, c = U.new_cache(w, capacity=n, K=K, V=V)
    ws = U.workspace(lay, c.capacity, w.budget)
    c.log_s[:] = torch.from_numpy(log_s).cuda()
    U.set_n_obs(c, 7)
    c.votes[:] = torch.from_numpy(g.integers(1, 4, size=(B, H, n)).astype(np.int32)).cuda()
    n_matched = _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(0.8))
    assert n_matched >= sum(copies.values())


@pytest.mark.parametrize("batch,period,budget_slots", [(1, 64, 820), (16, 64, 820), (17, 64, 820), (2, 200, 300), (4, 64, 40)])
def test_steady_state_match_shared_row_blocks(batch, period, budget_slots):
    """A period's worth of evictable slots per head.  With few heads up to four workgroups share the retained
    list of a 64-row block and join their per-row results through a ticket; with many heads a block has one
    workgroup.  8, 128 and 136 heads, several row blocks, a retained list shorter than the shares' column
    batches: every stage equals the oracle, twice in a row on the same workspace (the tickets return to zero)."""
    n = budget_slots + period
    w = W.CONFIGS["llama3_8b"].scaled(batch=batch, context=n, ratio=(budget_slots - 0.5) / n, period=period)
    assert w.budget == budget_slots
    alpha = U.f32(0.9)
    lay, c, ws = _observed_cache(w, 31 + batch, 2, alpha, dup=True)
    for rep in range(2):
        n_matched = _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(0.5), check_merge=(rep == 0 and batch <= 4))
    assert n_matched > 0
