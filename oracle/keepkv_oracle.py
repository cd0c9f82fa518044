"""CPU oracle of the KeepKV hot path (arXiv 2504.09936) -- TEST INFRASTRUCTURE ONLY.

Plain numpy, float64, one (batch, kv-head) cache at a time, no blocking or fusion.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
file; the product path never does, and this file imports nothing from the product.

Notation follows the paper (Sec. 3.1): for one head with head dimension d,
    logit_i = q . k_i / sqrt(d),      s_i = exp(logit_i)      (unnormalised score, Eq. 3)
    p_i     = Electoral Votes of slot i (Sec. 3.3.1, initialised to 1)
    S_i     = exponential moving average of s_i, s_hat_i its bias-corrected value (Eq. 8)
    K_e / K_c = to-be-evicted / retained slots (Alg. 1)
All scores are carried as natural logarithms (log s, log S, log s_hat).

Readings taken where the paper is silent (each is restated at the function it affects):
  * scores are the unnormalised exp(logit), as Eq. 3 defines s;
  * with grouped-query attention the score of a slot is that of the group's mean
    query, i.e. the mean logit over the query heads sharing the kv head;
  * bias correction uses the slot's own observation count n_i: s_hat = S / (1 - alpha^n_i);
  * several evicted slots matched to one retained slot are merged in one multi-way
    ZIP merge (App. A.3 form), not by repeated pairwise merges;
  * an evicted slot with no retained key above the threshold is dropped (plain
    eviction, Eq. 4) and its votes are added to a per-head `dropped` counter;
  * the merged key's scale ln(W/P) / (sum w ln s / W) is replaced by 1 when the
    denominator's magnitude is below `ELL_GUARD` (the formula is singular there);
  * merge-first prefill (App. B.4 gives the order, no algorithm): every slot links to its most
    similar earlier key if above the threshold; a linked slot is absorbed by its target unless
    the target is itself absorbed; each receiving slot and the slots it absorbs are merged in one
    multi-way ZIP merge; the eviction strategy then runs on the shorter cache.

Parity pins (tests/test_oracle_*.py): textbook softmax attention and vote duplication
(decode_attn); closed-form EMA sums (score_update); brute-force sort / cosine matrix
(select, match); Theorem 2, Lemma 4, the pairwise Eq. 7 and vote / mass conservation
(merge); Theorem 3 (perturbation_bound); brute force, Theorem 2, vote conservation and the
duplicate-key case of Lemma 4 (merge-first prefill).  The guard branch of `merge` has no pin in
the paper: parity unpinned for guarded slots.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

ELL_GUARD = 1.0e-3   # |sum w ln s / W| below this: merged key is the plain weighted mean


# --------------------------------------------------------------------------- attention (Eq. 6)
def decode_attn(q, k, v, votes, length, scale):
    """Vote-weighted attention of one kv head's query group over its cache (Eq. 6).

    q [G, d]; k, v [cap, d]; votes [cap] int; live slots are [0, length).
    Returns (o [G, d], lse [G], mean_logit [length]) where
      o_h   = sum_i p_i s_i^h v_i / sum_i p_i s_i^h,      s_i^h = exp(scale * q_h . k_i)
      lse_h = ln sum_i p_i s_i^h
      mean_logit_i = (1/G) sum_h scale * q_h . k_i   (log-score of the group-mean query).
    An empty cache gives o = 0, lse = -inf.
    """
    q = np.asarray(q, dtype=np.float64)
    G, d = q.shape
    if length == 0:
        return np.zeros((G, d)), np.full(G, -np.inf), np.zeros(0)
    kk = np.asarray(k[:length], dtype=np.float64)
    vv = np.asarray(v[:length], dtype=np.float64)
    p = np.asarray(votes[:length], dtype=np.float64)
    logit = scale * (q @ kk.T)                       # [G, S]  ln s_i^h
    z = logit + np.log(p)[None, :]                   # ln (p_i s_i^h)
    m = z.max(axis=1)
    e = np.exp(z - m[:, None])
    den = e.sum(axis=1)
    o = (e @ vv) / den[:, None]
    lse = m + np.log(den)
    return o, lse, logit.mean(axis=0)


# --------------------------------------------------------------------------- EMA scores (Eq. 8)
def score_update(log_S, n_obs, mean_logit, length, alpha):
    """One EMA step S <- alpha S + (1 - alpha) s for the live slots (Eq. 8, t > L branch).

    log_S [cap] holds ln S (-inf where nothing was observed yet), n_obs [cap] the number
    of observations folded in.  s = exp(mean_logit).  Returns new (log_S, n_obs) copies.
    Running this from S = 0 over w + 1 queries reproduces the t = L window sum of Eq. 8.
    """
    log_S = np.array(log_S, dtype=np.float64)
    n_obs = np.array(n_obs, dtype=np.int64)
    x = np.asarray(mean_logit, dtype=np.float64)[:length]
    if alpha == 0.0:
        new = x.copy()
    else:
        with np.errstate(divide="ignore"):
            new = np.logaddexp(math.log(alpha) + log_S[:length], math.log1p(-alpha) + x)
    log_S[:length] = new
    n_obs[:length] += 1
    return log_S, n_obs


def window_score(log_S, n_obs, q_win, k, length, scale, alpha, first_pos=-1):
    """EMA scores from a window of W queries at once (Eq. 8, t = L branch, written as the sum).

    q_win [W, G, d]: the window's queries of one kv head's group, oldest first; k [cap, d].
    s_{j,i} = exp(mean over the group of scale * q_{j,g} . k_i).  With first_pos >= 0 query j
    sits at sequence position first_pos + j and sees slot i only if i <= first_pos + j
    (causal prefill); with first_pos < 0 every live slot is visible to every query.  For a slot
    seen by the last n_i of the W queries,
        S_i <- alpha^{n_i} S_i + sum_{j >= W - n_i} (1 - alpha) alpha^{W-1-j} s_{j,i},  n_obs_i += n_i
    which from the empty state (S = 0, n = 0) is the window sum of Eq. 8.
    Returns new (log_S, n_obs) copies.
    """
    log_S = np.array(log_S, dtype=np.float64)
    n_obs = np.array(n_obs, dtype=np.int64)
    q = np.asarray(q_win, dtype=np.float64)
    W = q.shape[0]
    kk = np.asarray(k[:length], dtype=np.float64)
    x = scale * np.einsum("jgd,id->jgi", q, kk).mean(axis=1)                 # [W, length]  ln s_{j,i}
    j = np.arange(W)[:, None]
    i = np.arange(length)[None, :]
    vis = np.ones((W, length), dtype=bool) if first_pos < 0 else (i <= first_pos + j)
    n_vis = vis.sum(axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        if alpha == 0.0:
            coef = np.where(j == W - 1, 0.0, -np.inf)                        # only the last query counts
            old = np.where(n_vis > 0, -np.inf, log_S[:length])
        else:
            coef = math.log1p(-alpha) + (W - 1 - j) * math.log(alpha)
            old = log_S[:length] + n_vis * math.log(alpha)
        terms = np.where(vis, x + coef, -np.inf)
        new = np.logaddexp(old, np.logaddexp.reduce(terms, axis=0))
    upd = n_vis > 0
    log_S[:length][upd] = new[upd]
    n_obs[:length] += n_vis
    return log_S, n_obs


def log_s_hat(log_S, n_obs, alpha):
    """ln s_hat = ln S - ln(1 - alpha^n): bias-corrected EMA score (Eq. 8), per-slot count n.

    Slots never observed (n = 0) have s_hat = 0, i.e. ln s_hat = -inf.
    """
    log_S = np.asarray(log_S, dtype=np.float64)
    n = np.asarray(n_obs, dtype=np.float64)
    out = np.full(log_S.shape, -np.inf)
    seen = n > 0
    if alpha == 0.0:
        out[seen] = log_S[seen]
    else:
        out[seen] = log_S[seen] - np.log(-np.expm1(n[seen] * math.log(alpha)))
    return out


# --------------------------------------------------------------------------- selection (Alg. 1, selection step)
def select_by_key(rank, length, budget, n_sink, n_recent):
    """Split the live slots into retained and to-be-evicted sets under any ranking value.

    The method leaves the selection strategy open (Sec. 3.3.2, last paragraph; Sec. 4.4 combines
    it with other eviction methods): slots [0, n_sink) and [length - n_recent, length) are
    always kept; of the others the budget - n_sink - n_recent with the largest rank are kept,
    equal ranks resolved in favour of the lower index, NaN below every number.
    Returns (keep_idx ascending, evict_idx ascending) as int64 arrays.
    """
    if length <= budget:
        return np.arange(length, dtype=np.int64), np.zeros(0, dtype=np.int64)
    if n_sink + n_recent > budget:
        raise ValueError("n_sink + n_recent exceeds the budget")
    key = np.asarray(rank[:length], dtype=np.float64).copy()
    key[np.isnan(key)] = -np.inf
    protected = np.zeros(length, dtype=bool)
    protected[:n_sink] = True
    protected[length - n_recent:] = True
    cand = np.flatnonzero(~protected)
    n_heavy = budget - int(protected.sum())
    order = cand[np.lexsort((cand, -key[cand]))]                # rank descending, then index ascending
    keep = protected.copy()
    keep[order[:n_heavy]] = True
    return np.flatnonzero(keep).astype(np.int64), np.flatnonzero(~keep).astype(np.int64)


def select(log_S, n_obs, votes, length, budget, n_sink, n_recent, alpha):
    """Split the live slots into retained K_c and to-be-evicted K_e (Alg. 1, selection step).

    Policy (fixed budget, sink tokens, recent window, heavy hitters -- App. B.3) with the
    vote-weighted EMA mass ln p_i + ln s_hat_i as the ranking value of select_by_key.
    """
    if length <= budget:
        return np.arange(length, dtype=np.int64), np.zeros(0, dtype=np.int64)
    key = np.log(np.asarray(votes[:length], dtype=np.float64)) + log_s_hat(log_S[:length], n_obs[:length], alpha)
    return select_by_key(key, length, budget, n_sink, n_recent)


# --------------------------------------------------------------------------- matching (Alg. 1, matching step)
def _dots(a, b, exact_any_order):
    """a [m, d] . b [n, d] -> [m, n] in float64.

    For bfloat16-representable inputs every product has at most 16 significant bits and
    the d-term sum is exact in float64, so a library matmul gives the same bits in any
    order.  Otherwise the sum is taken channel by channel in index order, so that equal
    rows give equal results whatever their position.
    """
    if exact_any_order:
        return a @ b.T
    acc = np.zeros((a.shape[0], b.shape[0]))
    for c in range(a.shape[1]):
        acc += a[:, c, None] * b[None, :, c]
    return acc


def match(k, keep_idx, evict_idx, threshold, exact_any_order=False):
    """Merge target of every to-be-evicted key (Alg. 1, matching step).

    U[e, c] = cos(k_e, k_c) = (k_e . k_c) * (1/|k_e|) * (1/|k_c|); the target of e is the
    first maximiser of U[e, :] over the retained keys; it is used only if U > threshold
    (strict).  Returns (target [m] = position in keep_idx or -1, sim [m] = max_c U[e, c]).
    """
    k = np.asarray(k, dtype=np.float64)
    ke, kc = k[np.asarray(evict_idx, dtype=np.int64)], k[np.asarray(keep_idx, dtype=np.int64)]
    m = ke.shape[0]
    if m == 0 or kc.shape[0] == 0:
        return np.full(m, -1, dtype=np.int64), np.full(m, -np.inf)
    with np.errstate(divide="ignore", invalid="ignore"):
        rn_e = 1.0 / np.sqrt(_dots_self(ke))
        rn_c = 1.0 / np.sqrt(_dots_self(kc))
        U = (_dots(ke, kc, exact_any_order) * rn_e[:, None]) * rn_c[None, :]
    U = np.where(np.isfinite(U), U, -np.inf)          # zero-norm keys match nothing
    best = U.argmax(axis=1)                           # numpy returns the first maximiser
    sim = U[np.arange(m), best]
    target = np.where(sim > threshold, best, -1).astype(np.int64)
    return target, sim


def _dots_self(a):
    acc = np.zeros(a.shape[0])
    for c in range(a.shape[1]):
        acc += a[:, c] * a[:, c]
    return acc


# --------------------------------------------------------------------------- ZIP-Merging (Eq. 7)
@dataclass
class MergeResult:
    k: np.ndarray          # [budget', d] merged keys, keep_idx order
    v: np.ndarray
    votes: np.ndarray      # int64
    log_S: np.ndarray
    n_obs: np.ndarray      # int64
    dropped: int           # votes of evicted slots that found no target
    guarded: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=bool))
    ell_bar: np.ndarray = field(default_factory=lambda: np.zeros(0))


def merge(k, v, votes, log_S, n_obs, keep_idx, evict_idx, target, alpha):
    """Multi-way Zero Inference-Perturbation Merging with EMA scores (App. A.3 / A.4 form
    of Eq. 7; Alg. 1, merging step).

    For retained slot c with group g = {c} + {e : target[e] = c}, E_i = ln s_hat_i,
    w_i = p_i s_hat_i, W = sum w, P = sum p:
        v_r = sum w_i v_i / W
        k_r = (sum w_i k_i / W) * ln(W / P) / (sum w_i E_i / W)
        p_r = P,  ln s_hat_r = ln(W / P)   (so that p_r s_hat_r = sum p_i s_hat_i)
    The merged slot keeps the retained slot's observation count, n_r = max(n_c, 1), hence
    ln S_r = ln s_hat_r + ln(1 - alpha^n_r).  Slots whose group is {c} alone are copied.
    Members never observed (s_hat = 0) have weight 0; a group with no observed member is
    merged with weights p_i / P and stays unobserved.  Output rows follow keep_idx order.
    """
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    keep_idx = np.asarray(keep_idx, dtype=np.int64)
    evict_idx = np.asarray(evict_idx, dtype=np.int64)
    target = np.asarray(target, dtype=np.int64)
    nk, d = keep_idx.shape[0], k.shape[1]
    E = log_s_hat(log_S, n_obs, alpha)
    out = MergeResult(np.empty((nk, d)), np.empty((nk, d)), np.empty(nk, dtype=np.int64),
                      np.empty(nk), np.empty(nk, dtype=np.int64), 0,
                      np.zeros(nk, dtype=bool), np.full(nk, np.nan))
    out.dropped = int(np.asarray(votes)[evict_idx[target < 0]].sum())
    members = [[] for _ in range(nk)]
    for j, t in enumerate(target.tolist()):
        if t >= 0:
            members[t].append(int(evict_idx[j]))
    for r in range(nk):
        c = int(keep_idx[r])
        g = [c] + members[r]
        if len(g) == 1:
            out.k[r], out.v[r], out.votes[r] = k[c], v[c], votes[c]
            out.log_S[r], out.n_obs[r] = log_S[c], n_obs[c]
            continue
        g = np.array(g)
        p = np.asarray(votes, dtype=np.float64)[g]
        Eg = E[g]
        m = Eg.max()
        P = p.sum()
        out.votes[r] = int(np.asarray(votes)[g].sum())
        if not np.isfinite(m):
            # no member was ever observed: all weights vanish; fall back to vote weights
            wn = p / P
            out.k[r], out.v[r], out.log_S[r], out.n_obs[r] = wn @ k[g], wn @ v[g], -np.inf, 0
            out.guarded[r] = True
            continue
        n_r = max(int(n_obs[c]), 1)
        out.n_obs[r] = n_r
        w = p * np.exp(Eg - m)                       # p_i s_hat_i / e^m
        W = w.sum()
        wn = w / W
        L = m + math.log(W / P)                      # ln(sum p s_hat / sum p)
        pos = w > 0
        ell_bar = float((wn[pos] * Eg[pos]).sum())   # sum w ln s_hat / W
        out.ell_bar[r] = ell_bar
        kbar = wn @ k[g]
        out.v[r] = wn @ v[g]
        if abs(ell_bar) < ELL_GUARD:
            out.k[r] = kbar
            out.guarded[r] = True
        else:
            out.k[r] = kbar * (L / ell_bar)
        if alpha == 0.0:
            out.log_S[r] = L
        else:
            out.log_S[r] = L + math.log(-math.expm1(n_r * math.log(alpha)))
    return out


# --------------------------------------------------------------------------- merge-first prefill (Sec. 3.3.2, App. B.4)
def prefill_nearest_earlier(k, length, threshold, exact_any_order=False):
    """For every live slot i its most similar EARLIER key (App. B.4: during prefill, merge by key similarity
    before the eviction strategy is applied).

    U[i, j] = cos(k_i, k_j) for j < i, evaluated as in `match`; near[i] = the first maximiser j of U[i, :i] if
    U[i, near] > threshold (strict), else -1; slot 0 has no earlier key.  Returns (near [length] int64,
    sim [length] float64 = max_j U[i, j], -inf for slot 0).
    """
    k = np.asarray(k, dtype=np.float64)[:length]
    near = np.full(length, -1, dtype=np.int64)
    sim = np.full(length, -np.inf)
    if length < 2:
        return near, sim
    with np.errstate(divide="ignore", invalid="ignore"):
        rn = 1.0 / np.sqrt(_dots_self(k))
        U = (_dots(k, k, exact_any_order) * rn[:, None]) * rn[None, :]
    U = np.where(np.isfinite(U), U, -np.inf)
    for i in range(1, length):
        row = U[i, :i]
        j = int(row.argmax())                              # first maximiser
        sim[i] = row[j]
        if row[j] > threshold:
            near[i] = j
    return near, sim


def prefill_groups(near):
    """Merge groups of the merge-first prefill pass from the nearest-earlier-key links.

    The links near[i] -> j < i form a forest.  A slot is absorbed by the slot it links to unless that slot is
    itself absorbed (a slot that has been merged away cannot receive): walking down from a tree's first slot,
    slots at odd depth are absorbed by their parent, slots at even depth stay and receive their children.
    Every group is therefore one receiving slot plus slots whose own best earlier key it is, each with
    similarity above the threshold to it; chains of similar neighbours are not collapsed transitively.
    Returns (root_idx ascending, absorbed_idx ascending, target = position in root_idx of each absorbed slot).
    """
    near = np.asarray(near, dtype=np.int64)
    n = near.shape[0]
    absorbed = np.zeros(n, dtype=bool)
    for i in range(n):                                     # links point to lower indices: one ascending pass
        j = int(near[i])
        absorbed[i] = j >= 0 and not absorbed[j]
    root_idx = np.flatnonzero(~absorbed).astype(np.int64)
    absorbed_idx = np.flatnonzero(absorbed).astype(np.int64)
    pos = np.full(n, -1, dtype=np.int64)
    pos[root_idx] = np.arange(root_idx.shape[0])
    return root_idx, absorbed_idx, pos[near[absorbed_idx]]


def prefill_merge_first(cache, alpha, threshold, exact_any_order=False, storage_round=None):
    """The merging half of the merge-first prefill policy on every (batch, kv head), in place: nearest earlier
    key per slot, groups as in `prefill_groups`, one multi-way ZIP merge per group (`merge`), the surviving
    slots compacted in their original order.  Nothing is dropped; votes are conserved.  The eviction strategy
    (`compress`) is then applied to the shorter cache by the caller.  Returns per-head (near, root_idx)."""
    trace = []
    for b in range(cache.B):
        for h in range(cache.H):
            n = int(cache.len[b, h])
            near, _ = prefill_nearest_earlier(cache.k[b, h], n, threshold, exact_any_order)
            roots, absorbed, tgt = prefill_groups(near)
            res = merge(cache.k[b, h], cache.v[b, h], cache.votes[b, h], cache.log_S[b, h], cache.n_obs[b, h],
                        roots, absorbed, tgt, alpha)
            nk = roots.shape[0]
            kk, vv = res.k, res.v
            if storage_round is not None:
                kk, vv = storage_round(kk), storage_round(vv)
            cache.k[b, h, :nk], cache.v[b, h, :nk] = kk, vv
            cache.votes[b, h, :nk], cache.log_S[b, h, :nk], cache.n_obs[b, h, :nk] = res.votes, res.log_S, res.n_obs
            cache.len[b, h] = nk
            trace.append((near, roots))
    return trace


# --------------------------------------------------------------------------- Theorem 3
def perturbation_bound(eps, gamma):
    """Right-hand side of Theorem 3: 2 eps (1 + eps) gamma / (1 - eps)^2, for eps < 1."""
    return 2.0 * eps * (1.0 + eps) * gamma / (1.0 - eps) ** 2


# --------------------------------------------------------------------------- per-layer cache + loop
class Cache:
    """One layer's cache state for every (batch, kv head), float64 (or the caller's values)."""

    def __init__(self, batch, n_kv_heads, capacity, head_dim):
        self.B, self.H, self.cap, self.d = batch, n_kv_heads, capacity, head_dim
        self.k = np.zeros((batch, n_kv_heads, capacity, head_dim))
        self.v = np.zeros((batch, n_kv_heads, capacity, head_dim))
        self.votes = np.zeros((batch, n_kv_heads, capacity), dtype=np.int64)
        self.log_S = np.full((batch, n_kv_heads, capacity), -np.inf)
        self.n_obs = np.zeros((batch, n_kv_heads, capacity), dtype=np.int64)
        self.len = np.zeros((batch, n_kv_heads), dtype=np.int64)
        self.dropped = np.zeros((batch, n_kv_heads), dtype=np.int64)

    def append(self, k_t, v_t):
        """Append one token per (batch, kv head) with one vote and no score history."""
        for b in range(self.B):
            for h in range(self.H):
                i = int(self.len[b, h])
                self.k[b, h, i], self.v[b, h, i] = k_t[b, h], v_t[b, h]
                self.votes[b, h, i], self.log_S[b, h, i], self.n_obs[b, h, i] = 1, -np.inf, 0
                self.len[b, h] = i + 1


def attend(cache, q, scale):
    """decode_attn over every (batch, kv head); q [B, Hq, d]. Returns o [B,Hq,d], lse, logits list."""
    B, H, d = cache.B, cache.H, cache.d
    G = q.shape[1] // H
    o = np.zeros((B, H * G, d))
    lse = np.zeros((B, H * G))
    logits = np.zeros((B, H, cache.cap))
    for b in range(B):
        for h in range(H):
            n = int(cache.len[b, h])
            oo, ll, ml = decode_attn(q[b, h * G:(h + 1) * G], cache.k[b, h], cache.v[b, h],
                                     cache.votes[b, h], n, scale)
            o[b, h * G:(h + 1) * G], lse[b, h * G:(h + 1) * G] = oo, ll
            logits[b, h, :n] = ml
    return o, lse, logits


def observe(cache, logits, alpha):
    """score_update over every (batch, kv head)."""
    for b in range(cache.B):
        for h in range(cache.H):
            cache.log_S[b, h], cache.n_obs[b, h] = score_update(
                cache.log_S[b, h], cache.n_obs[b, h], logits[b, h], int(cache.len[b, h]), alpha)


def compress(cache, budget, n_sink, n_recent, alpha, threshold, exact_any_order=False,
             storage_round=None):
    """One compression event (select -> match -> merge) on every (batch, kv head), in place.

    `storage_round`, if given, is applied to the merged K and V (the cache's storage dtype).
    Returns per-head lists of (keep_idx, evict_idx, target) for inspection.
    """
    trace = []
    for b in range(cache.B):
        for h in range(cache.H):
            n = int(cache.len[b, h])
            keep, evict = select(cache.log_S[b, h], cache.n_obs[b, h], cache.votes[b, h], n,
                                 budget, n_sink, n_recent, alpha)
            tgt, _ = match(cache.k[b, h], keep, evict, threshold, exact_any_order)
            res = merge(cache.k[b, h], cache.v[b, h], cache.votes[b, h], cache.log_S[b, h],
                        cache.n_obs[b, h], keep, evict, tgt, alpha)
            nk = keep.shape[0]
            kk, vv = res.k, res.v
            if storage_round is not None:
                kk, vv = storage_round(kk), storage_round(vv)
            cache.k[b, h, :nk], cache.v[b, h, :nk] = kk, vv
            cache.votes[b, h, :nk], cache.log_S[b, h, :nk], cache.n_obs[b, h, :nk] = res.votes, res.log_S, res.n_obs
            cache.len[b, h] = nk
            cache.dropped[b, h] += res.dropped
            trace.append((keep, evict, tgt))
    return trace
