"""Comparison baselines of the paper's analysis, CPU float64 -- test infrastructure only.

Plain eviction (Sec. 3.2, Eq. 4) and convex-combination merging (Eq. 5; App. A.1 multi-way
form with the similarity-softmax and Gaussian-kernel weightings the paper names).  They exist
to reproduce the paper's qualitative claims next to the oracle of the method itself: eviction
and convex merging perturb the current step's output, and a convexly merged slot attracts less
attention than its members did (Theorem 1), while the vote-carrying merge does neither.
Nothing here is used by the HIP library, and there is no GPU counterpart.
"""
from __future__ import annotations

import numpy as np


def evict(k, v, keep_idx):
    """Discard every slot outside keep_idx (Sec. 3.2, plain eviction).  Returns (k', v')."""
    keep_idx = np.asarray(keep_idx, dtype=np.int64)
    return np.asarray(k, dtype=np.float64)[keep_idx], np.asarray(v, dtype=np.float64)[keep_idx]


def evicted_output(o, a_e, v_e):
    """Closed form of the output after discarding one pair (Eq. 4): (o - A_e v_e) / (1 - A_e)."""
    return (np.asarray(o, dtype=np.float64) - a_e * np.asarray(v_e, dtype=np.float64)) / (1.0 - a_e)


def convex_weights(k_members, k_c, scheme, sigma=1.0):
    """Normalised weights over the members of one merge group (App. A.1), the retained key first.

    'similarity': softmax of the cosine between each member key and the retained key;
    'gaussian'  : softmax of -|k_j - k_c|^2 / (2 sigma^2);
    'uniform'   : plain average.
    """
    k_members = np.asarray(k_members, dtype=np.float64)
    k_c = np.asarray(k_c, dtype=np.float64)
    if scheme == "similarity":
        z = (k_members @ k_c) / (np.linalg.norm(k_members, axis=1) * np.linalg.norm(k_c))
    elif scheme == "gaussian":
        z = -((k_members - k_c) ** 2).sum(1) / (2.0 * sigma * sigma)
    elif scheme == "uniform":
        z = np.zeros(k_members.shape[0])
    else:
        raise ValueError(f"unknown weighting {scheme!r}")
    w = np.exp(z - z.max())
    return w / w.sum()


def convex_merge(k, v, keep_idx, evict_idx, target, scheme="similarity", sigma=1.0):
    """Convex-combination merging (Eq. 5 in its multi-way form of App. A.1).

    Group of retained position r: the retained slot keep_idx[r] and every evict_idx[j] with
    target[j] == r; k_r = sum w_i k_i, v_r = sum w_i v_i with sum w_i = 1.  Unmatched evicted
    slots are discarded.  The result carries no merge history (every slot counts once).
    Returns (k', v') in keep_idx order.
    """
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    keep_idx = np.asarray(keep_idx, dtype=np.int64)
    evict_idx = np.asarray(evict_idx, dtype=np.int64)
    target = np.asarray(target, dtype=np.int64)
    ko, vo = k[keep_idx].copy(), v[keep_idx].copy()
    for r in range(keep_idx.shape[0]):
        members = evict_idx[target == r]
        if members.size == 0:
            continue
        g = np.concatenate(([keep_idx[r]], members))
        w = convex_weights(k[g], k[keep_idx[r]], scheme, sigma)
        ko[r], vo[r] = w @ k[g], w @ v[g]
    return ko, vo
