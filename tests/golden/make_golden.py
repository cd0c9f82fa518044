"""Writes tests/golden/tiny_run.json: a digest of the oracle's whole run on the tiny workload.

Calls only the oracle and the seeded input generators.  The file pins the oracle against
unintended change (the paper prints no worked numeric example to pin it to; its formulas are
pinned by the closed forms and invariants in tests/test_oracle_*.py).  Regenerate only together
with a deliberate, documented change of the oracle:

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import keepkv_oracle as O                      # noqa: E402
from paper_2504_09936_amd import workloads as W            # noqa: E402


def _digest(a) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()[:16]


def run(threshold: float) -> dict:
    w = W.CONFIGS["tiny"]
    seed, alpha = 0, w.alpha
    K, V = W.make_cache(w, seed)
    c = O.Cache(w.batch, w.n_kv_heads, w.capacity, w.head_dim)
    c.k[:, :, : w.context], c.v[:, :, : w.context] = K, V
    c.votes[:, :, : w.context] = 1
    c.len[:] = w.context
    G = w.group
    q_win = np.stack([W.make_query(w, seed, t - w.window) for t in range(w.window)], axis=2)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            c.log_S[b, h], c.n_obs[b, h] = O.window_score(
                c.log_S[b, h], c.n_obs[b, h], q_win[b, h * G:(h + 1) * G].transpose(1, 0, 2), c.k[b, h], w.context,
                w.scale, alpha)
    events = []

    def event():
        trace = O.compress(c, w.budget, w.n_sink, w.n_recent, alpha, threshold)
        events.append({"keep": _digest(np.concatenate([t[0] for t in trace])),
                       "evict": _digest(np.concatenate([t[1] for t in trace])),
                       "target": _digest(np.concatenate([t[2] for t in trace])),
                       "merged": int(sum((t[2] >= 0).sum() for t in trace)),
                       "votes_sum": int(c.votes[:, :, : w.budget].sum()), "dropped": int(c.dropped.sum())})

    event()
    outs = []
    for t in range(w.steps):
        k_t, v_t = W.make_token(w, seed, t)
        c.append(k_t.astype(np.float64), v_t.astype(np.float64))
        o, _, lg = O.attend(c, W.make_query(w, seed, t).astype(np.float64), w.scale)
        O.observe(c, lg, alpha)
        outs.append([round(float(x), 9) for x in (o.sum(), np.abs(o).sum(), o[0, 0, 0], o[-1, -1, -1])])
        if (t + 1) % w.period == 0:
            event()
    return {"threshold": threshold, "events": events, "outputs_sum_abs_first_last": outs,
            "final_log_S_sum": round(float(c.log_S[:, :, : w.budget].sum()), 6)}


if __name__ == "__main__":
    out = {"workload": "tiny, seed 0", "runs": [run(0.8), run(-2.0)]}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_run.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)
