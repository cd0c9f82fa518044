"""GPU parity on seeded random small shapes: batch, head layout, head dimension, dtype, capacity, live
lengths, budget and period drawn at random; one decode step (fused and unfused), a window-score pass and one
compression event each, all against the oracle."""
import numpy as np
import pytest
import torch

from oracle import keepkv_oracle as O
from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U
from tests.test_gpu_compress import _run_compress_stagewise

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _draw(seed):
    g = np.random.default_rng(1000 + seed)
    G = int(g.choice([1, 2, 4, 8]))
    Hkv = int(g.choice([1, 2, 3, 5]))
    D = int(g.choice([64, 128]))
    dtype = "bf16" if g.random() < 0.75 else "f32"
    B = int(g.integers(1, 4))
    N = int(g.integers(20, 700))
    ratio = float(g.uniform(0.05, 0.9))
    period = int(g.integers(1, 40))
    model = str(g.choice(["outlier", "mixture", "ar1", "decay"]))
    w = W.CONFIGS["llama3_8b"].scaled(batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=D, dtype=dtype, context=N,
                                      ratio=ratio, period=period, key_model=model, n_outlier=2, window=3)
    return w, g


@pytest.mark.parametrize("seed", range(64))
def test_random_shape(seed):
    kk = U.kk()
    w, g = _draw(seed)
    if w.budget < w.n_sink + 1 or w.budget >= w.context:
        pytest.skip("budget outside the policy's range for this draw")
    B, H, G, N = w.batch, w.n_kv_heads, w.group, w.context
    alpha = U.f32(float(g.choice([0.0, 0.5, 0.9])))
    K, V = W.make_cache(w, seed)
    votes = g.integers(1, 6, size=(B, H, N)).astype(np.int32)
    lens = g.integers(0, N + 1, size=(B, H)).astype(np.int32)
    lens.flat[0] = N
    cap = N + int(g.integers(1, 9))
    lay, c = U.new_cache(w, capacity=cap, K=K, V=V, votes=votes, lens=lens)
    ws = U.workspace(lay, cap, w.budget)

    # window scores (causal or not), then one fused decode step; both against the oracle on the downloaded state
    win = int(g.integers(1, max(2, min(6, 128 // G))))
    q_win = np.stack([W.make_query(w, seed, t - win) for t in range(win)], axis=2)
    first_pos = -1 if g.random() < 0.5 else int(g.integers(0, N))
    oc = U.download(c)
    kk.score_window(lay, c, U.to_device(q_win, w.dtype), win, alpha, first_pos)
    torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            n = int(lens[b, h])
            rs, rn = O.window_score(oc.log_S[b, h], oc.n_obs[b, h], q_win[b, h * G:(h + 1) * G].transpose(1, 0, 2),
                                    oc.k[b, h], n, U.f32(w.scale), alpha, first_pos)
            assert np.array_equal(U.n_obs(c)[b, h, :n].cpu().numpy(), rn[:n]), (seed, b, h)
            np.testing.assert_allclose(c.log_s[b, h, :n].cpu().numpy(), rs[:n], rtol=1e-5, atol=2e-4)

    q = W.make_query(w, seed, 0)
    k_t, v_t = W.make_token(w, seed, 0)
    out = torch.zeros(B, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    logits = torch.zeros(B, H, cap, dtype=torch.float32, device="cuda")
    oc = U.download(c)
    if g.random() < 0.5:
        c.len_hint = int(lens.max())
    kk.decode_step(lay, c, U.to_device(q, w.dtype), U.to_device(k_t, w.dtype), U.to_device(v_t, w.dtype), out, logits,
                   alpha, None, ws)
    torch.cuda.synchronize()
    c.len_hint = 0
    oc.append(k_t.astype(np.float64), v_t.astype(np.float64))
    o_ref, _, lg = O.attend(oc, q.astype(np.float64), w.scale)
    O.observe(oc, lg, alpha)
    err = U.storage_err_rows(U.to_host(out), o_ref, w.dtype)
    assert err.max() <= TOL, (seed, float(err.max()))
    assert np.array_equal(c.len.cpu().numpy(), oc.len)
    for b in range(B):
        for h in range(H):
            n = int(oc.len[b, h])
            np.testing.assert_allclose(c.log_s[b, h, :n].cpu().numpy(), oc.log_S[b, h, :n], rtol=2e-3, atol=2e-3)
            assert np.array_equal(U.n_obs(c)[b, h, :n].cpu().numpy(), oc.n_obs[b, h, :n])
            np.testing.assert_allclose(logits[b, h, :n].cpu().numpy(), lg[b, h, :n], rtol=2e-3, atol=2e-3)

    # one compression event on whatever state the steps above left
    _run_compress_stagewise(w, lay, c, ws, alpha, U.f32(float(g.choice([0.8, 0.3, -2.0]))))
