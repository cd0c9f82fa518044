"""GPU checks that are not parity with the oracle: run-to-run determinism of every entry point,
HIP-graph capture and replay of a decode step plus a compression event, and error statuses."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _state(c):
    n = c.capacity
    return [c.k.clone(), c.v.clone(), c.votes.clone(), c.log_s.clone(), c.born.clone(), c.t_obs.clone(), c.len.clone()]


def _restore(c, st):
    for dst, src in zip((c.k, c.v, c.votes, c.log_s, c.born, c.t_obs, c.len), st):
        dst.copy_(src)


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else (t.view(torch.int32) if t.dtype == torch.float32 else t)


def _setup(seed=0, batch=2, context=1200):
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=batch, context=context, period=16)
    alpha = U.f32(w.alpha)
    K, V = W.make_cache(w, seed)
    lay, big = U.new_cache(w, capacity=context, K=K, V=V)
    ws = kk.new_workspace(lay, context, w.budget)
    out = torch.zeros(w.batch, w.n_q_heads, w.head_dim, dtype=lay.torch_dtype, device="cuda")
    logits = torch.zeros(w.batch, w.n_kv_heads, context, dtype=torch.float32, device="cuda")
    for t in range(3):
        kk.decode_attn(lay, big, U.to_device(W.make_query(w, seed, t - 3), w.dtype), out, logits, None, ws)
        kk.score(lay, big, logits, alpha)
    torch.cuda.synchronize()
    return kk, w, alpha, lay, big, ws, out, logits


def _compress(kk, w, lay, src, dst, ws, alpha, T, bufs):
    keep, evict, n_ev, match, dropped = bufs
    kk.select(lay, src, w.budget, w.n_sink, w.n_recent, alpha, keep, evict, n_ev, ws)
    kk.match(lay, src, w.budget, keep, evict, n_ev, T, match, None, ws)
    kk.merge(lay, src, dst, w.budget, keep, evict, n_ev, match, alpha, dropped, ws)


def _bufs(w, cap):
    B, H = w.batch, w.n_kv_heads
    z = lambda *s, dt=torch.int32: torch.zeros(*s, dtype=dt, device="cuda")
    return z(B, H, w.budget), z(B, H, cap - w.budget), z(B, H), z(B, H, cap - w.budget), z(B, H, dt=torch.int64)


@pytest.mark.parametrize("threshold", [0.8, -2.0])
def test_every_entry_point_is_deterministic(threshold):
    kk, w, alpha, lay, big, ws, out, logits = _setup()
    T = U.f32(threshold)
    lay2, dst = U.new_cache(w, capacity=w.budget + w.period)
    results = []
    for rep in range(2):
        bufs = _bufs(w, big.capacity)
        dst.k.zero_(); dst.v.zero_()
        _compress(kk, w, lay, big, dst, ws, alpha, T, bufs)
        q = U.to_device(W.make_query(w, 0, 5), w.dtype)
        kt, vt = W.make_token(w, 0, 5)
        st = _state(dst)
        kk.decode_step(lay, dst, q, U.to_device(kt, w.dtype), U.to_device(vt, w.dtype), out, logits, alpha, None, ws)
        torch.cuda.synchronize()
        results.append([_bits(x).clone() for x in (*bufs[:4], bufs[4], out, logits, *_state(dst))])
        _restore(dst, st)
    for a, b in zip(*results):
        assert torch.equal(a, b)


def test_graph_replay_matches_eager():
    """A captured decode step + compression event replayed several times, with eager work and
    synchronisation in between, gives the eager result every time."""
    kk, w, alpha, lay, big, ws, out, logits = _setup(seed=1)
    T = U.f32(-2.0)
    bufs = _bufs(w, big.capacity)
    lay2, small = U.new_cache(w, capacity=w.budget + w.period)
    lay3, other = U.new_cache(w, capacity=w.budget + w.period)
    _compress(kk, w, lay, big, small, ws, alpha, T, bufs)
    sbufs = _bufs(w, small.capacity)
    q = U.to_device(W.make_query(w, 1, 0), w.dtype)
    kt, vt = (U.to_device(x, w.dtype) for x in W.make_token(w, 1, 0))
    small.len_hint = w.budget + 1
    torch.cuda.synchronize()
    start = _state(small)

    def body():
        kk.decode_step(lay, small, q, kt, vt, out, None, alpha, None, ws)
        _compress(kk, w, lay, small, other, ws, alpha, T, sbufs)

    body()                                             # eager reference (also warms one-time attributes)
    torch.cuda.synchronize()
    ref = [_bits(x).clone() for x in (out, *_state(small), *_state(other), *sbufs[:4])]
    graph = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()
    _restore(small, start)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=stream):
        body()
    for rep in range(4):
        _restore(small, start)
        other.k.normal_(); other.votes.fill_(-5)       # eager work between replays
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [_bits(x) for x in (out, *_state(small), *_state(other), *sbufs[:4])]
        n = w.budget
        for i, (a, b) in enumerate(zip(got, ref)):
            if 8 <= i <= 12:                           # destination cache (k, v, votes, log_s, born): the live prefix only
                a, b = a[:, :, :n], b[:, :, :n]
            assert torch.equal(a, b), (rep, i)


def test_error_statuses_on_device_buffers():
    kk, w, alpha, lay, big, ws, out, logits = _setup(batch=1, context=400)
    lib = kk._lib
    keep, evict, n_ev, match, dropped = _bufs(w, big.capacity)
    cs = big.c()
    P = lambda t: C.c_void_p(t.data_ptr())
    # a workspace that is too small is refused before any launch
    assert lib.keepkv_select(C.byref(lay.c()), C.byref(cs), w.budget, 4, 8, C.c_float(alpha), P(keep), P(evict), P(n_ev),
                             P(ws), 1024, None) == kk.ERR_WORKSPACE
    # merge into itself is refused
    assert lib.keepkv_merge(C.byref(lay.c()), C.byref(cs), C.byref(cs), w.budget, P(keep), P(evict), P(n_ev), P(match),
                            C.c_float(alpha), None, P(ws), ws.numel(), None) == kk.ERR_INVALID_ARG
    # unsupported budget for the MFMA matcher
    lay_b, huge = U.new_cache(w, capacity=6000)
    hs = huge.c()
    assert lib.keepkv_match(C.byref(lay.c()), C.byref(hs), 5000, P(keep), P(evict), P(n_ev), C.c_float(0.8), P(match),
                            None, P(ws), ws.numel(), None) == kk.ERR_UNSUPPORTED
    # NaN threshold
    assert lib.keepkv_match(C.byref(lay.c()), C.byref(cs), w.budget, P(keep), P(evict), P(n_ev), C.c_float(float("nan")),
                            P(match), None, P(ws), ws.numel(), None) == kk.ERR_INVALID_ARG
    # misaligned query pointer
    q = torch.zeros(w.n_q_heads * w.head_dim + 8, dtype=lay.torch_dtype, device="cuda")
    assert lib.keepkv_decode_attn(C.byref(lay.c()), C.byref(cs), C.c_void_p(q.data_ptr() + 2), P(out), None, None, P(ws),
                                  ws.numel(), None) == kk.ERR_INVALID_ARG
    torch.cuda.synchronize()


def test_measurement_probes_run_and_validate_arguments():
    kk = U.kk()
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    buf = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda")
    kk.probe_read(buf, 64, sink)
    kk.probe_read(buf[: 16 * 1000 + 16], 7, sink)            # ragged share per workgroup
    flops = kk.probe_mfma(8, 10, sink)
    assert kk.probe_mfma(8, 10, sink, True) == flops         # random operands: the same instruction count
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 10 * 4 * 2 * 32 * 32 * 16
    assert sink.sum().item() == 0.0                          # the sinks are never written in practice
    for bad in (lambda: kk.probe_read(buf[:24], 4, sink), lambda: kk.probe_read(buf, 0, sink),
                lambda: kk.probe_read(None, 4, sink), lambda: kk.probe_mfma(0, 10, sink),
                lambda: kk.probe_mfma(4, 0, sink)):
        with pytest.raises(kk.KeepKVError) as e:
            bad()
        assert e.value.status == kk.ERR_INVALID_ARG


def test_cache_state_dump_and_reload(tmp_path):
    """A cache dumped to a file and loaded into a fresh one gives the same decode step, bit for bit."""
    kk, w, alpha, lay, big, ws, out, logits = _setup(seed=3, batch=1, context=500)
    path = str(tmp_path / "cache.pt")
    big.save(path)
    other = kk.Cache(lay, big.capacity)
    other.load(path)
    q = U.to_device(W.make_query(w, 3, 9), w.dtype)
    res = []
    for c in (big, other):
        kk.decode_attn(lay, c, q, out, logits, None, ws)
        torch.cuda.synchronize()
        res.append((_bits(out).clone(), logits.clone(), [_bits(x).clone() for x in _state(c)]))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])
    for a, b in zip(res[0][2], res[1][2]):
        assert torch.equal(a, b)
    with pytest.raises(ValueError):
        kk.Cache(lay, big.capacity + 1).load(path)
