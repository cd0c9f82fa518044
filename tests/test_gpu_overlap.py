"""GPU check of the launch configurations that bench.py times: decode steps of several layers in rotation inside one
HIP graph, each layer's compression event either on the same stream or on a second stream beside the other
layers' steps (enqueued one step late, joined before the layer's next step), index lists and the side
workspace shared by all events.
The same sequence launched eagerly on a single stream must leave every cache in the same state bit for bit
(all kernels are deterministic), whatever the streams overlap; the eager sequence itself is what the other
GPU tests compare with the oracle.  The graph is replayed from identical starting states several times, with
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2504_09936_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _state(caches, cur, dropped):
    out = []
    for c2, cu in zip(caches, cur):
        c = c2[cu]
        n = int(c.len.max().item())
        out.append([c.len.clone(), c.votes[:, :, :n].clone(), U.n_obs(c)[:, :, :n].clone(), c.log_s[:, :, :n].clone(),
                    c.k[:, :, :n].clone().view(torch.int16), c.v[:, :, :n].clone().view(torch.int16)])
    out.append([dropped.clone()])
    return out


@pytest.mark.parametrize("period,layers,overlap,inplace", [(8, 4, True, False), (5, 3, True, False), (8, 4, False, False),
                                                          (8, 4, True, True), (5, 3, False, True)])
def test_graph_equals_eager_single_stream(period, layers, overlap, inplace):
    kk = U.kk()
    w = W.CONFIGS["llama3_8b"].scaled(batch=2, context=400, ratio=0.25, period=period)
    B, H, Hq, D, Bud, P, R = w.batch, w.n_kv_heads, w.n_q_heads, w.head_dim, w.budget, period, layers
    cap = Bud + P
    alpha, T = U.f32(w.alpha), U.f32(0.3)
    lay = U.layout_of(w)
    K = 16 * R * P // 4                                  # steps: every layer has several events
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    q = (torch.randn(K, B, Hq, D, device="cuda", generator=g) * 2).bfloat16()
    kt = torch.randn(K, B, H, D, device="cuda", generator=g).bfloat16()
    vt = torch.randn(K, B, H, D, device="cuda", generator=g).bfloat16()
    K0 = torch.randn(R, B, H, Bud, D, device="cuda", generator=g).bfloat16()
    V0 = torch.randn(R, B, H, Bud, D, device="cuda", generator=g).bfloat16()

    def fresh():
        caches = []
        for layer in range(R):
            pair = [kk.Cache(lay, cap), kk.Cache(lay, cap)]
            c = pair[0]
            c.k[:, :, :Bud] = K0[layer]
            c.v[:, :, :Bud] = V0[layer]
            c.votes[:, :, :Bud] = 1
            c.log_s[:, :, :Bud] = -1.0
            U.set_n_obs(c, 2, (slice(None), slice(None), slice(0, Bud)))
            c.len.fill_(Bud)
            caches.append(pair)
        return caches

    out = torch.zeros(B, Hq, D, dtype=torch.bfloat16, device="cuda")
    keep = torch.zeros(B, H, Bud, dtype=torch.int32, device="cuda")
    evict = torch.zeros(B, H, cap - Bud, dtype=torch.int32, device="cuda")
    n_ev = torch.zeros(B, H, dtype=torch.int32, device="cuda")
    match = torch.zeros(B, H, cap - Bud, dtype=torch.int32, device="cuda")
    ws, ws_side = kk.new_workspace(lay, cap, Bud), kk.new_workspace(lay, cap, Bud)

    def compress(c, d, dropped, layer, wsp, orders):
        if inplace:                                      # the event updates the cache where it is; `orders` = its slots by age
            kk.select_aged(lay, c, orders[layer], Bud, w.n_sink, w.n_recent, alpha, keep, evict, n_ev, wsp)
            kk.match(lay, c, Bud, keep, evict, n_ev, T, match, None, wsp)
            kk.merge_inplace(lay, c, orders[layer], Bud, keep, evict, n_ev, match, alpha, dropped[layer])
        else:
            kk.select(lay, c, Bud, w.n_sink, w.n_recent, alpha, keep, evict, n_ev, wsp)
            kk.match(lay, c, Bud, keep, evict, n_ev, T, match, None, wsp)
            kk.merge(lay, c, d, Bud, keep, evict, n_ev, match, alpha, dropped[layer], wsp)

    def new_orders():
        return torch.arange(Bud, dtype=torch.int32, device="cuda").repeat(R, B, H, 1).contiguous()

    def run(caches, dropped, overlapped, side, orders):
        cur = [0] * R
        since = [(layer * P) // R for layer in range(R)]
        pending = [None] * R
        deferred = []

        def launch_deferred():
            while deferred:
                c, d, layer, fork = deferred.pop(0)
                side.wait_event(fork)
                with torch.cuda.stream(side):
                    compress(c, d, dropped, layer, ws_side, orders)
                    pending[layer] = torch.cuda.Event()
                    pending[layer].record()

        for i in range(K):
            layer = i % R
            c = caches[layer][cur[layer]]
            if overlapped:
                if any(x[2] == layer for x in deferred):
                    launch_deferred()
                if pending[layer] is not None:
                    torch.cuda.current_stream().wait_event(pending[layer])
                    pending[layer] = None
            c.len_hint = Bud + since[layer]
            kk.decode_step(lay, c, q[i], kt[i], vt[i], out, None, alpha, None, ws)
            if overlapped:
                launch_deferred()
            since[layer] += 1
            if since[layer] == P:
                d = caches[layer][1 - cur[layer]]
                if overlapped:
                    fork = torch.cuda.Event()
                    fork.record()
                    deferred.append((c, d, layer, fork))
                else:
                    compress(c, d, dropped, layer, ws, orders)
                if not inplace:
                    cur[layer] = 1 - cur[layer]
                since[layer] = 0
        if overlapped:
            launch_deferred()
            torch.cuda.current_stream().wait_stream(side)
        return cur

    # eager, single stream
    caches_a, dropped_a = fresh(), torch.zeros(R, B, H, dtype=torch.int64, device="cuda")
    orders_a = new_orders()
    cur_a = run(caches_a, dropped_a, False, None, orders_a)
    torch.cuda.synchronize()
    ref = _state(caches_a, cur_a, dropped_a)
    assert int(dropped_a.sum().item()) >= 0 and all(int(c[cu].len.max().item()) <= cap for c, cu in zip(caches_a, cur_a))

    # one graph, events on a side stream or in line; replayed three times from the same starting state
    caches_b, dropped_b = fresh(), torch.zeros(R, B, H, dtype=torch.int64, device="cuda")
    start = [[[t.clone() for t in (c.k, c.v, c.votes, c.log_s, c.born, c.t_obs, c.len)] for c in pair] for pair in caches_b]
    stream, side = torch.cuda.Stream(), torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    orders_b = new_orders()
    with torch.cuda.graph(graph, stream=stream):
        cur_b = run(caches_b, dropped_b, overlap, side, orders_b)
    assert cur_b == cur_a
    for replay in range(3):
        for pair, saved in zip(caches_b, start):          # eager work between the replays: restore the state
            for c, s in zip(pair, saved):
                for t, s_t in zip((c.k, c.v, c.votes, c.log_s, c.born, c.t_obs, c.len), s):
                    t.copy_(s_t)
        dropped_b.zero_()
        orders_b.copy_(new_orders())
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(orders_a, orders_b)
        got = _state(caches_b, cur_b, dropped_b)
        for layer, (r_, g_) in enumerate(zip(ref, got)):
            for j, (x, y) in enumerate(zip(r_, g_)):
                assert torch.equal(x, y), ("replay", replay, "layer", layer, "field", j)
