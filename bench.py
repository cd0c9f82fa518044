#!/usr/bin/env python3
"""Benchmark of the KeepKV hot path on one MI355X.

A *step* is one pass of the whole hot path over one batch for one layer: append the new
token's (k, v), vote-weighted decode attention, EMA score update and -- every `period`
steps of that layer -- a compression event (select, match, merge into the layer's other
buffer).  Steps rotate over `--layers` distinct layer caches so that the working set
(layers x cache bytes) is far larger than the 256 MB Infinity Cache.  All inputs are
synthetic (paper_2504_09936_amd.workloads) and resident in HBM before the timed region.
The timed region is one HIP graph of exactly K steps.

Prints ONE JSON line; `value` is decode tokens/s per layer for the whole hot path
(batch x steps / time), with a `roofline` object for the decode-attention kernel and a
`cpu_baseline` object (the numpy oracle on the host cores, bounded sample).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the fused decode kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled
# by the copy-probe calibration (profiles/decode_hbm_traffic_llama3_8b.md).  Counters cannot be
# read from inside this process, so the figure is the recorded one for the default workload.
PMC_TRAFFIC_BYTES = {"llama3_8b": int((14470.7 * 2.00 + 1162.6 * 1.00) * 1024)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4096)
    ap.add_argument("--warmup", type=int, default=256)
    ap.add_argument("--workload", default="llama3_8b")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--threshold", type=float, default=None, help="merging threshold T (default: workload's, 0.8)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap", choices=("auto", "on", "off"), default="auto",
                    help="run each compression event on a second stream beside the other layers' decode steps.  "
                         "A branch to a second queue costs the decode stream 20-35 us per event whatever its length, "
                         "an event on the decode stream its own 50-60 us: auto overlaps when events are frequent "
                         "(period <= 32), where the side stream also has to hide several events at once")
    ap.add_argument("--unfused", action="store_true",
                    help="use keepkv_append + keepkv_decode_attn + keepkv_score instead of keepkv_decode_step")
    ap.add_argument("--window", type=int, default=None, help="observation passes before the first event")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain device copy of known size (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (every (batch, kv head) cache is independent; "
              "kv heads or batch would shard across GPUs with no exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2504_09936_amd import binding as kk
    from paper_2504_09936_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.copy_probe:
        n = 256 * 1024 * 1024                      # bytes read and bytes written per copy
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": n, "copies": 8}))
        return
    w = W.CONFIGS[args.workload]
    if args.window is not None:
        w = w.scaled(window=args.window)
    R, K, Wm = args.layers, args.steps, args.warmup
    B, Hq, H, D, P, Bud, N = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.period, w.budget, w.context
    args.overlap = args.overlap == "on" or (args.overlap == "auto" and P <= 32)
    alpha = float(np.float32(w.alpha))
    T = float(np.float32(w.threshold if args.threshold is None else args.threshold))
    bf16 = w.dtype == "bf16"
    lay = kk.Layout(B, Hq, H, D, kk.BF16 if bf16 else kk.F32, w.scale)
    esz = 2 if bf16 else 4
    cap = Bud + P

    def to_dev(a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        if bf16:
            return torch.from_numpy(W.to_bf16_bits(a).view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    # ------------------------------------------------------------------ buffers
    big = kk.Cache(lay, N)
    ws = kk.new_workspace(lay, N, Bud)
    keep = torch.zeros(B, H, Bud, dtype=torch.int32, device=dev)
    evict_big = torch.zeros(B, H, N - Bud, dtype=torch.int32, device=dev)
    match_big = torch.zeros(B, H, N - Bud, dtype=torch.int32, device=dev)
    evict_s = torch.zeros(B, H, cap - Bud, dtype=torch.int32, device=dev)
    match_s = torch.zeros(B, H, cap - Bud, dtype=torch.int32, device=dev)
    n_ev = torch.zeros(B, H, dtype=torch.int32, device=dev)
    dropped = torch.zeros(R, B, H, dtype=torch.int64, device=dev)
    logits = torch.zeros(B, H, N, dtype=torch.float32, device=dev)
    out = torch.zeros(B, Hq, D, dtype=lay.torch_dtype, device=dev)
    caches = [[kk.Cache(lay, cap), kk.Cache(lay, cap)] for _ in range(R)]
    cur = [0] * R

    ev = lambda: torch.cuda.Event(enable_timing=True)

    # ------------------------------------------------------------------ prefill: window passes + first event per layer
    t0 = time.time()
    K0, V0 = W.make_cache(w, 0)
    K0d, V0d = to_dev(K0), to_dev(V0)
    del K0, V0
    first = {"score_window": [], "select": [], "match": [], "merge": []}
    win_chunk = max(1, 128 // (Hq // H))          # queries per keepkv_score_window call
    for layer in range(R):
        # layers are token/batch rotations of the seeded prefill tensors: same statistics, distinct bytes
        big.k.copy_(torch.roll(K0d, shifts=(layer, 257 * layer), dims=(0, 2)))
        big.v.copy_(torch.roll(V0d, shifts=(layer, 257 * layer), dims=(0, 2)))
        if w.query_model == "mean":
            big.k[:, :, 0] = K0d[:, :, 0]
        big.votes.fill_(1); big.log_s.fill_(float("-inf")); big.n_obs.zero_(); big.len.fill_(N)
        # observation window (Eq. 8, t = L): all window queries in one pass over the keys
        q_win = to_dev(np.stack([W.make_query(w, layer, t - w.window) for t in range(w.window)], axis=2))
        e = [ev() for _ in range(4)]
        for j0 in range(0, w.window, win_chunk):
            j1 = min(w.window, j0 + win_chunk)
            kk.score_window(lay, big, q_win[:, :, j0:j1].contiguous() if (j0, j1) != (0, w.window) else q_win,
                            j1 - j0, alpha, -1)
        e[0].record()
        kk.select(lay, big, Bud, w.n_sink, w.n_recent, alpha, keep, evict_big, n_ev, ws)
        e[1].record()
        kk.match(lay, big, Bud, keep, evict_big, n_ev, T, match_big, None, ws)
        e[2].record()
        kk.merge(lay, big, caches[layer][0], Bud, keep, evict_big, n_ev, match_big, alpha, dropped[layer], ws)
        e[3].record()
        torch.cuda.synchronize()
        for i, name in enumerate(("select", "match", "merge")):
            first[name].append(e[i].elapsed_time(e[i + 1]) * 1e3)
    # window pass timed back to back over four full-size caches (a lone eager launch is dominated by launch
    # latency; four distinct caches exceed the 256 MB last-level cache, so the keys come from HBM)
    rot = [big] + [kk.Cache(lay, N) for _ in range(3)]
    for i, c in enumerate(rot[1:]):
        c.k.copy_(torch.roll(K0d, shifts=(i + 1, 1031 * (i + 1)), dims=(0, 2)))
        c.len.fill_(N)
    for rep in range(3):
        e0, e1 = ev(), ev()
        e0.record()
        for c in rot + rot:
            for j0 in range(0, w.window, win_chunk):
                j1 = min(w.window, j0 + win_chunk)
                kk.score_window(lay, c, q_win[:, :, j0:j1].contiguous() if (j0, j1) != (0, w.window) else q_win,
                                j1 - j0, alpha, -1)
        e1.record()
        torch.cuda.synchronize()
        first["score_window"].append(e0.elapsed_time(e1) * 1e3 / 8)
    del rot
    del K0d, V0d
    t_prefill = time.time() - t0

    # ------------------------------------------------------------------ per-step inputs, resident in HBM
    total_steps = Wm + K
    per_layer = (total_steps + R - 1) // R + 1
    q_all = torch.empty(R, per_layer, B, Hq, D, dtype=lay.torch_dtype, device=dev)
    k_all = torch.empty(R, per_layer, B, H, D, dtype=lay.torch_dtype, device=dev)
    v_all = torch.empty(R, per_layer, B, H, D, dtype=lay.torch_dtype, device=dev)
    for layer in range(R):
        prev = None
        qs, ks, vs = [], [], []
        for t in range(per_layer):
            qs.append(W.make_query(w, layer, t))
            k_t, v_t = W.make_token(w, layer, t, prev=prev)
            prev = (k_t, v_t) if w.key_model == "ar1" else None
            ks.append(k_t); vs.append(v_t)
        q_all[layer], k_all[layer], v_all[layer] = to_dev(np.stack(qs)), to_dev(np.stack(ks)), to_dev(np.stack(vs))

    step_no = [0] * R          # decode steps done per layer
    n_events = 0
    # Compression phases are staggered over the layers (layer L's first period is shorter by L*P/R steps), so
    # that the events are spread evenly over the steps instead of all layers compressing in the same round.
    # With --overlap each event runs on a second stream next to the decode steps of the other layers, and a
    # layer's next decode step waits for its own event only.
    since = [(layer * P) // R for layer in range(R)]   # steps since the layer's last event
    side = torch.cuda.Stream()
    ws_side = kk.new_workspace(lay, N, Bud)
    pending = [None] * R

    def decode(c, layer, t, since):
        """One decode step of `layer` with input set t; `since` = steps since its last compression."""
        if args.unfused:
            kk.append(lay, c, k_all[layer, t], v_all[layer, t], None)
            kk.decode_attn(lay, c, q_all[layer, t], out, logits, None, ws)
            kk.score(lay, c, logits, alpha)
        else:
            c.len_hint = Bud + since          # host-known bound on len before this step's append
            kk.decode_step(lay, c, q_all[layer, t], k_all[layer, t], v_all[layer, t], out, None, alpha, None, ws)

    def compress(c, d, layer, wsp):
        kk.select(lay, c, Bud, w.n_sink, w.n_recent, alpha, keep, evict_s, n_ev, wsp)
        kk.match(lay, c, Bud, keep, evict_s, n_ev, T, match_s, None, wsp)
        kk.merge(lay, c, d, Bud, keep, evict_s, n_ev, match_s, alpha, dropped[layer], wsp)

    deferred = []                                # events whose side-stream work is still to be enqueued

    def launch_deferred():
        # The side-stream work of an event is enqueued one step late: it depends on the event recorded right
        # after its layer's decode step all the same, but the main stream's next step is then already in the
        # queue (or graph) when the branch is created, and it is the branch, not the chain of decode steps,
        # that moves to another hardware queue.
        while deferred:
            c, d, layer, fork = deferred.pop(0)
            side.wait_event(fork)
            with torch.cuda.stream(side):
                compress(c, d, layer, ws_side)
                pending[layer] = torch.cuda.Event()
                pending[layer].record()

    def one_step(i):
        nonlocal n_events
        layer = i % R
        t = step_no[layer]
        c = caches[layer][cur[layer]]
        main = torch.cuda.current_stream()
        if any(x[2] == layer for x in deferred):  # (a single layer in rotation: its event cannot wait a step)
            launch_deferred()
        if pending[layer] is not None:           # the layer's last compression event ran on the side stream
            main.wait_event(pending[layer])
            pending[layer] = None
        decode(c, layer, t % per_layer, since[layer])
        launch_deferred()
        step_no[layer] = t + 1
        since[layer] += 1
        if since[layer] == P:
            d = caches[layer][1 - cur[layer]]
            if not args.overlap:
                compress(c, d, layer, ws)
            else:
                fork = torch.cuda.Event()
                fork.record()                    # on the main stream, right after this layer's step
                deferred.append((c, d, layer, fork))
            cur[layer] = 1 - cur[layer]
            since[layer] = 0
            n_events += 1

    def join_side():
        if args.overlap:
            launch_deferred()
            torch.cuda.current_stream().wait_stream(side)
            for layer in range(R):
                pending[layer] = None

    # ------------------------------------------------------------------ warm-up (eager), then the timed K steps
    for i in range(Wm):
        one_step(i)
    join_side()
    torch.cuda.synchronize()
    n_events = 0
    stream = torch.cuda.Stream()
    start, stop = ev(), ev()
    if args.no_graph:
        with torch.cuda.stream(stream):
            torch.cuda.synchronize()
            start.record()
            for i in range(Wm, Wm + K):
                one_step(i)
            join_side()
            stop.record()
        torch.cuda.synchronize()
    else:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(Wm, Wm + K):
                one_step(i)
            join_side()
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            start.record()
            graph.replay()
            stop.record()
        torch.cuda.synchronize()
    elapsed_ms = start.elapsed_time(stop)
    timed_events = n_events
    overflow_check = max(int(c[cu].len.max().item()) for c, cu in zip(caches, cur))
    assert overflow_check <= cap

    # ------------------------------------------------------------------ per-kernel durations
    # (1) steady-state compression events: advance every layer to the end of its period (eager),
    #     then time select / match / merge with HIP events on the launch stream.
    comp = {"select": [], "match": [], "merge": []}
    for layer in range(R):
        c = caches[layer][cur[layer]]
        while since[layer] != P:
            decode(c, layer, step_no[layer] % per_layer, since[layer])
            step_no[layer] += 1
            since[layer] += 1
    #     First the whole event of every layer, back to back inside one graph (the way the timed region launches
    #     them; an event reads its layer's cache and writes the other buffer, so replaying it changes nothing
    #     that the eager events below depend on): elapsed / layers = one event without host launch gaps.
    torch.cuda.synchronize()
    dropped_saved = dropped.clone()
    egraph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(egraph, stream=stream):
        for layer in range(R):
            compress(caches[layer][cur[layer]], caches[layer][1 - cur[layer]], layer, ws)
    torch.cuda.synchronize()
    g0, g1 = ev(), ev()
    with torch.cuda.stream(stream):
        egraph.replay()
        g0.record()
        egraph.replay()
        g1.record()
    torch.cuda.synchronize()
    event_graph_us = g0.elapsed_time(g1) * 1e3 / R
    dropped.copy_(dropped_saved)
    for layer in range(R):
        c = caches[layer][cur[layer]]
        since[layer] = 0
        d = caches[layer][1 - cur[layer]]
        e = [ev() for _ in range(4)]
        e[0].record()
        kk.select(lay, c, Bud, w.n_sink, w.n_recent, alpha, keep, evict_s, n_ev, ws)
        e[1].record()
        kk.match(lay, c, Bud, keep, evict_s, n_ev, T, match_s, None, ws)
        e[2].record()
        kk.merge(lay, c, d, Bud, keep, evict_s, n_ev, match_s, alpha, dropped[layer], ws)
        e[3].record()
        torch.cuda.synchronize()
        for j, name in enumerate(("select", "match", "merge")):
            comp[name].append(e[j].elapsed_time(e[j + 1]) * 1e3)
        cur[layer] = 1 - cur[layer]
    # (2) the decode kernel: a graph of decode steps only (every layer now sits at len = budget, so
    #     P/2 steps per layer stay inside the period), HIP events around the replay on the stream the
    #     kernels run on; average duration = elapsed / launches (back-to-back launches, no host gaps).
    n_dec = R * (P // 2)
    dgraph = torch.cuda.CUDAGraph()
    base_step = list(step_no)
    with torch.cuda.graph(dgraph, stream=stream):
        for i in range(n_dec):
            layer = i % R
            decode(caches[layer][cur[layer]], layer, (base_step[layer] + i // R) % per_layer, i // R)
    torch.cuda.synchronize()
    d0, d1 = ev(), ev()
    with torch.cuda.stream(stream):
        d0.record()
        dgraph.replay()
        d1.record()
    torch.cuda.synchronize()
    dec_us = d0.elapsed_time(d1) * 1e3 / n_dec
    live_mean = Bud + (P // 2 + 1) / 2.0          # slots per head attended, averaged over the replay
    slots = B * H * live_mean

    # algorithmic bytes of one launch.  Per live slot: K and V rows and votes (4 B); the unfused attention
    # call also writes the logit that feeds the EMA (4 B), the fused step instead reads and writes the EMA
    # state in place (ln S and n: 16 B) and keeps the logit on chip.  Plus Q in and O out.
    dec_bytes = slots * (2 * D * esz + 4 + (4 if args.unfused else 16)) + 2 * B * Hq * D * esz
    achieved = dec_bytes / (dec_us * 1e-6) / 1e9

    # what the GPU sustains on plain work of the same size (one launch reading a buffer as large as the decode
    # working set, 32 distinct buffers in rotation, same number of workgroups), on a large stream, and on
    # back-to-back bf16 MFMAs -- context for the fractions of the published peaks
    def graph_time(fn, n_launch, reps=4):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            fn()
        torch.cuda.synchronize()
        t0_, t1_ = ev(), ev()
        with torch.cuda.stream(stream):
            g.replay()
            t0_.record()
            for _ in range(reps):
                g.replay()
            t1_.record()
        torch.cuda.synchronize()
        return t0_.elapsed_time(t1_) * 1e3 / (reps * n_launch)

    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    ws_bytes = int(dec_bytes) // 16 * 16
    bufs = [torch.randint(0, 255, (ws_bytes,), dtype=torch.uint8, device=dev) for _ in range(R)]
    n_wg = B * H * ((cap + 127) // 128)
    small_us = graph_time(lambda: [kk.probe_read(b_, n_wg, sink) for b_ in bufs], R)
    del bufs
    big_buf = torch.randint(0, 255, (1 << 30,), dtype=torch.uint8, device=dev)
    big_us = graph_time(lambda: [kk.probe_read(big_buf, 4096, sink) for _ in range(2)], 2)
    del big_buf
    flops_box = []
    mfma_us = graph_time(lambda: flops_box.append(kk.probe_mfma(2048, 2000, sink)), 1)
    # the same instruction stream on random bf16 operands: the clock that the part sustains depends on the data
    mfma_rand_us = graph_time(lambda: flops_box.append(kk.probe_mfma(2048, 2000, sink, True)), 1)
    measured = {"read_decode_working_set_GBps": round(ws_bytes / small_us / 1e3, 1),
                "read_1GiB_GBps": round((1 << 30) / big_us / 1e3, 1),
                "mfma_bf16_TFLOPs": round(flops_box[-1] / mfma_us / 1e6, 1),
                "mfma_bf16_random_operands_TFLOPs": round(flops_box[-1] / mfma_rand_us / 1e6, 1)}
    roofline = {"bound": "hbm", "kernel": "decode_mfma_kernel" if bf16 else "decode_attn_kernel", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": (PMC_TRAFFIC_BYTES.get(w.name) if not args.unfused else None), "bytes_per_launch": int(dec_bytes),
                "avg_launch_us": round(dec_us, 2),
                "frac_of_measured_read": round(achieved / measured["read_decode_working_set_GBps"], 4)}

    M1 = N - Bud
    match_first_us = float(np.median(first["match"]))
    # window pass: keys read once, (log_s, n_obs) read and written, per slot of the uncompressed cache
    win_bytes = B * H * N * (D * (2 if w.dtype == "bf16" else 4) + 16) * len(range(0, w.window, win_chunk))
    win_gbs = win_bytes / (float(np.median(first["score_window"])) * 1e-6) / 1e9
    match_first_tflops = 2.0 * M1 * Bud * D * B * H / (match_first_us * 1e-6) / 1e12

    # ------------------------------------------------------------------ CPU baseline: the oracle on one layer
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import keepkv_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = 1
        src = caches[0][cur[0]]
        oc = O.Cache(B, H, cap, D)
        f = (lambda t_: W.from_bf16_bits(t_.view(torch.int16).cpu().numpy().view(np.uint16))) if bf16 else (lambda t_: t_.cpu().numpy())
        oc.k[:], oc.v[:] = f(src.k), f(src.v)
        oc.votes[:], oc.n_obs[:], oc.len[:] = src.votes.cpu().numpy(), src.n_obs.cpu().numpy(), src.len.cpu().numpy()
        oc.log_S[:] = src.log_s.cpu().numpy().astype(np.float64)
        room = cap - int(oc.len.max())
        n_cpu = 2 * P
        tc = time.perf_counter()
        done = 0
        for t in range(n_cpu):
            if int(oc.len.max()) == cap:
                O.compress(oc, Bud, w.n_sink, w.n_recent, alpha, T, exact_any_order=bf16,
                           storage_round=(W.round_bf16 if bf16 else None))
            k_t, v_t = W.make_token(w, 0, t)
            oc.append(k_t, v_t)
            q = W.make_query(w, 0, t).astype(np.float64)
            _, _, lg = O.attend(oc, q, w.scale)
            O.observe(oc, lg, alpha)
            done += 1
            if time.perf_counter() - tc > 30.0:
                break
        dt = time.perf_counter() - tc
        cpu = {"value": round(B * done / dt, 1), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": f"one layer, {done} decode steps of the same workload (append, attention, score; "
                         f"a compression event every {P} steps), numpy float64"}

    tokens_per_s = B * K / (elapsed_ms * 1e-3)
    res = {
        "metric": "decode attn tokens/s + compress us/layer at 10% budget; % HBM/MFMA roofline",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(elapsed_ms / K, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} Hq={Hq} Hkv={H} D={D} {w.dtype}, context {N} -> budget {Bud} "
                               f"({w.ratio:.0%}), period {P}, T={T:g}, alpha={alpha:g}",
                   "layers_rotated": R, "graph": not args.no_graph, "fused_step": not args.unfused, "compress_events_timed": timed_events,
                   "compress_overlapped": args.overlap},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels_us": {
            "decode_step": round(dec_us, 2),
            "compress_steady": {k_: (round(float(np.median(v_)), 1) if v_ else None) for k_, v_ in comp.items()},
            "compress_steady_event_in_graph": round(event_graph_us, 1),
            "compress_first": {k_: round(float(np.median(v_)), 1) for k_, v_ in first.items()},
        },
        "match_first_event": {"bound": "mfma", "achieved": round(match_first_tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                              "unit": "TFLOP/s", "frac": round(match_first_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                              "frac_of_measured_mfma": round(match_first_tflops / measured["mfma_bf16_TFLOPs"], 4),
                              "frac_of_measured_mfma_random_operands":
                                  round(match_first_tflops / measured["mfma_bf16_random_operands_TFLOPs"], 4)},
        "measured_rates": measured,
        "score_window_prefill": {"bound": "hbm", "achieved": round(win_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": round(win_gbs / HBM_PEAK_GBS, 4)},
        "prefill_s": round(t_prefill, 1),
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
