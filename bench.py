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
(batch x steps / median time of five replays of the K-step graph; how many compression events fell into the K
steps is `config.compress_events_timed`, and `decode_tokens_per_s`, `compress_us_per_layer` and
`tokens_per_s_with_events_amortised` give the metric's two halves whatever K is), with a `roofline` object for the decode-attention kernel and a
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
N_REPLAY = 5               # timed replays of the K-step graph; the median is reported
MFMA_BF16_PEAK_TFLOPS = 2500.0


def traffic_from_profile(workload: str, kernel: str):
    """HBM bytes per launch of the decode kernel as recorded in profiles/decode_hbm_traffic_<workload>.md
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads
    for a plain copy of known size).  Counters cannot be read from inside this process; the recorded figure
    is used only if the summary is for exactly the kernel instance this run launches, else None."""
    import re
    path = os.path.join(ROOT, "profiles", f"decode_hbm_traffic_{workload}.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"<!--\s*bench:\s*kernel=(\S+)\s+fetch_kib=([0-9.]+)\s+write_kib=([0-9.]+)\s+fetch_factor=([0-9.]+)\s+"
                  r"write_factor=([0-9.]+)\s*-->", text)
    if not m or m.group(1) != kernel:
        return None
    fetch, write, ff, wf = (float(m.group(i)) for i in range(2, 6))
    return int((fetch * ff + write * wf) * 1024)


def _limit_blas_threads():
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except Exception:
        pass


def oracle_units_worker(job):
    """cpu_baseline leg (runs in a process of its own that imports numpy, the oracle and the input generators
    only): decode steps of one layer on a subset of its (batch, kv head) units, starting from a cache of
    `budget` tokens of the workload's recipe; returns its wall time."""
    import time as _t

    import numpy as _np

    from oracle import keepkv_oracle as O
    from paper_2504_09936_amd import workloads as W
    w = W.CONFIGS[job["workload"]]
    units, n_steps, alpha, T = job["units"], job["n_steps"], job["alpha"], job["T"]
    bf16 = w.dtype == "bf16"
    G, Bud, cap = w.group, w.budget, w.budget + w.period
    K0, V0 = W.make_cache(w.scaled(context=Bud), 0)
    caches = []
    for b, h in units:
        oc = O.Cache(1, 1, cap, w.head_dim)
        oc.k[0, 0, :Bud], oc.v[0, 0, :Bud] = K0[b, h], V0[b, h]
        oc.votes[0, 0, :Bud] = 1
        oc.len[0, 0] = Bud
        caches.append(oc)
    del K0, V0
    t0 = _t.perf_counter()
    for t in range(n_steps):
        k_t, v_t = W.make_token(w, 0, t)
        q = W.make_query(w, 0, t).astype(_np.float64)
        for (b, h), oc in zip(units, caches):
            if int(oc.len[0, 0]) == cap:
                O.compress(oc, Bud, w.n_sink, w.n_recent, alpha, T, exact_any_order=bf16,
                           storage_round=(W.round_bf16 if bf16 else None))
            oc.append(k_t[b:b + 1, h:h + 1], v_t[b:b + 1, h:h + 1])
            _, _, lg = O.attend(oc, q[b:b + 1, h * G:(h + 1) * G], w.scale)
            O.observe(oc, lg, alpha)
    return _t.perf_counter() - t0


def run_cpu_baseline(w, alpha, T):
    """The oracle as it stands (numpy float64, a Python loop over (batch, kv head) units) on one layer of the
    workload: (i) one process with the BLAS pool held to one thread, (ii) one process per host core available
    to this process (affinity mask), the layer's units dealt over them.  Both run the same decode steps
    (append, attention, score; a compression event every period).  Runs before this process touches the GPU:
    the worker processes are started from a process that holds no GPU state."""
    import multiprocessing as mp
    B, H, P = w.batch, w.n_kv_heads, w.period
    n_aff = len(os.sched_getaffinity(0))
    all_units = [(b, h) for b in range(B) for h in range(H)]
    ctx = mp.get_context("spawn")

    def run_pool(n_proc, n_steps, units):
        shares = [units[i::n_proc] for i in range(n_proc)]
        shares = [u for u in shares if u]
        jobs = [{"workload": w.name, "units": u, "n_steps": n_steps, "alpha": alpha, "T": T} for u in shares]
        with ctx.Pool(len(shares), initializer=_limit_blas_threads) as pool:
            times = pool.map(oracle_units_worker, jobs)
        return max(times), len(shares)            # the slowest worker's loop: the job's time without process start-up

    # calibrate on a few units, then size both legs to about ten seconds each
    cal_units = all_units[:: max(1, len(all_units) // 4)][:4]
    t_cal, _ = run_pool(1, 8, cal_units)
    per_unit_step = max(t_cal, 1e-4) / (8 * len(cal_units))
    n1 = int(max(8, min(8 * P, 10.0 / (per_unit_step * len(all_units)))))
    t1, _ = run_pool(1, n1, all_units)
    n_proc = min(n_aff, len(all_units))
    nN = int(max(8, min(32 * P, 10.0 * n_proc / (per_unit_step * len(all_units)))))
    tN, used = run_pool(n_proc, nN, all_units)
    return {"value": round(B * nN / tN, 1), "unit": "tokens/s", "cores": int(used), "kind": "oracle",
            "sample": f"one layer of the same workload (a cache of {w.budget} tokens of its recipe), {nN} decode steps "
                      f"(append, attention, score; a compression event every {P} steps), numpy float64, the layer's "
                      f"{len(all_units)} (batch, kv head) units dealt over {used} processes of one thread each "
                      f"(affinity mask: {n_aff} cores)",
            "single_thread": {"value": round(B * n1 / t1, 1), "unit": "tokens/s", "cores": 1,
                              "sample": f"{n1} decode steps, one process, BLAS pool held to one thread"}}


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
    ap.add_argument("--events", choices=("auto", "inplace", "compact"), default="auto",
                    help="steady-state compression events: rewrite the cache into the layer's other buffer (compact) or "
                         "update it where it is (inplace: keepkv_select_aged / keepkv_merge_inplace).  auto = inplace "
                         "from 128 (batch, kv head) units on when a period has at most 256 steps")
    ap.add_argument("--unfused", action="store_true",
                    help="use keepkv_append + keepkv_decode_attn + keepkv_score instead of keepkv_decode_step")
    ap.add_argument("--window", type=int, default=None, help="observation passes before the first event")
    ap.add_argument("--decode-wavefronts", type=int, default=0, choices=(0, 4, 8, -1),
                    help="launch override of the decode kernel (keepkv_cache.plan_wavefronts): 4 or 8 wavefronts per "
                         "workgroup of the matrix-core kernel, -1 = the vector-ALU kernel on a bf16 cache; 0 = the plan's")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain device copy of known size (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (every (batch, kv head) cache is independent; "
              "kv heads or batch would shard across GPUs with no exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    from paper_2504_09936_amd import workloads as W
    cpu = None
    if not args.no_cpu_baseline and not args.copy_probe:
        w_ = W.CONFIGS[args.workload]
        cpu = run_cpu_baseline(w_, float(np.float32(w_.alpha)),
                               float(np.float32(w_.threshold if args.threshold is None else args.threshold)))

    import torch

    from paper_2504_09936_amd import binding as kk

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
    for pair in caches:
        for c in pair:
            c.plan_wavefronts = args.decode_wavefronts
    cur = [0] * R

    ev = lambda: torch.cuda.Event(enable_timing=True)

    # ------------------------------------------------------------------ prefill: window passes + first event per layer
    t0 = time.time()
    K0, V0 = W.make_cache(w, 0)
    K0d, V0d = to_dev(K0), to_dev(V0)
    del K0, V0
    first = {"score_window": [], "select": [], "match": [], "merge": []}
    merge_first = {"match": [], "merge": [], "receivers": None}
    win_chunk = max(1, 128 // (Hq // H))          # queries per keepkv_score_window call
    for layer in range(R):
        # layers are token/batch rotations of the seeded prefill tensors: same statistics, distinct bytes
        big.k.copy_(torch.roll(K0d, shifts=(layer, 257 * layer), dims=(0, 2)))
        big.v.copy_(torch.roll(V0d, shifts=(layer, 257 * layer), dims=(0, 2)))
        if w.query_model == "mean":
            big.k[:, :, 0] = K0d[:, :, 0]
        big.votes.fill_(1); big.log_s.fill_(float("-inf")); big.born.zero_(); big.t_obs.zero_(); big.len.fill_(N)
        # observation window (Eq. 8, t = L): all window queries in one pass over the keys
        q_win = to_dev(np.stack([W.make_query(w, layer, t - w.window) for t in range(w.window)], axis=2))
        e = [ev() for _ in range(4)]
        for j0 in range(0, w.window, win_chunk):
            j1 = min(w.window, j0 + win_chunk)
            kk.score_window(lay, big, q_win[:, :, j0:j1].contiguous() if (j0, j1) != (0, w.window) else q_win,
                            j1 - j0, alpha, -1)
        if layer < 2 and N <= 32768:
            # the merge-first prefill pass (App. B.4), timed on the same prefill cache; its output is not used
            # further: the timed decode loop continues from the usual (evict-first) event below
            if layer == 0:
                mf_near = torch.zeros(B, H, N, dtype=torch.int32, device=dev)
                mf_dst = kk.Cache(lay, N)
            p = [ev() for _ in range(3)]
            p[0].record()
            kk.prefill_match(lay, big, T, mf_near, None, ws)
            p[1].record()
            kk.prefill_merge(lay, big, mf_dst, mf_near, alpha, ws)
            p[2].record()
            torch.cuda.synchronize()
            merge_first["match"].append(p[0].elapsed_time(p[1]) * 1e3)
            merge_first["merge"].append(p[1].elapsed_time(p[2]) * 1e3)
            merge_first["receivers"] = float(mf_dst.len.float().mean().item())
            if layer == 1:
                del mf_near, mf_dst
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

    # In-place events: the cache keeps its buffer; `orders[layer]` lists the slots below the budget by age (the
    # first event wrote them in age order).
    # (auto: from 128 heads on, where rewriting the cache costs more than the in-place kernel's longer chain of
    # dependent loads; measured 44 against 39 us per event at 64 heads, 316 against 525 us at 1024)
    inplace = args.events == "inplace" or (args.events == "auto" and P <= 256 and B * H >= 128)
    orders = [torch.arange(Bud, dtype=torch.int32, device=dev).repeat(B, H, 1).contiguous() for _ in range(R)] if inplace else []

    def compress(c, d, layer, wsp):
        if inplace:
            kk.select_aged(lay, c, orders[layer], Bud, w.n_sink, w.n_recent, alpha, keep, evict_s, n_ev, wsp)
            kk.match(lay, c, Bud, keep, evict_s, n_ev, T, match_s, None, wsp)
            kk.merge_inplace(lay, c, orders[layer], Bud, keep, evict_s, n_ev, match_s, alpha, dropped[layer])
        else:
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
            if not inplace:
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
        # Every replay must run the K steps (and events) that were captured, on the state they were captured
        # for: appending the same tokens to a cache that already holds them would feed the events exact
        # duplicates.  The caches of all layers are put back before each replay (outside the timed region).
        fields = ("k", "v", "votes", "log_s", "born", "t_obs", "len")
        state_at_capture = [[{f_: getattr(c, f_).clone() for f_ in fields} for c in pair] for pair in caches]
        dropped_at_capture = dropped.clone()
        orders_at_capture = [o.clone() for o in orders]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(Wm, Wm + K):
                one_step(i)
            join_side()
        torch.cuda.synchronize()

        def restore_state():
            for pair, saved in zip(caches, state_at_capture):
                for c, st in zip(pair, saved):
                    for f_ in fields:
                        getattr(c, f_).copy_(st[f_])
            dropped.copy_(dropped_at_capture)
            for o, so in zip(orders, orders_at_capture):
                o.copy_(so)

        replay_ms = []
        for rep in range(1 + N_REPLAY):           # one untimed replay first
            restore_state()
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                start.record()
                graph.replay()
                stop.record()
            torch.cuda.synchronize()
            if rep > 0:
                replay_ms.append(start.elapsed_time(stop))
    if args.no_graph:
        replay_ms = [start.elapsed_time(stop)]
    elapsed_ms = float(np.median(replay_ms))
    if not args.no_graph:
        del state_at_capture
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
    #     (an in-place event changes its cache: the caches and slot lists are put back before every replay)
    torch.cuda.synchronize()
    dropped_saved = dropped.clone()
    ev_fields = ("k", "v", "votes", "log_s", "born", "t_obs", "len")
    ev_saved = [{f_: getattr(caches[layer][cur[layer]], f_).clone() for f_ in ev_fields} for layer in range(R)] if inplace else []
    ev_orders = [o.clone() for o in orders]

    def ev_restore():
        for layer in range(len(ev_saved)):
            for f_ in ev_fields:
                getattr(caches[layer][cur[layer]], f_).copy_(ev_saved[layer][f_])
            orders[layer].copy_(ev_orders[layer])

    egraph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(egraph, stream=stream):
        for layer in range(R):
            compress(caches[layer][cur[layer]], caches[layer][1 - cur[layer]], layer, ws)
    torch.cuda.synchronize()
    eg_runs = []
    for rep in range(1 + N_REPLAY):
        ev_restore()
        torch.cuda.synchronize()
        g0, g1 = ev(), ev()
        with torch.cuda.stream(stream):
            g0.record()
            egraph.replay()
            g1.record()
        torch.cuda.synchronize()
        if rep > 0:
            eg_runs.append(g0.elapsed_time(g1) * 1e3 / R)
    event_graph_us = float(np.median(eg_runs))
    dropped.copy_(dropped_saved)
    ev_restore()
    del ev_saved
    for layer in range(R):
        c = caches[layer][cur[layer]]
        since[layer] = 0
        d = caches[layer][1 - cur[layer]]
        e = [ev() for _ in range(4)]
        e[0].record()
        if inplace:
            kk.select_aged(lay, c, orders[layer], Bud, w.n_sink, w.n_recent, alpha, keep, evict_s, n_ev, ws)
        else:
            kk.select(lay, c, Bud, w.n_sink, w.n_recent, alpha, keep, evict_s, n_ev, ws)
        e[1].record()
        kk.match(lay, c, Bud, keep, evict_s, n_ev, T, match_s, None, ws)
        e[2].record()
        if inplace:
            kk.merge_inplace(lay, c, orders[layer], Bud, keep, evict_s, n_ev, match_s, alpha, dropped[layer])
        else:
            kk.merge(lay, c, d, Bud, keep, evict_s, n_ev, match_s, alpha, dropped[layer], ws)
        e[3].record()
        torch.cuda.synchronize()
        for j, name in enumerate(("select", "match", "merge")):
            comp[name].append(e[j].elapsed_time(e[j + 1]) * 1e3)
        if not inplace:
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
    lens_dec = [c[cu].len.clone() for c, cu in zip(caches, cur)]
    dec_runs = []
    for rep in range(1 + N_REPLAY):
        for c, cu, l in zip(caches, cur, lens_dec):
            c[cu].len.copy_(l)
        torch.cuda.synchronize()
        d0, d1 = ev(), ev()
        with torch.cuda.stream(stream):
            d0.record()
            dgraph.replay()
            d1.record()
        torch.cuda.synchronize()
        if rep > 0:
            dec_runs.append(d0.elapsed_time(d1) * 1e3 / n_dec)
    dec_us = float(np.median(dec_runs))
    live_mean = Bud + (P // 2 + 1) / 2.0          # slots per head attended, averaged over the replay
    slots = B * H * live_mean

    # algorithmic bytes of one launch.  Per live slot: K and V rows and votes (4 B); the unfused attention
    # call also writes the logit that feeds the EMA (4 B), the fused step instead updates the EMA state in
    # place and keeps the logit on chip: ln S read and written (8 B) and the slot's observation count read and
    # written (8 B).  Plus Q in and O out.  This library keeps the count as (head's step counter - slot's
    # origin) and so moves no per-slot count in a decode step: `bytes_moved_per_launch` is the same sum without
    # those 8 B; `frac` stays on the algorithmic figure, `frac_of_moved_bytes` is the other one.
    dec_bytes = slots * (2 * D * esz + 4 + (4 if args.unfused else 16)) + 2 * B * Hq * D * esz
    dec_bytes_moved = slots * (2 * D * esz + 4 + (4 if args.unfused else 8)) + 2 * B * Hq * D * esz
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
    ns_, per_, wv_ = kk.decode_plan(lay, cap)
    if args.decode_wavefronts in (4, 8):
        wv_ = args.decode_wavefronts
    if bf16 and args.decode_wavefronts == -1:
        kernel_instance = "decode_attn_kernel (vector ALU, bf16)"
    elif bf16:
        kernel_instance = (f"decode_mfma_kernel<{D},{Hq // H},{'false' if args.unfused else 'true'},"
                           f"{'true' if per_ <= wv_ * 32 else 'false'},{wv_}>")
    else:
        kernel_instance = "decode_attn_kernel"
    traffic = traffic_from_profile(w.name, kernel_instance)
    roofline = {"bound": "hbm", "kernel": kernel_instance, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "bytes_per_launch": int(dec_bytes), "bytes_moved_per_launch": int(dec_bytes_moved),
                "frac_of_moved_bytes": round(dec_bytes_moved / (dec_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                "avg_launch_us": round(dec_us, 2),
                "frac_of_measured_read": round(achieved / measured["read_decode_working_set_GBps"], 4)}

    M1 = N - Bud
    match_first_us = float(np.median(first["match"]))
    # window pass: keys read once, log_s read and written, per slot of the uncompressed cache
    win_bytes = B * H * N * (D * (2 if w.dtype == "bf16" else 4) + 16) * len(range(0, w.window, win_chunk))
    win_gbs = win_bytes / (float(np.median(first["score_window"])) * 1e-6) / 1e9
    match_first_tflops = 2.0 * M1 * Bud * D * B * H / (match_first_us * 1e-6) / 1e12

    # ------------------------------------------------------------------ CPU baseline: the oracle on one layer
    tokens_per_s = B * K / (elapsed_ms * 1e-3)
    first_event_us = sum(float(np.median(first[k_])) for k_ in ("select", "match", "merge"))
    # the metric's two halves, independent of how many events fell into the K timed steps: the decode step
    # alone, and a step with one steady-state event per `period` steps of a layer amortised in
    amortised_us = dec_us + event_graph_us / P
    res = {
        "metric": "decode attn tokens/s + compress us/layer at 10% budget; % HBM/MFMA roofline",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(elapsed_ms / K, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} Hq={Hq} Hkv={H} D={D} {w.dtype}, context {N} -> budget {Bud} "
                               f"({w.ratio:.0%}), period {P}, T={T:g}, alpha={alpha:g}",
                   "layers_rotated": R, "graph": not args.no_graph, "fused_step": not args.unfused, "compress_events_timed": timed_events,
                   "compress_overlapped": args.overlap, "steady_events": "in place" if inplace else "compacting"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "decode_tokens_per_s": round(B / (dec_us * 1e-6), 1),
        "compress_us_per_layer": {"steady_event": round(event_graph_us, 1), "first_event": round(first_event_us, 1),
                                  "period": P},
        "tokens_per_s_with_events_amortised": round(B / (amortised_us * 1e-6), 1),
        "timed_replays_ms": [round(x, 4) for x in replay_ms],
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
        "prefill_merge_first_pass": (None if not merge_first["match"] else {
            "match_us": round(float(np.median(merge_first["match"])), 1),
            "merge_us": round(float(np.median(merge_first["merge"])), 1),
            "match_TFLOPs": round(B * H * N * (N - 1) * D / (float(np.median(merge_first["match"])) * 1e-6) / 1e12, 1),
            "slots_left_per_head": round(merge_first["receivers"], 1), "threshold": T}),
        "measured_rates": measured,
        "score_window_prefill": {"bound": "hbm", "achieved": round(win_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": round(win_gbs / HBM_PEAK_GBS, 4)},
        "prefill_s": round(t_prefill, 1),
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
