#!/usr/bin/env python3
"""Benchmark of the mixed action+decode attention step on one MI355X.

A "step" is one pass of the whole hot path over one batch: host batch build (block
tables, slots, work list, one descriptor upload) and, for each of the 18 layers, the
KV append of the new tokens followed by the mixed attention launch.  The default
workload is the stress configuration (64 decode streams with own histories
~U{1..2048} on 8 shared 2048-token prefixes, plus two 50-query action chunks, pool
fragmented by seeded churn), because it is the one configuration whose 18 distinct
layers (about 1.5 GB of live KV) cannot sit in the 256 MB memory-side cache, so the
HBM roofline means something.  All inputs are synthetic, seeded, and resident in HBM
before the timed region starts.

Prints ONE JSON line.  `value` is microseconds per 18-layer mixed step.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, vendor figure
TOKEN_BYTES = 1024          # K + V of one token in one layer: 2 * 256 * 2 B
QO_BYTES = 2 * 8 * 256 * 2  # one query token read + one output token written


def _build_state(workload, device, split_tokens, stream_split_tokens=0, max_partials=16384):
    """Replays the set-up part of a trace (everything before its first attended step) with
    random resident data; returns the world and the remaining steps."""
    import torch
    from paper_2603_14371_amd import binding as B
    from paper_2603_14371_amd.harness import GpuWorld
    w = workload
    gw = GpuWorld(w, None, device=device, split_tokens=split_tokens,
                  stream_split_tokens=stream_split_tokens, want_lse=False,
                  max_partials=max_partials)
    gen = torch.Generator(device=device)
    gen.manual_seed(w["seed"])
    L = w["n_layers"]
    stream = torch.cuda.current_stream(device).cuda_stream
    rest = []
    for i, op in enumerate(w["trace"]):
        k = op["op"]
        if k == "step" and op.get("attend", True):
            rest = w["trace"][i:]
            break
        if k == "prefix_append":
            for layer in range(L):
                kv = torch.randn((2, op["n"], 256), device=device, generator=gen).to(torch.bfloat16)
                B.oxy_prefix_append(gw.pool, op["pid"], layer, kv[0].data_ptr(), kv[1].data_ptr(),
                                    op["n"], op["pos0"], stream)
            torch.cuda.synchronize(device)
        elif k == "step":
            n_tok = sum(n for _, n in op["items"])
            batch = B.oxy_batch_build(gw.pool, op["items"], B.BATCH_APPEND_ONLY, stream)
            if not op.get("churn"):
                for layer in range(L):
                    kv = torch.randn((2, n_tok, 256), device=device, generator=gen).to(torch.bfloat16)
                    B.oxy_stream_append(gw.pool, batch, layer, kv[0].data_ptr(), kv[1].data_ptr(),
                                        stream)
                torch.cuda.synchronize(device)
            B.oxy_batch_destroy(batch)
        else:
            gw.apply(op)
    return gw, rest


class StepRunner:
    """Holds resident per-layer inputs for a fixed batch shape and runs whole steps."""

    def __init__(self, gw, n_tok, device, seed):
        import torch
        self.gw = gw
        self.L = gw.n_layers
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        mk = lambda *shape: torch.randn(shape, device=device, generator=gen).to(torch.bfloat16)
        self.k = mk(self.L, n_tok, 256)
        self.v = mk(self.L, n_tok, 256)
        self.q = mk(self.L, n_tok, 8, 256)
        self.o = torch.empty_like(self.q)
        self.stream = torch.cuda.current_stream(device).cuda_stream
        self.n_tok = n_tok

    def step(self, items, events=None, mode="fold", graph=False):
        """One whole step: batch build, then append + attention for every layer (the per-layer
        loop runs below the ABI in oxy_step_layers).  mode: "fold" = the attention work items
        write the new rows themselves (two launches per layer), "separate" = append, work items,
        merge (three launches), "fuse" = the merge of layer l shares a launch with the append of
        layer l+1 (only possible because all layers' K/V are resident here).  graph: the
        launches of the step are recorded once per batch shape and replayed with one graph
        launch (OXY_STEP_GRAPH)."""
        from paper_2603_14371_amd import binding as B
        gw = self.gw
        flags = {"fold": B.STEP_FOLD_APPEND, "separate": 0, "fuse": B.STEP_FUSE_ACROSS_LAYERS}[mode]
        if graph:
            flags |= B.STEP_GRAPH
        batch = B.oxy_batch_build(gw.pool, items, 0, self.stream)
        B.oxy_step_layers(gw.pool, batch, 0, self.L, self.k.data_ptr(), self.v.data_ptr(),
                          self.k.stride(0) * 2, self.q.data_ptr(), self.o.data_ptr(),
                          self.q.stride(0) * 2, 0, 0, gw.scale, flags, events, self.stream)
        B.oxy_batch_destroy(batch)


class EventSet:
    """Timing events of one step, handed to the library as raw handles: for the layers in `timed`
    (all, if None) the begin and end of the work-item kernel and of the merge kernel (the
    kernels' own timestamps); the other layers are launched as in the untimed run.  Timing only
    a few layers per step keeps the timed launches inside a normal back-to-back sequence: with
    events on every launch the sequence is serialised by the event packets, and each kernel runs
    ~5 % slower than it does in the run that `value` times."""

    def __init__(self, n_layers, timed=None):
        import ctypes
        import torch
        self.layers = list(range(n_layers)) if timed is None else sorted(set(timed))
        self.ev = {}
        raw = [None] * (4 * n_layers)
        for layer in self.layers:
            for j in range(4):
                e = torch.cuda.Event(enable_timing=True)
                e.record()          # creates the underlying hipEvent_t
                self.ev[(layer, j)] = e
                raw[4 * layer + j] = e.cuda_event
        self.raw = (ctypes.c_void_p * len(raw))(*raw)

    def work_us(self):
        return [self.ev[(l, 0)].elapsed_time(self.ev[(l, 1)]) * 1e3 for l in self.layers]

    def merge_us(self):
        return [self.ev[(l, 2)].elapsed_time(self.ev[(l, 3)]) * 1e3 for l in self.layers]


def _live_kv_tokens(gw, items):
    """Unique KV tokens one layer of this step has to read: every distinct prefix once plus
    every item's own tokens (after the step's append)."""
    from paper_2603_14371_amd import binding as B
    prefixes = {}
    own = 0
    for sid, n_new in items:
        pid, kind, own_len, _ = B.oxy_stream_info(gw.pool, sid)
        if pid != -1:
            prefixes[pid] = B.oxy_prefix_info(gw.pool, pid)[0]
        own += n_new if kind == B.KIND_ACTION else own_len + n_new
    return sum(prefixes.values()) + own


def bench_stress(args, device, workload=None, alt_schedules=True):
    import torch
    from paper_2603_14371_amd import synth
    w = workload or synth.stress(mixed_steps=2 * args.warmup + 9 * args.steps + 2)
    t0 = time.time()
    n_streams = max(len(op["items"]) for op in w["trace"] if op["op"] == "step")
    gw, rest = _build_state(w, device, args.split_tokens, args.stream_split_tokens,
                            max_partials=max(16384, 64 * n_streams))
    setup_s = time.time() - t0
    steps = [op for op in rest if op["op"] == "step"]
    items = steps[0]["items"]
    n_tok = sum(n for _, n in items)
    n_decode = sum(1 for sid, n in items if n == 1)
    runner = StepRunner(gw, n_tok, device, w["seed"] + 1)
    for i in range(args.warmup):
        runner.step(steps[i]["items"])
    kv0 = _live_kv_tokens(gw, steps[args.warmup]["items"])
    # ---- timed region: exactly `steps` whole steps, no per-kernel instrumentation
    torch.cuda.synchronize(device)
    host_us = []
    t_start = time.perf_counter()
    for i in range(args.steps):
        h0 = time.perf_counter()
        runner.step(steps[args.warmup + i]["items"])
        host_us.append((time.perf_counter() - h0) * 1e6)
    torch.cuda.synchronize(device)
    step_us = (time.perf_counter() - t_start) / args.steps * 1e6
    # ---- spread: four more blocks of `steps` steps each, timed the same way
    block_us = [step_us]
    for blk in range(4 if alt_schedules else 0):
        first = 2 * args.warmup + (5 + blk) * args.steps
        torch.cuda.synchronize(device)
        t_start = time.perf_counter()
        for i in range(args.steps):
            runner.step(steps[first + i]["items"])
        torch.cuda.synchronize(device)
        block_us.append((time.perf_counter() - t_start) / args.steps * 1e6)
    # ---- the same steps again with HIP events around two layers' launches per step (on the
    # stream the kernels run on) for the roofline figure
    L = gw.n_layers
    sets = [EventSet(L, timed=[(7 * i) % L, (7 * i + L // 2) % L]) for i in range(args.steps)]
    torch.cuda.synchronize(device)
    t_start = time.perf_counter()
    for i in range(args.steps):
        runner.step(steps[args.warmup + args.steps + i]["items"], sets[i].raw)
    torch.cuda.synchronize(device)
    step_us_ev = (time.perf_counter() - t_start) / args.steps * 1e6
    # ---- and with the other launch schedules: three launches per layer, and the cross-layer
    # fusion (merge l + append l+1 in one launch)
    other = {}
    for j, mode in enumerate(("separate", "fuse")):
        if args.no_alt_schedules or not alt_schedules:
            other[mode] = float("nan")
            continue
        torch.cuda.synchronize(device)
        t_start = time.perf_counter()
        for i in range(args.steps):
            runner.step(steps[args.warmup + (2 + j) * args.steps + i]["items"], mode=mode)
        torch.cuda.synchronize(device)
        other[mode] = (time.perf_counter() - t_start) / args.steps * 1e6
    # ---- and the two-launch schedule recorded and replayed (one graph launch per step)
    if args.no_alt_schedules or not alt_schedules:
        other["fold_graph"] = float("nan")
    else:
        first = args.warmup + 4 * args.steps
        for i in range(args.warmup):
            runner.step(steps[first + i]["items"], graph=True)
        torch.cuda.synchronize(device)
        host_graph = []
        t_start = time.perf_counter()
        for i in range(args.steps):
            h0 = time.perf_counter()
            runner.step(steps[first + args.warmup + i]["items"], graph=True)
            host_graph.append((time.perf_counter() - h0) * 1e6)
        torch.cuda.synchronize(device)
        other["fold_graph"] = (time.perf_counter() - t_start) / args.steps * 1e6
        other["host_graph"] = float(np.mean(host_graph))
        from paper_2603_14371_amd import binding as B
        other["graph_stats"] = B.oxy_step_graph_stats(gw.pool)
    attn_us = [t for es in sets for t in es.work_us()]
    attn_avg_us = float(np.mean(attn_us))
    merge_avg_us = float(np.mean([t for es in sets for t in es.merge_us()]))
    # every step appends one token per decode stream: unique KV tokens of the instrumented steps
    kv_tokens = kv0 + n_decode * (args.steps + (args.steps - 1) / 2.0)
    alg_bytes = kv_tokens * TOKEN_BYTES + n_tok * QO_BYTES
    achieved = alg_bytes / (attn_avg_us * 1e-6) / 1e9
    res = {
        "step_us": step_us,
        "step_us_blocks": [round(b, 2) for b in block_us],
        "step_us_with_events": step_us_ev,
        "step_us_separate": other["separate"],
        "step_us_fused": other["fuse"],
        "step_us_graph": other["fold_graph"],
        "graph_stats": other.get("graph_stats"),
        "host_us_per_step_graph": other.get("host_graph", float("nan")),
        "attn_launch_us": attn_avg_us,
        "merge_launch_us": merge_avg_us,
        "alg_bytes_per_launch": alg_bytes,
        "kv_gbps": achieved,
        "decode_tokens_per_s": n_decode / (step_us * 1e-6),
        "host_us_per_step": float(np.mean(host_us)),
        "n_q_tokens": n_tok,
        "setup_s": setup_s,
        "unique_kv_tokens": kv_tokens,
    }
    gw.close()
    return res


def bench_sweep(args, device, series=((0, 0, (64, 128, 256, 512)), (512, 512, (64, 128, 256, 512)),
                                      (1024, 1024, (512, 1024, 2048)))):
    """The stress geometry at growing stream counts (groups of 8 streams per 2048-token prefix,
    own histories ~U{1..2048}, two action chunks): where the work-item kernel gets to on the
    HBM roofline as a launch grows.  The number of layers shrinks as the streams grow so that
    every point cycles through at least ~1.5 GB of distinct KV (the memory-side cache holds
    256 MB) without filling the card.  Three series (split_tokens, stream_split_tokens, stream
    counts): the default split sizes of the pool (256 tokens per work item on these lengths, what
    the 64-stream launch needs to fill the chip), 512-token work items, which pay off once a
    launch has several times more work items than the chip holds at once, and 1024-token work
    items (the largest the pool accepts) on launches of 0.7 to 2.7 GB: the rate the kernel
    settles at when the fixed cost of a launch no longer counts."""
    import argparse as _ap
    import torch
    from paper_2603_14371_amd import synth
    out = []
    for split, stream_split, counts in series:
        for n in counts:
            layers = max(3, -(-18 * 64 // n))
            blocks = 8192 * n // 64
            a = _ap.Namespace(**vars(args))
            a.steps, a.warmup = max(4, args.steps // 2), 2
            a.split_tokens = split or args.split_tokens
            a.stream_split_tokens = stream_split or args.stream_split_tokens
            w = synth.stress(n_layers=layers, n_streams=n, num_blocks=blocks,
                             mixed_steps=a.warmup + 2 * a.steps + 2)
            r = bench_stress(a, device, workload=w, alt_schedules=False)
            both = r["attn_launch_us"] + r["merge_launch_us"]
            out.append({"streams": n, "layers": layers,
                        "tokens_per_work_item": a.split_tokens or 256,
                        "alg_bytes_per_launch": round(r["alg_bytes_per_launch"]),
                        "attn_launch_us": round(r["attn_launch_us"], 2),
                        "merge_launch_us": round(r["merge_launch_us"], 2),
                        "gbps": round(r["kv_gbps"], 1),
                        "frac": round(r["kv_gbps"] / HBM_PEAK_GBPS, 4),
                        "frac_with_merge": round(r["alg_bytes_per_launch"] / (both * 1e-6) / 1e9
                                                 / HBM_PEAK_GBPS, 4),
                        "step_us": round(r["step_us"], 1)})
            torch.cuda.empty_cache()
    return out


def bench_frame(device, split_tokens, frames=3, graph=True):
    """pi0.5-shaped single frame (secondary figures): prefix append of 832 tokens x 18 layers,
    10 mixed steps (50-query chunk + 1 decode token), then 54 decode-only steps."""
    import torch
    from paper_2603_14371_amd import binding as B, synth
    w = synth.pi05_frame()
    trace = []                      # ids continue across the repeated frames
    for f in range(frames + 1):
        for op in synth.pi05_frame()["trace"]:
            op = dict(op)
            if "pid" in op and op["pid"] >= 0:
                op["pid"] += f
            if "sid" in op:
                op["sid"] += 2 * f
            if op["op"] == "step":
                op["items"] = [(s + 2 * f, n) for s, n in op["items"]]
            trace.append(op)
    w["trace"] = trace
    from paper_2603_14371_amd.harness import GpuWorld
    gw = GpuWorld(w, None, device=device, split_tokens=split_tokens, want_lse=False)
    L = gw.n_layers
    gen = torch.Generator(device=device)
    gen.manual_seed(1)
    pk = torch.randn((L, 2, 832, 256), device=device, generator=gen).to(torch.bfloat16)
    runner_mixed = StepRunner(gw, 51, device, 2)
    runner_dec = StepRunner(gw, 1, device, 3)
    stream = torch.cuda.current_stream(device).cuda_stream
    t_prefix, t_mixed, t_dec = [], [], []
    n_frame_ops = len(trace) // (frames + 1)
    for f in range(frames + 1):
        ops = trace[f * n_frame_ops:(f + 1) * n_frame_ops]
        torch.cuda.synchronize(device)
        marks = {"prefix": 0.0, "mixed": 0.0, "dec": 0.0}
        for op in ops:
            t0 = time.perf_counter()
            if op["op"] == "prefix_append":
                B.oxy_prefix_append_layers(gw.pool, op["pid"], 0, L, pk[0, 0].data_ptr(),
                                           pk[0, 1].data_ptr(), pk.stride(0) * 2, 832,
                                           0, stream)
                torch.cuda.synchronize(device)
                marks["prefix"] += time.perf_counter() - t0
            elif op["op"] == "step":
                if op["mixed"]:
                    runner_mixed.step(op["items"], graph=graph)
                else:
                    runner_dec.step(op["items"], graph=graph)
                # a real decode loop needs the token of step j before step j+1: sync per step
                torch.cuda.synchronize(device)
                marks["mixed" if op["mixed"] else "dec"] += time.perf_counter() - t0
            else:
                gw.apply(op)
        if f > 0:
            t_prefix.append(marks["prefix"])
            t_mixed.append(marks["mixed"])
            t_dec.append(marks["dec"])
    graph_stats = B.oxy_step_graph_stats(gw.pool)
    gw.close()
    mixed_us = float(np.mean(t_mixed)) / 10 * 1e6
    dec_us = float(np.mean(t_dec)) / 54 * 1e6
    t_action = float(np.mean(t_prefix)) + float(np.mean(t_mixed))
    return {
        "prefix_append_us": float(np.mean(t_prefix)) * 1e6,
        "mixed_step_us": mixed_us,
        "decode_only_step_us": dec_us,
        "action_hz": 1.0 / t_action,
        "actions_per_s": 50.0 / t_action,
        "decode_tokens_per_s_mixed": 1.0 / (mixed_us * 1e-6),
        "decode_tokens_per_s_decode_only": 1.0 / (dec_us * 1e-6),
        "launches": "one recorded graph per step" if graph else "two per layer from the host",
        "graph_instantiated_updated_replayed": list(graph_stats),
    }


def _frame_both(device, split_tokens):
    """The pi0.5 frame with two launches per layer issued from the host and, beside it, with
    every step replayed from its recording (one graph launch per step)."""
    rnd = lambda d: {k: (round(v, 2) if isinstance(v, float) else v) for k, v in d.items()}
    out = rnd(bench_frame(device, split_tokens, graph=False))
    out["recorded_graph"] = rnd(bench_frame(device, split_tokens, graph=True))
    return out


def bench_cross_task(device, split_tokens, n_steps=64, reps=3):
    """Cross-task sharing vs isolated execution on identical shapes: one refcounted 832-token
    prefix with one batch per step, against four prefix copies with one batch per task per step
    (the paper's "isolated execution" baseline).  Whole trace: prefix appends + n_steps steps."""
    import torch
    from paper_2603_14371_amd import binding as B, synth
    from paper_2603_14371_amd.harness import GpuWorld
    out = {}
    for name, isolated in (("shared", False), ("isolated", True)):
        times, blocks = [], 0
        for rep in range(reps + 1):
            w = synth.cross_task(isolated=isolated, n_steps=n_steps)
            gw = GpuWorld(w, None, device=device, split_tokens=split_tokens, want_lse=False,
                          max_q_tokens=64, max_append_tokens=1024)
            L = gw.n_layers
            gen = torch.Generator(device=device)
            gen.manual_seed(7)
            pk = torch.randn((L, 2, 832, 256), device=device, generator=gen).to(torch.bfloat16)
            runner = StepRunner(gw, 53, device, 8)
            stream = runner.stream
            torch.cuda.synchronize(device)
            t0 = time.perf_counter()
            for op in w["trace"]:
                if op["op"] == "prefix_append":
                    B.oxy_prefix_append_layers(gw.pool, op["pid"], 0, L, pk[0, 0].data_ptr(),
                                               pk[0, 1].data_ptr(), pk.stride(0) * 2, op["n"],
                                               op["pos0"], stream)
                elif op["op"] == "step":
                    runner.step(op["items"])
                elif "release" in op["op"]:
                    if blocks == 0:
                        blocks = w["num_blocks"] - B.oxy_pool_stats(gw.pool)[0]
                    gw.apply(op)
                else:
                    gw.apply(op)
            torch.cuda.synchronize(device)
            if rep > 0:
                times.append(time.perf_counter() - t0)
            gw.close()
        out[name + "_us"] = float(np.median(times)) * 1e6
        out[name + "_pool_blocks"] = blocks
    out["speedup_vs_isolated"] = out["isolated_us"] / out["shared_us"]
    out["steps"] = n_steps
    return out


def bench_cross_frame(device, split_tokens, frames=40, warm=16):
    """Config 2 as stated: 8 request slots carried across frames, targets ~U{16..512}, k = 10
    tokens per frame, a fresh 832-token prefix and one 50-query x 10-step chunk per frame, page
    16 on a shuffled free order, 18 layers.  Per frame: prefix KV write, fan-out, 10 mixed steps
    (host-synchronised per step, as a decode loop is), releases.  Frames after `warm` are timed:
    by then all eight slots are occupied and histories span 1..~400 own tokens."""
    import torch
    from paper_2603_14371_amd import binding as B, synth
    from paper_2603_14371_amd.harness import GpuWorld
    w = synth.cross_frame(n_frames=frames)
    gw = GpuWorld(w, None, device=device, split_tokens=split_tokens, want_lse=False)
    L = gw.n_layers
    gen = torch.Generator(device=device)
    gen.manual_seed(11)
    pk = torch.randn((L, 2, 832, 256), device=device, generator=gen).to(torch.bfloat16)
    runners = {}
    stream = torch.cuda.current_stream(device).cuda_stream
    frame_us, step_us, batch = [], [], []
    own = {}
    for f, (lo, hi) in enumerate(w["frames"]):
        torch.cuda.synchronize(device)
        t_frame = time.perf_counter()
        for op in w["trace"][lo:hi]:
            if op["op"] == "prefix_append":
                B.oxy_prefix_append_layers(gw.pool, op["pid"], 0, L, pk[0, 0].data_ptr(),
                                           pk[0, 1].data_ptr(), pk.stride(0) * 2, op["n"],
                                           op["pos0"], stream)
            elif op["op"] == "step":
                n_tok = sum(n for _, n in op["items"])
                if n_tok not in runners:
                    runners[n_tok] = StepRunner(gw, n_tok, device, 100 + n_tok)
                t0 = time.perf_counter()
                runners[n_tok].step(op["items"])
                torch.cuda.synchronize(device)
                if f >= warm:
                    step_us.append((time.perf_counter() - t0) * 1e6)
                    batch.append(len(op["items"]) - 1)
                for sid, n in op["items"]:
                    if n == 1:
                        own[sid] = own.get(sid, 0) + 1
            else:
                gw.apply(op)
        torch.cuda.synchronize(device)
        if f >= warm:
            frame_us.append((time.perf_counter() - t_frame) * 1e6)
    gw.close()
    fr = float(np.median(frame_us))
    return {"frames_timed": len(frame_us), "frame_us_median": fr,
            "frame_us_min": float(np.min(frame_us)), "frame_us_max": float(np.max(frame_us)),
            "mixed_step_us_median": float(np.median(step_us)),
            "decode_batch_mean": float(np.mean(batch)),
            "longest_own_history": int(max(own.values())),
            "action_hz": 1e6 / fr, "decode_tokens_per_s": float(np.mean(batch)) * 10 / (fr * 1e-6)}


def bench_action(args, device, n_chunks=8, chunk=50):
    """The action-chunk path alone: n_chunks chunks of 50 queries, each on a prefix of its own,
    no decode items -- the dense (MFMA) side of the method in isolation.  Two geometries: the
    pi0.5 prefix (832 tokens: prefix phase as streamed token pairs, chunk phase as tiles that
    read the step's new rows) and the stress prefix (2048 tokens: prefix phase as 8-token
    tiles).  Reports the work-item kernel's time per layer and its matrix-core rate: executed
    (counters, see profiles/) = what the kernel issues: row blocks padded to 16, P as hi+lo;
    algorithmic = 4*8*256 flop per (query token, visible key)."""
    import torch
    from paper_2603_14371_amd import synth
    out = {}
    for prefix_len in (832, 2048):
        b = synth._TraceBuilder()
        pids = [b.prefix(prefix_len) for _ in range(n_chunks)]
        acts = [b.stream(pid, synth.ACTION) for pid in pids]
        for _ in range(args.warmup + 2 * args.steps):
            b.step([(a, chunk) for a in acts], mixed=True)
        w = synth._workload("action_only", 14371700, 18, 2048, b.trace)
        gw, rest = _build_state(w, device, args.split_tokens, args.stream_split_tokens)
        steps = [op for op in rest if op["op"] == "step"]
        n_tok = n_chunks * chunk
        runner = StepRunner(gw, n_tok, device, 17)
        for i in range(args.warmup):
            runner.step(steps[i]["items"])
        torch.cuda.synchronize(device)
        t0 = time.perf_counter()
        for i in range(args.steps):
            runner.step(steps[args.warmup + i]["items"])
        torch.cuda.synchronize(device)
        step_us = (time.perf_counter() - t0) / args.steps * 1e6
        L = gw.n_layers
        sets = [EventSet(L, timed=[(7 * i) % L, (7 * i + L // 2) % L]) for i in range(args.steps)]
        for i in range(args.steps):
            runner.step(steps[args.warmup + args.steps + i]["items"], sets[i].raw)
        torch.cuda.synchronize(device)
        attn_us = float(np.mean([t for es in sets for t in es.work_us()]))
        merge_us = float(np.mean([t for es in sets for t in es.merge_us()]))
        flop = 4.0 * 8 * 256 * n_tok * (prefix_len + chunk)
        out["prefix_%d" % prefix_len] = {
            "q_tokens": n_tok, "step_us": round(step_us, 2), "attn_launch_us": round(attn_us, 2),
            "merge_launch_us": round(merge_us, 2),
            "algorithmic_gflop_per_launch": round(flop / 1e9, 3),
            "algorithmic_tflops": round(flop / (attn_us * 1e-6) / 1e12, 1),
            "frac_of_bf16_mfma_peak_algorithmic": round(flop / (attn_us * 1e-6) / 1e12 / 2500.0, 4),
        }
        gw.close()
    return out


def _arrival_patterns(frames, seed=14371300):
    """Arrival patterns of the paper's workload generalisation (Sec. 4.4): per frame the list
    of total decode lengths N of the observations that arrive (seeded, synthetic)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    pats = {"one_per_frame": [[60]] * frames}
    for r in (2, 4):
        pats["uniform_%d" % r] = [[60] * r] * frames
    for lam in (0.5, 1.0, 2.0):
        pats["poisson_%g" % lam] = [[60] * int(rng.poisson(lam)) for _ in range(frames)]
    for name, p_short in (("short1_long3", 0.25), ("short1_long1", 0.5), ("short3_long1", 0.75)):
        pats["lengths_" + name] = [[20 if rng.random() < p_short else 100] for _ in range(frames)]
    return pats


def bench_arrivals(device, split_tokens, frames=24, warm=12, k=10, s_act=10, chunk=50,
                   prefix_len=832):
    """Attention-only version of the paper's arrival-pattern sweep and ablation (Sec. 4.3-4.4):
    frames are driven by the library's scheduler; per pattern and variant the frame time, the
    per-request action frequency 1/T, the mean decode batch and the totals per second.  The
    prefill is represented by its KV write (prefix append) only; the host synchronises after
    every step, as a decode loop that samples on the host would."""
    import torch
    from paper_2603_14371_amd import binding as B, synth
    from paper_2603_14371_amd.harness import GpuWorld
    nb, L = 8192, 18
    w = synth._workload("arrivals", 14371300, L, nb, [])
    gw = GpuWorld(w, None, device=device, split_tokens=split_tokens, want_lse=False,
                  max_q_tokens=4 * chunk + 80, max_append_tokens=1024, max_partials=16384)
    gen = torch.Generator(device=device)
    gen.manual_seed(5)
    pk = torch.randn((L, 2, prefix_len, 256), device=device, generator=gen).to(torch.bfloat16)
    runner = StepRunner(gw, 4 * chunk + 80, device, 6)
    stream = runner.stream
    out = {}
    for pname, arrivals in _arrival_patterns(warm + frames).items():
        res = {}
        for mname, mode in (("batched", B.SCHED_BATCHED), ("unbatched", B.SCHED_UNBATCHED),
                            ("upper_bound", B.SCHED_UPPER_BOUND)):
            sched = B.oxy_sched_create(gw.pool, k, s_act, chunk, 64, mode)
            t_frames, n_dec_items, n_dec_steps, n_obs = [], 0, 0, 0
            for t, targets in enumerate(arrivals):
                torch.cuda.synchronize(device)
                t0 = time.perf_counter()
                for n in targets:
                    pid = B.oxy_prefix_create(gw.pool)
                    B.oxy_prefix_append_layers(gw.pool, pid, 0, L, pk[0, 0].data_ptr(),
                                               pk[0, 1].data_ptr(), pk.stride(0) * 2, prefix_len,
                                               0, stream)
                    B.oxy_sched_admit(sched, pid, n)
                while True:
                    items, n_action = B.oxy_sched_next_step(sched)
                    if not items:
                        break
                    runner.step(items)
                    torch.cuda.synchronize(device)
                    if t >= warm and len(items) > n_action:
                        n_dec_items += len(items) - n_action
                        n_dec_steps += 1
                B.oxy_sched_end_frame(sched)
                if t >= warm:
                    t_frames.append(time.perf_counter() - t0)
                    n_obs += len(targets)
            B.oxy_sched_destroy(sched)
            T = float(np.mean(t_frames))
            res[mname] = {
                "frame_ms": round(T * 1e3, 3),
                "action_hz_per_request": round(1.0 / T, 1),
                "avg_decode_batch": round(n_dec_items / max(1, n_dec_steps), 2),
                "actions_per_s": round(n_obs * chunk / sum(t_frames), 1),
                "decode_tokens_per_s": round(n_dec_items / sum(t_frames), 1),
            }
        # the paper's reference baseline: isolated sequential execution, no sharing, no batching
        # (one prefill copy per task, action steps alone, then the request alone to completion)
        t_frames, n_obs, n_dec = [], 0, 0
        for t, targets in enumerate(arrivals):
            if t < warm - 2:          # nothing carries over between frames here
                continue
            torch.cuda.synchronize(device)
            t0 = time.perf_counter()
            for n in targets:
                pids = []
                for _ in range(2):
                    pid = B.oxy_prefix_create(gw.pool)
                    B.oxy_prefix_append_layers(gw.pool, pid, 0, L, pk[0, 0].data_ptr(),
                                               pk[0, 1].data_ptr(), pk.stride(0) * 2, prefix_len,
                                               0, stream)
                    pids.append(pid)
                act = B.oxy_stream_create(gw.pool, pids[0], B.KIND_ACTION)
                dec = B.oxy_stream_create(gw.pool, pids[1], B.KIND_DECODE)
                for _ in range(s_act):
                    runner.step([(act, chunk)])
                    torch.cuda.synchronize(device)
                for _ in range(n):
                    runner.step([(dec, 1)])
                    torch.cuda.synchronize(device)
                B.oxy_stream_release(gw.pool, act)
                B.oxy_stream_release(gw.pool, dec)
                for pid in pids:
                    B.oxy_prefix_release(gw.pool, pid)
            if t >= warm:
                t_frames.append(time.perf_counter() - t0)
                n_obs += len(targets)
                n_dec += sum(targets)
        T = float(np.mean(t_frames))
        res["isolated_baseline"] = {
            "frame_ms": round(T * 1e3, 3), "action_hz_per_request": round(1.0 / T, 1),
            "avg_decode_batch": 1.0, "actions_per_s": round(n_obs * chunk / sum(t_frames), 1),
            "decode_tokens_per_s": round(n_dec / sum(t_frames), 1)}
        out[pname] = res
    gw.close()
    return out


def bench_calibration(device, split_tokens, targets_hz=(350.0, 300.0, 250.0), n_len=60, s_act=10,
                      chunk=50, prefix_len=832, reps=12):
    """Attention-only version of the offline calibration of the per-frame budget k (Sec. 3.2):
    measure the cost of a mixed step and of a decode-only step for every decode batch size,
    let the library pick the largest k whose steady-state frame meets a target frame rate, then
    run scheduler-driven frames with that k and report the measured frame time beside the
    modelled one."""
    import torch
    from paper_2603_14371_amd import binding as B, synth
    from paper_2603_14371_amd.harness import GpuWorld
    nb, L, bmax = 8192, 18, n_len
    w = synth._workload("calibration", 14371400, L, nb, [])
    gw = GpuWorld(w, None, device=device, split_tokens=split_tokens, want_lse=False,
                  max_q_tokens=chunk + bmax + 8, max_append_tokens=1024, max_partials=16384)
    gen = torch.Generator(device=device)
    gen.manual_seed(9)
    pk = torch.randn((L, 2, prefix_len, 256), device=device, generator=gen).to(torch.bfloat16)
    runner = StepRunner(gw, chunk + bmax + 8, device, 10)
    stream = runner.stream

    def new_prefix():
        pid = B.oxy_prefix_create(gw.pool)
        B.oxy_prefix_append_layers(gw.pool, pid, 0, L, pk[0, 0].data_ptr(), pk[0, 1].data_ptr(),
                                   pk.stride(0) * 2, prefix_len, 0, stream)
        return pid

    def timed(items):
        ts = []
        for i in range(reps + 3):
            torch.cuda.synchronize(device)
            t0 = time.perf_counter()
            runner.step(items)
            torch.cuda.synchronize(device)
            if i >= 3:
                ts.append(time.perf_counter() - t0)
        return float(np.median(ts)) * 1e6

    # cost tables: one action chunk on a fresh observation + b requests in mid-life, each on the
    # prefix of its own birth frame
    act_pid = new_prefix()
    act = B.oxy_stream_create(gw.pool, act_pid, B.KIND_ACTION)
    dec = []
    t_mixed, t_dec = [timed([(act, chunk)])], [0.0]
    for b in range(1, bmax + 1):
        sid = B.oxy_stream_create(gw.pool, new_prefix(), B.KIND_DECODE)
        batch = B.oxy_batch_build(gw.pool, [(sid, n_len // 2)], B.BATCH_APPEND_ONLY, stream)
        B.oxy_batch_destroy(batch)      # history of half a request (contents do not matter)
        dec.append(sid)
        if b <= 12 or b % 6 == 0 or b == bmax:
            t_mixed.append(timed([(act, chunk)] + [(s_, 1) for s_ in dec]))
            t_dec.append(timed([(s_, 1) for s_ in dec]))
        else:
            t_mixed.append(None)
            t_dec.append(None)
    for tab in (t_mixed, t_dec):        # batch sizes not measured: linear between neighbours
        known = [i for i, v in enumerate(tab) if v is not None]
        for i, v in enumerate(tab):
            if v is None:
                lo = max(j for j in known if j < i)
                hi = min(j for j in known if j > i)
                tab[i] = tab[lo] + (tab[hi] - tab[lo]) * (i - lo) / (hi - lo)
    torch.cuda.synchronize(device)
    t0 = time.perf_counter()
    for _ in range(5):
        pid = new_prefix()
    torch.cuda.synchronize(device)
    t_obs = (time.perf_counter() - t0) / 5 * 1e6
    B.oxy_stream_release(gw.pool, act)
    for sid in dec:
        B.oxy_stream_release(gw.pool, sid)
    out = {"t_observation_us": round(t_obs, 1),
           "t_mixed_us": {str(b): round(t_mixed[b], 1) for b in (0, 1, 2, 4, 6, 12, bmax)},
           "t_decode_us": {str(b): round(t_dec[b], 1) for b in (1, 2, 4, 6, 12, bmax)},
           "targets": []}
    for hz in targets_hz:
        k, model_us = B.oxy_sched_calibrate(t_mixed, t_dec, t_obs, s_act, n_len, 1, 1e6 / hz)
        rec = {"target_hz": hz, "k": k, "modelled_frame_us": round(model_us, 1)}
        if k > 0:
            sched = B.oxy_sched_create(gw.pool, k, s_act, chunk, 0, B.SCHED_BATCHED)
            warm = -(-n_len // k) + 2
            ts = []
            for t in range(warm + 16):
                torch.cuda.synchronize(device)
                f0 = time.perf_counter()
                B.oxy_sched_admit(sched, new_prefix(), n_len)
                while True:
                    items, _ = B.oxy_sched_next_step(sched)
                    if not items:
                        break
                    runner.step(items)
                    torch.cuda.synchronize(device)
                B.oxy_sched_end_frame(sched)
                if t >= warm:
                    ts.append(time.perf_counter() - f0)
            B.oxy_sched_destroy(sched)
            rec["measured_frame_us"] = round(float(np.mean(ts)) * 1e6, 1)
            rec["measured_hz"] = round(1.0 / float(np.mean(ts)), 1)
            rec["decode_tokens_per_s"] = round(n_len / float(np.mean(ts)), 1)
        out["targets"].append(rec)
    gw.close()
    return out


def stream_probe(device, n_bytes, layers=18, reps=5):
    """What a plain read-only streaming kernel reaches on this machine for the same bytes per
    launch as one attention launch (cycling over `layers` distinct regions so that nothing sits
    in the memory-side cache), and for a launch four times as large."""
    import torch
    from paper_2603_14371_amd import benchaid
    out = {}
    stream = torch.cuda.current_stream(device).cuda_stream
    sink = torch.zeros(64, dtype=torch.uint8, device=device)
    for label, nb in (("same_bytes", n_bytes), ("4x_bytes", 4 * n_bytes)):
        nb = (int(nb) // (128 * 1024)) * (128 * 1024)
        buf = torch.empty(layers * nb, dtype=torch.uint8, device=device).fill_(3)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(reps * layers)]
        torch.cuda.synchronize(device)
        for r in range(reps):
            for l in range(layers):
                a, b = ev[r * layers + l]
                a.record()
                benchaid.read(buf.data_ptr() + l * nb, nb, sink.data_ptr(), stream)
                b.record()
        torch.cuda.synchronize(device)
        us = [a.elapsed_time(b) * 1e3 for a, b in ev[layers:]]
        out[label] = {"bytes": nb, "us": round(float(np.mean(us)), 2),
                      "gbps": round(nb / (float(np.mean(us)) * 1e-6) / 1e9, 1)}
        del buf
    return out


def pmc_probe(device, reps=3, mib=256):
    """Plain copies of known size, so that traffic counters can be calibrated in the same run."""
    import torch
    from paper_2603_14371_amd import benchaid
    n = mib << 20
    src = torch.empty(n, dtype=torch.uint8, device=device).fill_(1)
    dst = torch.empty(n, dtype=torch.uint8, device=device)
    stream = torch.cuda.current_stream(device).cuda_stream
    for _ in range(reps):
        benchaid.copy(dst.data_ptr(), src.data_ptr(), n, stream)
    torch.cuda.synchronize(device)
    return n


def cpu_baseline(sample_layers=12):
    """The float64 oracle, as it stands, on one layer of a stress-shaped mixed step."""
    from oracle import attention
    from paper_2603_14371_amd import synth
    rng = np.random.default_rng(5)
    w = synth.stress(mixed_steps=1, churn_ops=0)
    hist = w["hist"]
    bits = lambda *shape: synth.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    prefixes = [(bits(2048, 256), bits(2048, 256)) for _ in range(8)]
    own = [(bits(h + 1, 256), bits(h + 1, 256)) for h in hist]
    qs = [bits(1, 8, 256) for _ in hist]
    chunk = [(bits(50, 256), bits(50, 256), bits(50, 8, 256)) for _ in range(2)]
    t0 = time.perf_counter()
    for _ in range(sample_layers):
        for i, (ko, vo) in enumerate(own):
            kp, vp = prefixes[i // 8]
            attention.attend_item(attention.DECODE, qs[i], kp, vp, ko, vo, 0.0625)
        for i, (kc, vc, qc) in enumerate(chunk):
            kp, vp = prefixes[i]
            attention.attend_item(attention.ACTION, qc, kp, vp, kc, vc, 0.0625)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return {"value": dt / sample_layers * 18 * 1e6, "unit": "us/step", "cores": int(threads),
            "kind": "oracle",
            "sample": "%d of 18 layers of one stress mixed step (attention only), scaled x18/%d; "
                      "host has %d cores" % (sample_layers, sample_layers, os.cpu_count())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--split-tokens", type=int, default=0)
    ap.add_argument("--stream-split-tokens", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-frame", action="store_true")
    ap.add_argument("--no-cross-task", action="store_true")
    ap.add_argument("--no-arrivals", action="store_true")
    ap.add_argument("--only-arrivals", action="store_true",
                    help="run only the arrival-pattern sweep (frames driven by the scheduler)")
    ap.add_argument("--no-alt-schedules", action="store_true",
                    help="profiling aid: skip the passes with the other launch schedules")
    ap.add_argument("--sweep-streams", action="store_true",
                    help="run only the stream-count sweep (64..2048 streams, stress geometry)")
    ap.add_argument("--only-stress", action="store_true",
                    help="profiling aid: the stress section only")
    ap.add_argument("--only-action", action="store_true",
                    help="only the action-chunk path in isolation (MFMA rate of the dense side)")
    ap.add_argument("--only-frame", action="store_true",
                    help="profiling aid: run only the pi0.5-shaped frame section")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="also launch plain 256 MiB copies (calibration of traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard by prefix group: a "
              "prefix and the streams attached to it per GPU); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    device = torch.device("cuda:0")
    if args.sweep_streams:
        print(json.dumps({"stream_sweep": bench_sweep(args, device)}))
        return
    if args.only_stress:
        s = bench_stress(args, device)
        print(json.dumps({k: (round(v, 2) if isinstance(v, float) else v) for k, v in s.items()}))
        return
    if args.only_action:
        print(json.dumps({"action_only": bench_action(args, device)}))
        return
    if args.only_frame:
        print(json.dumps({"pi05_frame": _frame_both(device, args.split_tokens),
                          "cross_frame": bench_cross_frame(device, args.split_tokens)}))
        return
    if args.only_arrivals:
        print(json.dumps({"arrival_patterns": bench_arrivals(device, args.split_tokens),
                          "budget_calibration": bench_calibration(device, args.split_tokens)}))
        return
    s = bench_stress(args, device)
    out = {
        "metric": "mixed action+decode attention step us (18 layers: append + attention)",
        "value": round(s["step_us"], 2), "unit": "us/step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(s["step_us"] / 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "stress: 64 decode streams (own ~U{1..2048}) on 8 shared 2048-token "
                               "prefixes + 2 action chunks of 50, 18 layers, 8q/1kv, d=256, page 16, "
                               "fragmented pool", "q_tokens": s["n_q_tokens"],
                   "unique_kv_tokens_per_layer": round(s["unique_kv_tokens"])},
        "kv_hbm_gbps": round(s["kv_gbps"], 1),
        "kv_hbm_frac_of_peak": round(s["kv_gbps"] / HBM_PEAK_GBPS, 4),
        "decode_tokens_per_s": round(s["decode_tokens_per_s"], 1),
        "host_us_per_step": round(s["host_us_per_step"], 1),
        "roofline": {"bound": "hbm", "achieved": round(s["kv_gbps"], 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(s["kv_gbps"] / HBM_PEAK_GBPS, 4),
                     "traffic": None,
                     "kernel": "attn_kernel (all work items of one layer)",
                     "launch_us": round(s["attn_launch_us"], 2),
                     "merge_launch_us": round(s["merge_launch_us"], 2),
                     "alg_bytes_per_launch": round(s["alg_bytes_per_launch"])},
    }
    blk = s["step_us_blocks"]
    out["value_spread"] = {"blocks_of_steps": len(blk), "us_per_step": blk, "min": min(blk),
                           "median": round(float(np.median(blk)), 2), "max": max(blk),
                           "note": "value is the first block; the others repeat it on later steps"}
    with_merge = s["alg_bytes_per_launch"] / ((s["attn_launch_us"] + s["merge_launch_us"]) * 1e-6) / 1e9
    out["roofline"]["frac_attention_plus_merge"] = round(with_merge / HBM_PEAK_GBPS, 4)
    out["launch_schedule"] = "per layer: work items (new rows appended by the work items " \
                             "themselves) + merge"
    out["step_us_with_events"] = round(s["step_us_with_events"], 2)
    if not args.no_alt_schedules:
        out["step_us_three_launches_per_layer"] = round(s["step_us_separate"], 2)
        out["step_us_merge_append_fused_across_layers"] = round(s["step_us_fused"], 2)
        out["step_us_recorded_graph"] = round(s["step_us_graph"], 2)
        out["host_us_per_step_recorded_graph"] = round(s["host_us_per_step_graph"], 1)
    traffic_file = os.path.join(ROOT, "profiles", "pmc_traffic_stress.json")
    if os.path.exists(traffic_file):
        import hashlib
        t = json.load(open(traffic_file))
        src = os.path.join(ROOT, "paper_2603_14371_amd", "csrc", "oxy_kernels.hip")
        now = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
        out["roofline"]["traffic"] = t["hbm_bytes_per_launch"]
        out["roofline"]["traffic_source"] = "profiles/pmc_traffic_stress.json (rocprofv3 --pmc " \
                                            "FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size)"
        # the counters cannot be read from inside this process: the figure is the committed one,
        # stamped with the kernel source it was measured on
        out["roofline"]["traffic_measured_at_commit"] = t.get("measured_at_commit")
        out["roofline"]["traffic_kernel_source_unchanged"] = t.get("kernel_source_sha256_16") == now
    sp = stream_probe(device, s["alg_bytes_per_launch"])
    out["roofline"]["plain_streaming_kernel"] = sp
    out["roofline"]["frac_of_plain_streaming_same_bytes"] = round(
        s["kv_gbps"] / sp["same_bytes"]["gbps"], 4)
    if args.pmc_probe:
        out["pmc_probe_bytes"] = pmc_probe(device)
    if not args.no_cross_task:
        out["cross_task"] = {k: round(v, 2) for k, v in
                             bench_cross_task(device, args.split_tokens).items()}
    if not args.no_frame:
        out["action_only"] = bench_action(args, device)
        out["pi05_frame"] = _frame_both(device, args.split_tokens)
        out["cross_frame"] = {k: (round(v, 2) if isinstance(v, float) else v) for k, v in
                              bench_cross_frame(device, args.split_tokens).items()}
    if not args.no_arrivals:
        out["arrival_patterns"] = bench_arrivals(device, args.split_tokens)
        out["budget_calibration"] = bench_calibration(device, args.split_tokens)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
