#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step is one pass of the whole path over one batch group of synthetic input already resident
in HBM: gate + top-k + dispatch plan (moe_route), then gather, grouped SwiGLU expert FFN and
weighted combine (moe_layer_forward).  Headline workload: the Mixtral-8x7B-shaped decode layer
(d_model 4096, d_ff 14336, 8 experts, top-2, 8 batches x 64 sequences x 1 token, bf16, experts
resident), bound by HBM.  Prints ONE JSON line with tokens/s, the roofline of the dominant kernel
(timed live with HIP events on the compute stream, between the launches inside the library) and
the CPU oracle timed on a bounded sample of the same workload.  Without --workload the line
also carries, under "legs", the other two rooflines the metric names: the prefill layer (matrix
cores) and the streamed stacks (host link: achieved GB/s, idle fraction of the link and of the
compute stream from the library's events around every copy and every kernel group).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # published dense bf16 matrix-core peak


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, data, budget_s: float = 15.0):
    """The oracle as it stands, on the host cores, on a bounded token sample."""
    from oracle import ref
    from paper_2502_06888_amd import inputs as I
    x, wg = I.as_f32(data.x), I.as_f32(data.wg)
    w1 = [I.as_raw(t) for t in data.w1]
    w3 = [I.as_raw(t) for t in data.w3]
    w2 = [I.as_raw(t) for t in data.w2]
    cores = ref.num_threads()

    def run(n):
        tok = np.arange(n, dtype=np.int32)
        t0 = time.perf_counter()
        ref.moe_layer(x[:n], wg, w1, w3, w2, w.top_k, [0, n], w.dtype, tokens=tok)
        return time.perf_counter() - t0

    probe_n = min(w.n_tokens, max(cores, 8))
    t_probe = run(probe_n)
    n = int(min(w.n_tokens, max(probe_n, probe_n * budget_s / max(t_probe, 1e-3))))
    n = max(cores, n // cores * cores)
    n = min(n, w.n_tokens)
    t = run(n) if n != probe_n else t_probe
    return {"value": n / t, "unit": "tokens/s", "cores": cores, "cpu_model": cpu_model(), "kind": "oracle",
            "sample": f"first {n} of {w.n_tokens} tokens of the same workload "
                      f"(gate, top-k, dispatch and fp64 SwiGLU experts), {t:.1f} s"}


def recorded_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` from the committed counter summary (FETCH_SIZE +
    WRITE_SIZE, each scaled by the copy-kernel calibration) and the git head the summary was
    recorded at; (None, None) when no summary covers it.  Counters cannot be read from inside a
    timed run, so this figure is the recorded one."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        f"{kernel}_{workload}_hbm_traffic.md")
    traffic, head = None, None
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = int(float(line.split(":", 1)[1]))
                if line.startswith("git_head:"):
                    head = line.split(":", 1)[1].strip()
    except OSError:
        pass
    return traffic, head


def planner_report(ctx, w, xs, ys, K, compute, torch, B):
    """Measurement stage + constraint solving of the planner on layer 0, then a sweep over the
    number of batches per group n: measured time of the layer against the model
    max(transfer time of the activated experts, compute time of the group)."""
    tpb = w.batch_tokens[0]
    rows = []
    for n in [b for b in (1, 2, 4, 8, 16, 32) if b <= w.n_batches]:
        N = n * tpb
        bo = [i * tpb for i in range(n + 1)]
        x, y = xs[0][:N], ys[0][:N]
        with torch.cuda.stream(compute):
            m = ctx.measure(0, x, bo, y, reps=3)
            t_comp = (m["t_c_gate_group_s"] + m["t_c_gather_s"] + sum(m["t_c_expert_s"]) + m["t_c_combine_s"])
            t_io = m["n_active"] * m["t_io_expert_s"]
            # the layer as the pipeline runs it: on-demand transfers, compute as they land
            reps, t0 = 3, None
            for r in range(reps + 1):
                if r == 1:
                    compute.synchronize(); t0 = time.perf_counter()
                ctx.route(0, x, bo)
                counts, order, na = ctx.route_wait()
                ctx.stream_experts(0, order[:na], B.MOE_ON_DEMAND)
                ctx.layer_forward(0, x, y)
            compute.synchronize()
            t_layer = (time.perf_counter() - t0) / reps
        pred = max(t_io, t_comp)
        rows.append({"n_batches": n, "tokens": N, "n_active": m["n_active"],
                     "t_io_expert_ms": m["t_io_expert_s"] * 1e3, "t_gate_group_us": m["t_c_gate_group_s"] * 1e6,
                     "t_experts_us": sum(m["t_c_expert_s"]) * 1e6,
                     "t_compute_us": t_comp * 1e6, "t_transfers_ms": t_io * 1e3,
                     "layer_ms_measured": t_layer * 1e3, "layer_ms_predicted": pred * 1e3,
                     "compute_bubble_measured": 1.0 - t_comp / t_layer,
                     "compute_bubble_predicted": 1.0 - t_comp / pred})
        last = m
    # smallest n that satisfies the inequality group, from the figures of the largest group:
    # per-batch gate time, hot experts = the first K in execution order, the rest queued
    n = rows[-1]["n_batches"]
    order = last["exec_order"]
    hot, cold = order[:K], order[K:]
    t_c_hot = sum(last["t_c_expert_s"][e] for e in hot)
    t_c_q = [last["t_c_expert_s"][e] for e in cold]
    n_min_moe = B.moe_plan_batches(0.0, last["t_c_gate_group_s"] / n, t_c_hot, t_c_q, 0.0, 0.0, last["t_io_expert_s"], K)
    # t_c_A: the attention layer of one batch (the batch's tokens as sequences, 512 cached
    # positions, caches in HBM, weights resident: t_IO_A = 0), measured with the library's events
    t_c_A = measure_attention_batch(w, tpb, torch)
    n_min = B.moe_plan_batches(t_c_A, last["t_c_gate_group_s"] / n, t_c_hot, t_c_q, 0.0, 0.0, last["t_io_expert_s"], K)
    return {"layer": 0, "tokens_per_batch": tpb, "K": K, "n_min": n_min, "n_min_without_attention": n_min_moe,
            "t_c_A_us": t_c_A * 1e6, "sweep": rows,
            "note": "t_IO_A = t_IO_G = 0: attention weights and gate resident; t_c_A from the attention "
                    "layer with d_model/128 query heads, 8 key-value heads of 128, 512 cached positions"}


def measure_attention_batch(w, n_seq, torch, pos: int = 512) -> float:
    """Kernel time of the attention layer for one batch of the workload's model width."""
    from paper_2502_06888_amd import attn_binding as A
    from paper_2502_06888_amd import inputs as I
    hq = w.d_model // 128
    aw = I.AttnWorkload("plan_attn", w.d_model, hq, 8 if hq % 8 == 0 and hq <= 64 else hq, 128, (n_seq,) * 2, (pos,) * 2,
                        pos + 64, kv_on_host=False, seed=w.seed)
    ctx = A.AttnContext(A.config_for(aw), "cuda:0")
    ws = I.gen_attn_weights(aw, 0)
    ctx.set_weights(*[ws[k].to("cuda:0") for k in ("norm", "wq", "wk", "wv", "wo")])
    batches = []
    for b in range(aw.n_batches):
        k, v = [t.to("cuda:0") for t in I.gen_kv_cache(aw, 0, b)]
        h = I.gen_attn_hidden(aw, 0, b).to("cuda:0")
        batches.append(A.AttnBatch(k, v, h, torch.empty_like(h), pos))
    ctx.forward_group(batches)
    ctx.synchronize()
    ctx.set_profiling(1)
    best = None
    for _ in range(5):
        ctx.forward_group(batches)
        t = ctx.profile().compute_busy_s / aw.n_batches
        best = t if best is None else min(best, t)
    ctx.close()
    return best


_STREAMS = {}


def shared_streams(torch):
    """One compute and one copy stream for the whole run, created once and in this order.  The
    runtime maps streams onto a few hardware queues as they are created and destroyed; with fresh
    streams for every leg the copy stream of a later leg now and then lands on the compute
    stream's queue, and its copies then wait behind the expert kernels (measured: 281 instead of
    235 ms per pass on the fine-grained stack, depending only on how many streams earlier legs had
    created)."""
    if not _STREAMS:
        _STREAMS["compute"] = torch.cuda.Stream()
        _STREAMS["copy"] = torch.cuda.Stream()
    return _STREAMS["compute"], _STREAMS["copy"]


def release_memory(torch):
    """Hand cached device and pinned host blocks back (the streamed stacks pin tens of GiB each)."""
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()


def measure_link_peak(torch, nbytes: int = 1 << 30, reps: int = 5) -> float:
    """Best host->device rate of one large copy from pinned memory on this machine, GB/s."""
    src = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    st = shared_streams(torch)[1]
    best = 0.0
    with torch.cuda.stream(st):
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            dst.copy_(src, non_blocking=True)
            e1.record(st)
            e1.synchronize()
            best = max(best, nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return best


def bench_streamed(w, args):
    """Streamed stack: all routed experts in pinned host memory, a window of device slots, the
    next layer's hot experts prefetched while the current layer computes.  A step is one pass
    over all layers for one batch group (one decode step of the stack)."""
    import torch
    from paper_2502_06888_amd import binding as B
    from paper_2502_06888_amd import inputs as I
    dev = torch.device("cuda:0")
    compute, copy = shared_streams(torch)
    q4 = args.weight_bits == 4
    cfg = B.make_config(w.d_model, w.d_ff, w.n_experts, w.top_k, w.n_shared, w.n_layers,
                        w.window_layers, w.n_tokens, w.n_batches, B.MOE_BF16, 1, 4 if q4 else 0)
    ctx = B.MoeContext(cfg, compute, copy)
    link_peak = measure_link_peak(torch)
    t_setup = time.perf_counter()
    xs, noise = [], None
    for l in range(w.n_layers):                      # placement: generate, pack, park in pinned memory
        data, noise = I.gen_layer(w, l, noise, threads=16, with_experts=not q4)
        ctx.set_gate(l, data.wg.to(dev))
        for e in range(w.n_experts + w.n_shared):
            where = B.MOE_HOST_PINNED if e < w.n_experts else B.MOE_RESIDENT
            if q4:
                trip = I.gen_expert_q4(w, l, e)
                ctx.set_expert_q4(l, e, tuple(tuple(t.to(dev) for t in m) for m in trip), where)
            else:
                ctx.set_expert(l, e, data.w1[e].to(dev), data.w3[e].to(dev), data.w2[e].to(dev), where)
        xs.append(data.x.to(dev))
        del data
    t_setup = time.perf_counter() - t_setup
    ys = [torch.empty((w.n_tokens, w.d_model), dtype=w.torch_dtype, device=dev) for _ in xs]
    bo = [int(v) for v in w.batch_offsets]
    K = args.prefetch if args.prefetch >= 0 else w.top_k
    use_corr = args.prefetch_policy == "corr"
    if use_corr:
        # table warm-up (the paper's pre-run): route other batch groups of the same model through
        # the stack; no experts are moved or computed.  The table is then frozen, so that the
        # accuracy below is measured on a batch group it has never seen.
        ctx.corr_enable(1)
        with torch.cuda.stream(compute):
            for grp in range(8):
                ww, nz = I.scaled(w, token_seed=1000 + grp), None
                for l in range(w.n_layers):
                    dl, nz = I.gen_layer(ww, l, nz, with_experts=False)
                    ctx.route(l, dl.x.to(dev), bo)
                ctx.route_wait()
        ctx.corr_enable(2)
    acc = {"predicted": 0, "in_true_topk": 0, "activated": 0}
    guess = {}

    def one_pass():
        n_active = []
        for l in range(w.n_layers):
            ctx.route(l, xs[l], bo)
            counts, order, na = ctx.route_wait()
            if l in guess and guess[l]:                                  # score the guess made for l
                true_top = set(np.argsort(-np.asarray(counts), kind="stable")[:len(guess[l])].tolist())
                acc["predicted"] += len(guess[l])
                acc["in_true_topk"] += sum(1 for e in guess[l] if e in true_top)
                acc["activated"] += sum(1 for e in guess[l] if counts[e] > 0)
            ctx.stream_experts(l, order[:na], B.MOE_ON_DEMAND)          # what the gate selected
            nxt = (l + 1) % w.n_layers
            if use_corr and nxt >= 1:
                hot = ctx.corr_predict(nxt, K) if K > 0 else []
            else:                                                        # previous layer's busiest
                hot = list(np.argsort(-np.asarray(counts), kind="stable")[:K])
            guess[nxt] = [int(e) for e in hot]
            if hot:
                ctx.stream_experts(nxt, hot, B.MOE_PREFETCH)            # guess for the next layer
            ctx.layer_forward(l, xs[l], ys[l])
            n_active.append(na)
        return n_active

    plan_report = None
    if args.plan:
        plan_report = planner_report(ctx, w, xs, ys, K, compute, torch, B)
    with torch.cuda.stream(compute):
        for _ in range(max(1, args.warmup if args.warmup < 5 else 1)):
            one_pass()
    torch.cuda.synchronize()
    ctx.reset_stats()
    acc.update(predicted=0, in_true_topk=0, activated=0)
    steps = args.steps if args.steps <= 20 else 5
    with torch.cuda.stream(compute):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            n_active = one_pass()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    st = ctx.stats()
    gbs = st["bytes_h2d"] / wall / 1e9
    # the same pass once more with the library's events around every copy and every kernel group:
    # busy time of the link (union over the copy streams) and of the compute stream over the wall
    # time from the first copy's start to the last kernel's end
    ctx.reset_stats()
    ctx.set_profiling(True)
    with torch.cuda.stream(compute):
        one_pass()
    torch.cuda.synchronize()
    pst = ctx.stats()
    ctx.set_profiling(False)
    wall_ns = max(1, pst["wall_ns"])
    # smallest number of batches per group for which compute would cover the transfers (the
    # planner's inequality group, without an attention layer in between): measured on layer 0
    with torch.cuda.stream(compute):
        m = ctx.measure(0, xs[0], bo, ys[0], reps=2)
    order = m["exec_order"]
    n_min = B.moe_plan_batches(0.0, m["t_c_gate_group_s"] / w.n_batches, sum(m["t_c_expert_s"][e] for e in order[:K]),
                               [m["t_c_expert_s"][e] for e in order[K:]], 0.0, 0.0, m["t_io_expert_s"], K)
    out = {
        "metric": "moe_stack_tokens_per_s", "value": w.n_tokens * steps / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": 1, "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "d_model": w.d_model, "d_ff": w.d_ff, "n_experts": w.n_experts,
                   "top_k": w.top_k, "n_shared": w.n_shared, "n_layers": w.n_layers,
                   "tokens": w.n_tokens, "n_batches": w.n_batches, "window_layers": w.window_layers,
                   "weight_bits": args.weight_bits,
                   "prefetch_per_layer": K, "prefetch_policy": args.prefetch_policy,
                   "experts": "pinned host memory",
                   "n_active_per_layer": n_active},
        "token_layers_per_s": w.n_tokens * w.n_layers * steps / wall,
        "host_link": {"achieved_GBps": gbs, "measured_peak_GBps": link_peak, "nominal_peak_GBps": 64.0,
                      "frac_of_nominal": gbs / 64.0, "frac_of_measured": gbs / link_peak,
                      "rate_shortfall_vs_probe": 1.0 - gbs / link_peak,
                      "bytes_h2d_per_step": st["bytes_h2d"] / steps, "copies_per_step": st["n_copies"] / steps,
                      "prefetch_hits_per_step": st["n_prefetch_hits"] / steps,
                      "prefetch_unused_per_step": st["n_prefetch_unused"] / steps},
        "prefetch": {"predicted": acc["predicted"],
                     "hot_accuracy": acc["in_true_topk"] / max(1, acc["predicted"]),
                     "activated_fraction": acc["activated"] / max(1, acc["predicted"])},
        "pipeline": {"profiled_pass_wall_ms": wall_ns * 1e-6, "copy_busy_ms": pst["copy_busy_ns"] * 1e-6,
                     "compute_busy_ms": pst["compute_busy_ns"] * 1e-6,
                     "bubble_link_idle": 1.0 - pst["copy_busy_ns"] / wall_ns,
                     "bubble_compute_idle": 1.0 - pst["compute_busy_ns"] / wall_ns,
                     "copy_rate_GBps": pst["bytes_h2d"] / max(1, pst["copy_busy_ns"]),
                     "n_min_batches_for_full_overlap": n_min,
                     "note": "bubble_link_idle = 1 - copy busy / wall (the binding resource); bubble_compute_idle "
                             "= 1 - compute busy / wall is the paper's bubble: compute waiting for transfers"},
        "setup_s": t_setup,
    }
    if plan_report is not None:
        out["planner"] = plan_report
    ctx.close()
    del ctx, xs, ys
    release_memory(torch)
    return out


def attn_cpu_baseline(w, ws, hs, caches, budget_s: float = 12.0):
    """The attention oracle on the host cores: whole batches of the workload, in order, until the
    time budget is used or the workload is done."""
    from oracle import attn_ref, ref
    from paper_2502_06888_amd import inputs as I
    raw = {k: I.as_raw(v) for k, v in ws.items()}
    cores = ref.num_threads()
    done, t = 0, 0.0
    for b in range(w.n_batches):
        x, kc, vc = I.as_f32(hs[b]), I.as_raw(caches[b][0]), I.as_raw(caches[b][1])
        t0 = time.perf_counter()
        attn_ref.attn_decode(x, raw["norm"], raw["wq"], raw["wk"], raw["wv"], raw["wo"], kc, vc,
                             w.batch_pos[b], w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, w.rms_eps)
        t += time.perf_counter() - t0
        done += w.batch_seqs[b]
        if t > budget_s:
            break
    return {"value": done / t, "unit": "tokens/s", "cores": cores, "cpu_model": cpu_model(), "kind": "oracle",
            "sample": f"first {done} of {w.n_tokens} sequences (whole batches) of the same workload, fp64 "
                      f"attention layer over {w.batch_pos[0]} cached positions, {t:.1f} s"}


def bench_attention(w, args):
    """Attention (non-expert) layer of one decoding step over the batch group: batch by batch,
    each batch's key-value cache and hidden state either resident in HBM or streamed from pinned
    host memory by the load / store streams.  A step is one moe_attn_forward_group call."""
    import torch
    from paper_2502_06888_amd import attn_binding as A
    from paper_2502_06888_amd import inputs as I
    dev = torch.device("cuda:0")
    ctx = A.AttnContext(A.config_for(w), dev)
    ws = I.gen_attn_weights(w, 0)
    ctx.set_weights(*[ws[n].to(dev) for n in ("norm", "wq", "wk", "wv", "wo")])
    hs = [I.gen_attn_hidden(w, 0, b) for b in range(w.n_batches)]
    caches = [I.gen_kv_cache(w, 0, b) for b in range(w.n_batches)]
    link_peak = measure_link_peak(torch) if w.kv_on_host else None
    batches = []
    for b in range(w.n_batches):
        if w.kv_on_host:
            k, v = caches[b][0].pin_memory(), caches[b][1].pin_memory()
            h_in = hs[b].pin_memory()
            h_out = torch.zeros_like(h_in).pin_memory()
        else:
            k, v, h_in = caches[b][0].to(dev), caches[b][1].to(dev), hs[b].to(dev)
            h_out = torch.zeros_like(h_in)
        batches.append(A.AttnBatch(k, v, h_in, h_out, w.batch_pos[b]))
    steps = min(args.steps, 20 if w.kv_on_host else 200)
    warmup = min(args.warmup, 2 if w.kv_on_host else 20)
    if args.calibrate_copy:       # a kernel of known traffic for counter runs
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        del src, dst
        torch.cuda.synchronize()
    for _ in range(max(1, warmup)):
        ctx.forward_group(batches)
    ctx.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ctx.forward_group(batches)
    ctx.synchronize()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    ctx.set_profiling(1)                         # separate passes: event timing of the streams
    prof = []
    for _ in range(3):
        ctx.forward_group(batches)
        prof.append(ctx.profile())
    pr = min(prof, key=lambda p: p.wall_s)
    ctx.set_profiling(8)                         # kernels: 8 launches between each event pair
    prof = []
    for _ in range(3):
        ctx.forward_group(batches)
        prof.append(ctx.profile())
    ctx.set_profiling(0)
    pk = min(prof, key=lambda p: p.kernel_s[3])
    names = ["rmsnorm", "qkv_proj", "qkv_finish", "attn_decode", "out_proj", "out_finish"]
    kern_us = {n: pk.kernel_s[i] * 1e6 for i, n in enumerate(names)}
    dq, dkv = w.n_q_heads * w.head_dim, w.n_kv_heads * w.head_dim
    kv_bytes = sum(2 * w.batch_seqs[b] * dkv * (w.batch_pos[b] + 1) * 2 for b in range(w.n_batches))
    attn_bytes = kv_bytes + sum(w.batch_seqs[b] * dq * (4 + 2) for b in range(w.n_batches))
    weight_bytes = ((dq + 2 * dkv) * w.d_model + w.d_model * dq) * 2
    out = {
        "metric": "attn_layer_tokens_per_s", "value": w.n_tokens / wall, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": max(1, warmup), "ms_per_step": wall * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "d_model": w.d_model, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "n_batches": w.n_batches,
                   "seqs_per_batch": list(w.batch_seqs), "cached_positions": list(w.batch_pos),
                   "cache": "pinned host memory" if w.kv_on_host else "HBM"},
        "kernels_us_per_step": kern_us,
        "pipeline": {"wall_ms": pr.wall_s * 1e3, "load_busy_ms": pr.load_busy_s * 1e3,
                     "store_busy_ms": pr.store_busy_s * 1e3, "compute_busy_ms": pr.compute_busy_s * 1e3,
                     "bytes_loaded": pr.bytes_loaded, "bytes_stored": pr.bytes_stored},
    }
    # a device-resident group is run in one pass (one launch per kernel for all batches, the
    # projection weights read once); a streamed group batch by batch
    launches = w.n_batches if w.kv_on_host else 1
    t_attn = pk.kernel_s[3] / launches
    layer_bytes = kv_bytes + weight_bytes * launches
    out["roofline"] = {"bound": "hbm", "kernel": "attn_decode_kernel", "launches_per_step": launches,
                       "achieved": attn_bytes / launches / t_attn / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": attn_bytes / launches / t_attn / 1e9 / HBM_PEAK_GBS,
                       "traffic": recorded_traffic(w.name, "attn_decode_kernel")[0],
                       "traffic_recorded_at": recorded_traffic(w.name, "attn_decode_kernel")[1],
                       "algorithmic_bytes_per_launch": attn_bytes // launches,
                       "layer_bytes_per_step": layer_bytes,
                       "layer_GBps": layer_bytes / pr.compute_busy_s / 1e9}
    if w.kv_on_host:
        gbs = pr.bytes_loaded / pr.wall_s / 1e9
        out["host_link"] = {"achieved_GBps": gbs, "measured_peak_GBps": link_peak, "nominal_peak_GBps": 64.0,
                            "frac_of_nominal": gbs / 64.0, "frac_of_measured": gbs / link_peak,
                            "bubble_link_idle": max(0.0, 1.0 - pr.load_busy_s / pr.wall_s),
                            "copy_rate_GBps": pr.bytes_loaded / pr.load_busy_s / 1e9,
                            "compute_busy_fraction": pr.compute_busy_s / pr.wall_s}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = attn_cpu_baseline(w, ws, hs, caches)
    ctx.close()
    return out


def bench_resident(w, args, data=None, steps=None, warmup=None, with_cpu_baseline=True):
    """One all-resident layer (decode or prefill shape): K timed steps after W warm-up steps, then
    per-kernel durations from the library's events and the roofline of the dominant kernel."""
    import torch
    from paper_2502_06888_amd import binding as B
    from paper_2502_06888_amd import inputs as I
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    dev = torch.device("cuda:0")
    q4 = args.weight_bits == 4
    if data is None:
        data, _ = I.gen_layer(w, 0, threads=16, with_experts=not q4)
    compute = shared_streams(torch)[0]
    cfg = B.make_config(w.d_model, w.d_ff, w.n_experts, w.top_k, w.n_shared, 1, 0, w.n_tokens,
                        w.n_batches, B.MOE_F32 if w.dtype == "f32" else B.MOE_BF16, 1, 4 if q4 else 0)
    ctx = B.MoeContext(cfg, compute)
    if args.h_planes or args.split_k or args.variant:
        ctx.set_tuning(args.split_k, args.h_planes, args.variant)
    ctx.set_gate(0, data.wg.to(dev))
    for e in range(w.n_experts + w.n_shared):
        if q4:
            trip = I.gen_expert_q4(w, 0, e)
            ctx.set_expert_q4(0, e, tuple(tuple(t.to(dev) for t in m) for m in trip))
        else:
            if args.zero_weights:   # power probe: the same launches, addresses and traffic, all products zero
                z1, z2 = torch.zeros_like(data.w1[e], device=dev), torch.zeros_like(data.w2[e], device=dev)
                ctx.set_expert(0, e, z1, z1, z2)
            else:
                ctx.set_expert(0, e, data.w1[e].to(dev), data.w3[e].to(dev), data.w2[e].to(dev))
    x = data.x.to(dev)
    y = torch.empty((w.n_tokens, w.d_model), dtype=w.torch_dtype, device=dev)
    bo = [int(v) for v in w.batch_offsets]
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)       # 1 GiB read
        dst = torch.empty_like(src)                                     # 1 GiB written
        for _ in range(3):
            torch.add(src, 1, out=dst)
        del src, dst
    torch.cuda.synchronize()

    def step():
        ctx.route(0, x, bo)
        ctx.layer_forward(0, x, y)

    # Settling (untimed, before the warm-up steps): a GPU that sat idle during set-up starts at
    # its boost clock, overshoots its power limit and throttles for some tens of milliseconds;
    # the steady state a serving loop sees comes after that.
    settle_steps = 0
    with torch.cuda.stream(compute):
        step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while (time.perf_counter() - t0) * 1e3 < args.settle_ms:
            for _ in range(8):
                step()
            torch.cuda.synchronize()
            settle_steps += 8
        for _ in range(warmup):
            step()
    torch.cuda.synchronize()

    # timed region: exactly K steps, inputs resident, bracketed by device synchronisation
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(compute):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(compute)
        for _ in range(steps):
            step()
        ev1.record(compute)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    dev_ms = ev0.elapsed_time(ev1)
    ms_per_step = max(wall_ms, dev_ms) / steps

    # per-kernel durations, HIP events recorded by the library between its launches
    ctx.reset_stats()
    ctx.set_profiling(True)
    prof = {}
    reps = max(10, min(50, steps))
    with torch.cuda.stream(compute):
        for _ in range(reps):
            step()
            for k_, v in ctx.profile().items():
                prof[k_] = prof.get(k_, 0.0) + v / reps
    ctx.set_profiling(False)
    counts, order, n_active = ctx.route_wait()
    st = ctx.stats()

    elt = w.elt_bytes
    A = w.n_tokens * w.top_k
    # algorithmic bytes of the dominant kernel (up projections + SwiGLU): W1 and W3 of every
    # activated expert once, the gathered token rows once, H written once
    wbytes = 9.0 / 16.0 if q4 else elt      # 4-bit codes + one (scale, zero point) pair per 64 weights
    up_bytes = int(n_active * 2 * w.d_model * w.d_ff * wbytes) + A * w.d_model * elt + A * w.d_ff * elt
    layer_bytes = (int(n_active * 3 * w.d_model * w.d_ff * wbytes) + w.n_tokens * w.d_model * elt * 2 +
                   2 * A * w.d_ff * elt + A * w.d_model * 4)
    achieved = up_bytes / (prof["up_ms"] * 1e-3) / 1e9 if prof.get("up_ms", 0) > 0 else 0.0
    # gate and up projections: 2 flops x rows x d x 2f.  Above the machine balance (2.5 PFLOP/s over
    # 8 TB/s = 312 flop/byte) the kernel is priced against the dense bf16 MFMA peak instead
    up_flops = 2.0 * A * w.d_model * 2 * w.d_ff
    layer_flops = 2.0 * A * w.d_model * 3 * w.d_ff
    traffic, traffic_head = (None, None) if q4 else recorded_traffic(w.name, "ffn_up_kernel")
    if w.dtype == "bf16" and up_flops / up_bytes > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        tf = up_flops / (prof["up_ms"] * 1e-3) / 1e12 if prof.get("up_ms", 0) > 0 else 0.0
        down_tf = (2.0 * A * w.d_model * w.d_ff) / (prof["down_ms"] * 1e-3) / 1e12 if prof.get("down_ms", 0) > 0 else 0.0
        roofline = {"bound": "mfma", "kernel": "ffn_up_kernel", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic,
                    "traffic_recorded_at": traffic_head,
                    "algorithmic_flops": up_flops, "algorithmic_bytes": up_bytes,
                    "down_kernel_TFLOPs": down_tf, "down_kernel_frac": down_tf / MFMA_BF16_PEAK_TFLOPS,
                    "layer_TFLOPs": layer_flops / (ms_per_step * 1e-3) / 1e12,
                    "layer_frac": layer_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    else:
        roofline = {"bound": "hbm", "kernel": "ffn_up_kernel", "achieved": achieved,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "traffic": traffic, "traffic_recorded_at": traffic_head, "algorithmic_bytes": up_bytes}

    out = {
        "metric": "moe_layer_tokens_per_s", "value": w.n_tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "d_model": w.d_model, "d_ff": w.d_ff,
                   "n_experts": w.n_experts, "top_k": w.top_k, "n_batches": w.n_batches,
                   "tokens": w.n_tokens,
                   "experts": "resident in HBM" + (", all-zero weights (power probe)" if args.zero_weights else ""),
                   "weight_bits": args.weight_bits,
                   "n_active": n_active,
                   "h_format": "f32" if w.dtype == "f32" else
                               "fp16 + fp16 remainder plane (" + ("always multiplied" if args.h_planes == 2
                                                                  else "multiplied where needed") + ")",
                   "remainder_plane_workgroups_per_step": st["h_remainder_wgs"] / reps,
                   "h_values_clamped": st["h_saturated"],
                   "settle_steps_untimed": settle_steps,
                   "tokens_per_expert": counts},
        "roofline": roofline,
        "kernels_us": {k_.replace("_ms", ""): round(v * 1e3, 2) for k_, v in prof.items()},
        "layer": {"algorithmic_bytes": layer_bytes,
                  "hbm_frac_of_peak": layer_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                  "device_ms_per_step": dev_ms / steps},
    }
    ctx.close()
    if with_cpu_baseline and not args.no_cpu_baseline and not q4:
        out["cpu_baseline"] = cpu_baseline(w, data)
    return out, data


LEG_KEYS = ("value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config", "roofline", "kernels_us",
            "layer", "token_layers_per_s", "host_link", "pipeline", "setup_s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=None,
                    help="one workload only (default: the decode layer as the headline plus the prefill "
                         "layer and the streamed stacks as legs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-legs", action="store_true", help="headline workload only")
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="untimed steps run before the warm-up until the clocks have settled")
    ap.add_argument("--h-planes", type=int, default=0,
                    help="0 = library default (remainder plane of H multiplied where needed), 2 = always")
    ap.add_argument("--split-k", type=int, default=0, help="0 = library default")
    ap.add_argument("--variant", type=int, default=0,
                    help="launch shape of the bf16 expert kernels (moe_set_tuning); 0 = library default")
    ap.add_argument("--prefetch", type=int, default=-1,
                    help="streamed stacks: experts prefetched per layer (-1 = top_k)")
    ap.add_argument("--prefetch-policy", choices=["prev", "corr"], default="prev",
                    help="streamed stacks: prefetch the previous layer's busiest experts (prev) or "
                         "the correlation table's prediction (corr, warmed up on other batch groups)")
    ap.add_argument("--weight-bits", type=int, choices=[16, 4], default=16,
                    help="expert weights as bf16 (16) or as 4-bit codes in groups of 64 (4)")
    ap.add_argument("--plan", action="store_true",
                    help="streamed stacks: run the planner's measurement stage on layer 0, solve the "
                         "overlap inequalities for n, and sweep the number of batches per group")
    ap.add_argument("--zero-weights", action="store_true",
                    help="resident workloads: place all-zero expert weights (routing, launches and memory "
                         "traffic unchanged, every product zero): what remains of the step time shows how much "
                         "of it the data-dependent power of the matrix cores costs through the clock")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB -> 1 GiB elementwise copy kernel before the "
                         "timed region, so that a counter run has a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2502_06888_amd import binding as B
    from paper_2502_06888_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load_library()  # fails loudly when the HIP library is not built

    if args.workload in I.ATTN_WORKLOADS:
        print(json.dumps(bench_attention(I.ATTN_WORKLOADS[args.workload], args)))
        return
    if args.workload is not None:
        w = I.WORKLOADS[args.workload]
        out = bench_streamed(w, args) if w.streamed else bench_resident(w, args)[0]
        print(json.dumps(out))
        return

    # headline: the decode layer (HBM roofline); then the other legs of the metric
    wd = I.WORKLOADS["mixtral8x7b_decode"]
    out, data = bench_resident(wd, args)
    if not args.no_legs:
        # a leg that cannot run on this machine (say, not enough pinnable host memory for the 36 GiB
        # stack) is reported as such; the headline above stands on its own
        legs = {}

        def run_leg(key, fn):
            try:
                leg = fn()
                legs[key] = {k: leg[k] for k in LEG_KEYS if k in leg}
            except Exception as exc:                # noqa: BLE001 - reported, not hidden
                legs[key] = {"error": f"{type(exc).__name__}: {exc}"[:300]}
            release_memory(torch)

        wp = I.WORKLOADS["mixtral8x7b_prefill"]     # matrix-core roofline: same layer, 16384 tokens
        dp = I.LayerData(x=I.gen_x_gaussian(wp), wg=data.wg, w1=data.w1, w3=data.w3, w2=data.w2)
        run_leg(wp.name, lambda: bench_resident(wp, args, data=dp, steps=min(args.steps, 20),
                                                warmup=min(args.warmup, 5), with_cpu_baseline=False)[0])
        del data, dp
        release_memory(torch)
        for name, bits in (("finegrained_stream", 16), ("finegrained_stream", 4), ("mixtral8x22b_stream", 16)):
            args.weight_bits = bits                 # host-link roofline and the pipeline's bubbles
            run_leg(name + ("_4bit" if bits == 4 else ""), lambda: bench_streamed(I.WORKLOADS[name], args))
        out["legs"] = legs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
