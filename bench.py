#!/usr/bin/env python3
"""Benchmark of the DapQ eviction step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch, all layers and heads:
  dapq_rope_apply (pseudo queries to positions L_p..L_p+N-1) -> dapq_score (pass 1 and pass 2 over K: one kernel where
  the library can run both in one launch, else dapq_score_stats and dapq_score_accumulate, timed separately)
  -> dapq_pool_topk (max-pool + TopK) -> dapq_gather.
Inputs are resident in HBM before the timed region.  Prints one JSON line:
  value     prompt keys scored+evicted per second (layers x KV heads x prompt keys / step time)
  roofline  the dominant kernel against the nearer roof (HBM for up to ~310 query rows per KV head,
            dense bf16 MFMA beyond): algorithmic bytes (flops) of one launch / its average duration,
            timed with events on the launch stream inside the timed region
  cpu_baseline  the float64 oracle on the host cores (one worker process per core, one layer per task), on a
            bounded sample of the same workload, run before the GPU is touched

`--ceilings` measures, instead of the step, what this chip can do for the instruction mix of the score passes:
read-only streams, the passes' slice (one MFMA + the vector work on two logits) with no memory traffic, and the
passes themselves with the keys in HBM, in the memory-side cache and in L2 (profiles/score_c2_ceiling.md).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch), each scaled
# by what the same counter reads for kernels of known size in the same run (the 2 GiB read-stream probe; the
# fp32 -> bf16 conversion of the input generator: 128 MiB read, 64 MiB written); profiles/score_c2_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = {    # (workload, N, kernel)
    ("C2", 64, "score"): 4.341e9,         # both passes in one kernel: 4.307 GB fetched (K twice, Q once) + 32 MiB written
    ("C2", 32, "score"): 4.333e9,         # 4.299 GB fetched + 32 MiB written
    ("C2", 64, "score_pass2"): 2.201e9,   # 2.167 GB fetched (keys + the pseudo queries once per head) + 32 MiB written
    ("C2", 64, "score_pass1"): 2.171e9,   # 2.169 GB fetched + 2 MiB of partial row statistics written
    ("C2", 32, "score_pass2"): 2.190e9,   # 2.156 GB fetched + 32 MiB written
    ("C2", 32, "score_pass1"): 2.157e9,   # 2.156 GB fetched + 1 MiB written
}
# Where those figures come from: the profile file and the commit whose score kernels were profiled.  A CPU test
# (tests/test_bench_host.py) fails when csrc/score.hip has changed since that commit, i.e. when they are stale.
TRAFFIC_SOURCE = {"file": "profiles/score_c2_hbm_traffic.md", "commit": "ef1131b"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the clock governor needs about 50 steps after idle to settle (a boost, a deep throttle, then the sustained
    # clock): the defaults time the sustained rate
    ap.add_argument("--settle-ms", type=float, default=150.0,
                    help="untimed steps are run for this long before the warm-up so that the timed steps see the "
                         "sustained clock whatever --warmup is (reported as settle_steps)")
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="C2", help="C1..C5 (C2 is the configuration the metric is quoted on)")
    ap.add_argument("--n-pseudo", type=int, default=None, help="override N (the C4 sweep)")
    ap.add_argument("--layers", type=int, default=None, help="override the layer count (fits memory / quick runs)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-layers", type=int, default=None, help="layers the CPU oracle baseline runs (0 = skip)")
    ap.add_argument("--ceilings", action="store_true",
                    help="measure the chip's ceilings for the score passes instead of the step (see the module text)")
    ap.add_argument("--event-stride", type=int, default=1,
                    help="every how many timed steps the kernels are bracketed by event records (each record is a "
                         "marker in the queue that costs about a microsecond of the step it is in: with 8 the step is "
                         "0.6 %% shorter and the passes, which then get no pause at all, 0.7 %% longer)")
    ap.add_argument("--post-idle-steps", type=int, default=20,
                    help="steps timed right after set-up and a pause, before the clock governor has settled "
                         "(reported as ms_per_step_post_idle; 0 = skip)")
    ap.add_argument("--split-passes", action="store_true",
                    help="time the two score passes as separate launches even where the library can run both in one "
                         "kernel (how the per-pass profiles are taken)")
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points around the step (extended normaliser, decode over the compact "
                         "cache, recall); reported under extras_ms, not part of value")
    return ap.parse_args()


def _cpu_worker(w, seed, L, layers, ready, done):
    """One worker process of the oracle leg: prepares the inputs of its layers (not timed), waits for the start
    signal, then runs the rotation of the pseudo queries and the eviction step on each of them."""
    import numpy as np
    import threadpoolctl
    import workloads as W
    from oracle import dapq_oracle as O
    with threadpoolctl.threadpool_limits(1):     # one core per worker process
        inputs = []
        for layer in layers:
            qp = W.q_pre(w, seed, layer, 0)
            k = np.empty((L, w.n_kv_heads, w.head_dim), dtype=np.uint16)
            v = np.empty_like(k)
            for kv in range(w.n_kv_heads):
                k[:, kv] = W.k_pre(w, seed, layer, 0, kv, L, qp)
                v[:, kv] = W.v_rows(w, seed, layer, 0, kv, L)
            inputs.append((qp, O.rope_apply(k, W.k_positions(L), w.theta)[None], v[None]))
        ready.wait()
        for qp, k, v in inputs:
            q = O.rope_apply(qp.transpose(1, 0, 2), W.q_positions(L, w.n_pseudo), w.theta).transpose(1, 0, 2)
            O.compress(q[None, None], k, v, w.n_kv_heads, w.budget, None, w.pool_width, w.scale)
        done.wait()


def cpu_baseline(w, seed, n_layers):
    """Times the oracle (rope of the pseudo queries + the eviction step) on n_layers layers of the workload
    (sequence 0 only for ragged batches) on the host cores: one single-threaded worker process per core, each with
    its share of the layers.  Must run before anything touches the GPU (the workers are forked).  Input generation
    and the rotation of K are preparation and are not timed, as on the GPU side: the clock runs from the moment
    every worker has its inputs to the moment the last one is finished."""
    import multiprocessing as mp
    import workloads as W

    L = W.seq_lens(w, seed)[0]
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    workers = max(1, min(cores, 16, n_layers))    # a one-GPU machine has a share of 16 cores
    ctx = mp.get_context("fork")
    ready, done = ctx.Barrier(workers + 1), ctx.Barrier(workers + 1)
    procs = [ctx.Process(target=_cpu_worker, args=(w, seed, L, list(range(i, n_layers, workers)), ready, done))
             for i in range(workers)]
    for p in procs:
        p.start()
    try:
        ready.wait(timeout=600)
        t0 = time.perf_counter()
        done.wait(timeout=600)
        dt = time.perf_counter() - t0
    finally:
        for p in procs:
            p.join(timeout=30)
            if p.is_alive():
                p.terminate()
    if any(p.exitcode != 0 for p in procs):
        raise RuntimeError("a worker of the oracle leg failed")
    keys = n_layers * w.n_kv_heads * L
    return {
        "value": keys / dt, "unit": "keys/s", "cores": workers, "kind": "oracle",
        "sample": f"{n_layers} of {w.n_layers} layers x {w.n_kv_heads} KV heads x {L} keys of {w.name} "
                  f"(sequence 0), {dt:.1f} s wall clock; {workers} single-threaded worker processes, "
                  f"{(n_layers + workers - 1) // workers} layer(s) each",
    }


class Context:
    """Everything one benchmark step needs, resident in HBM: inputs, outputs, workspace, and step()."""

    def __init__(self, w, seed, dev, overrides=None, keep_pooled=False, split_passes=False):
        """keep_pooled: also write the pooled scores to self.P (the tests look at them); otherwise pooling
        happens inside the selection kernel whenever dapq_pool_topk can fuse the two.
        split_passes: call dapq_score_stats and dapq_score_accumulate even where dapq_score would run both passes
        in one kernel (the per-pass profiles under profiles/ are taken this way).
        overrides: optional {(layer_index, sequence, kv_head): (k_bits [L, d], v_bits [L, d])} of post-RoPE
        host slices written over the device-generated ones; the parity tests use it to give the oracle and
        the GPU the same bits for the heads they compare."""
        import numpy as np
        import torch
        import paper_2603_11564_amd as D
        import workloads as W

        self.w, self.dev, self.D = w, dev, D
        data = W.device_fill(w, seed, dev)
        self.lens = lens = data["lens"]
        self.cu = data["cu_seqlens"] if w.ragged is not None else None
        self.cu_host = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        self.tokens = tokens = int(sum(lens))
        self.k, self.v = k, v = data["k"], data["v"]
        d, Hq, Hkv, N, nl, B = w.head_dim, w.n_q_heads, w.n_kv_heads, w.n_pseudo, w.n_layers, w.batch
        if w.layout == "hnd":
            kstr = (Hkv * tokens * d, 0, tokens * d, d)
            rope_k = (d, tokens * d)
        else:
            kstr = (tokens * Hkv * d, 0, d, Hkv * d)
            rope_k = (Hkv * d, d)
        for li in range(nl):       # keys are cached already rotated; done once, outside the timed region
            D.dapq_rope_apply(k[li], k[li], data["k_pos"], tokens, Hkv, d, rope_k[0], rope_k[1], w.theta, 0)
        if overrides:
            for (li, b, kv), (kb, vb) in overrides.items():
                kt = torch.from_numpy(kb.view(np.int16)).to(dev).view(torch.bfloat16)
                vt = torch.from_numpy(vb.view(np.int16)).to(dev).view(torch.bfloat16)
                s0, s1 = int(self.cu_host[b]), int(self.cu_host[b + 1])
                assert kt.shape[0] == s1 - s0
                if w.layout == "hnd":
                    k[li, kv, s0:s1].copy_(kt)
                    v[li, kv, s0:s1].copy_(vt)
                else:
                    k[li, s0:s1, kv].copy_(kt)
                    v[li, s0:s1, kv].copy_(vt)
        # pseudo queries laid out [layer][Hq][batch][N][d]: (sequence, pseudo token) is then one row axis and
        # (layer, head) one head axis, so a single rope call covers the whole batch
        self.q_pre = data["q"].permute(0, 2, 1, 3, 4).contiguous()
        self.q = torch.empty_like(self.q_pre)
        qstr = (Hq * B * N * d, N * d, B * N * d, d)
        self.shape = D.make_shape(n_layers=nl, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, n_pseudo=N,
                                  total_tokens=tokens, cu_seqlens=self.cu, k_strides=kstr, v_strides=kstr,
                                  q_strides=qstr, scale=w.scale)
        self.ws = torch.empty(D.workspace_bytes(self.shape), dtype=torch.uint8, device=dev)
        # both passes in one kernel (dense batches of up to 256 rows per KV head and at most 4 chunks per sequence)
        self.single_launch = D.score_single_launch(self.shape) and not split_passes
        self.names = (["rope", "score", "pool_topk", "gather"] if self.single_launch else
                      ["rope", "score_pass1", "score_pass2", "pool_topk", "gather"])
        self.lse2 = torch.empty((nl, B, Hq, N), dtype=torch.float32, device=dev)
        self.S = torch.empty((nl, Hkv, tokens), dtype=torch.float32, device=dev)
        # dapq_pool_topk pools inside the selection kernels for windows up to 9: heads up to 65536 keys in one kernel,
        # longer ones in pieces through a workspace of candidate lists; else it needs P as scratch
        longest = max(lens) if w.ragged is None else tokens
        n_topk_ws = D.topk_workspace_bytes(self.shape, w.budget)
        self.topk_ws = torch.empty(n_topk_ws, dtype=torch.uint8, device=dev) if n_topk_ws else None
        self.fused_select = w.pool_width <= 9 and (longest <= 65536 or self.topk_ws is not None)
        self.P = torch.empty_like(self.S) if (keep_pooled or not self.fused_select) else None
        self.idx = torch.zeros((nl, B, Hkv, w.budget), dtype=torch.int32, device=dev)
        self.count = torch.zeros((nl, B, Hkv), dtype=torch.int32, device=dev)
        self.k_out = torch.zeros((nl, B, Hkv, w.budget, d), dtype=torch.bfloat16, device=dev)
        self.v_out = torch.zeros_like(self.k_out)
        self.q_pos = data["q_pos"].reshape(-1).contiguous()
        self.stream = torch.cuda.current_stream()
        self.key_units = nl * Hkv * tokens

    def step(self, events=None):
        """One step; events (len(self.names) + 1 of them) bracket the calls in the order of self.names."""
        D, w, stream = self.D, self.w, self.stream
        d, Hq, N, nl = w.head_dim, w.n_q_heads, w.n_pseudo, w.n_layers
        at = [0]

        def mark():
            if events is not None:
                events[at[0]].record(stream)
            at[0] += 1
        mark()
        D.dapq_rope_apply(self.q_pre, self.q, self.q_pos, w.batch * N, nl * Hq, d, d, w.batch * N * d, w.theta, 0, stream)
        mark()
        if self.single_launch:
            D.dapq_score(self.shape, self.q, self.k, self.S, self.ws, stream)
        else:
            D.dapq_score_stats(self.shape, self.q, self.k, self.lse2, self.ws, stream)
            mark()
            D.dapq_score_accumulate(self.shape, self.q, self.k, self.lse2, self.S, self.ws, stream)
        mark()
        D.dapq_pool_topk(self.shape, self.S, w.pool_width, w.budget, None, self.idx, self.count, self.P, stream, self.topk_ws)
        mark()
        D.dapq_gather(self.shape, self.k, self.v, self.idx, self.count, w.budget, self.k_out, self.v_out, stream)
        mark()


def read_stream_gbs(dev, n_bytes=2 << 30):
    """What a read-only stream of 2 GiB (the key bytes of C2) reaches on this machine, outside the timed region: with plain
    16-byte loads from many waves, and through the score kernels' own path (one wave per SIMD, LDS-direct loads into a
    ring of 32-key sub-blocks).  The practical ceilings of a pass that only moved the keys, for scale beside the 8 TB/s
    data-sheet peak."""
    import torch
    from paper_2603_11564_amd import ceiling
    a = torch.empty(n_bytes, dtype=torch.uint8, device=dev)
    a.fill_(1)
    torch.cuda.synchronize()
    res = {"plain_loads": ceiling.stream(a, 0, 8192)["gbs"], "lds_ring": ceiling.stream(a, 1, 5, 1)["gbs"]}
    del a
    return res


def shader_clock_mhz():
    """The shader clock the driver reports right now (the starred level of pp_dpm_sclk), or None."""
    import glob
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            for line in open(path):
                if "*" in line:
                    return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except (OSError, ValueError, IndexError):
            continue
    return None


def board_power_watts():
    """(what the board draws right now, its power cap) in watts as the driver reports them (hwmon power1_input or
    power1_average, power1_cap), or (None, None)."""
    import glob
    for hw in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
        try:
            cap = float(open(os.path.join(hw, "power1_cap")).read()) * 1e-6
            for leaf in ("power1_input", "power1_average"):
                path = os.path.join(hw, leaf)
                if os.path.exists(path):
                    return float(open(path).read()) * 1e-6, cap
        except (OSError, ValueError):
            continue
    return None, None


def time_passes(ctx, shape, warm, reps):
    """Average duration (ms) of the two score passes for `shape`, each launched back to back on its own, and of
    dapq_score (both in one kernel where the library can), with the shader clock (<name>_mhz) and the board power
    (<name>_watts; power_cap_watts) the driver reports while the queued launches run (None where it cannot be read)."""
    import torch
    D, stream = ctx.D, ctx.stream
    res = {"power_cap_watts": board_power_watts()[1]}
    calls = {
        "score_pass1": lambda: D.dapq_score_stats(shape, ctx.q, ctx.k, ctx.lse2, ctx.ws, stream),
        "score_pass2": lambda: D.dapq_score_accumulate(shape, ctx.q, ctx.k, ctx.lse2, ctx.S, ctx.ws, stream),
        "score": lambda: D.dapq_score(shape, ctx.q, ctx.k, ctx.S, ctx.ws, stream),
    }
    for name, fn in calls.items():
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        clocks, watts = [], []
        while not e1.query():       # the launches are queued: the GPU is still working through them
            time.sleep(0.03)
            clocks.append(shader_clock_mhz())
            watts.append(board_power_watts()[0])
        torch.cuda.synchronize()
        res[name] = e0.elapsed_time(e1) / reps
        res[name + "_mhz"] = clocks[2:-1]       # (the first samples see the governor still settling)
        res[name + "_watts"] = watts[2:-1]
    return res


def ceilings(ctx, args):
    """The measurements behind profiles/score_c2_ceiling.md, in one run on one box."""
    import torch
    from paper_2603_11564_amd import ceiling
    w, dev = ctx.w, ctx.dev
    g, N, d = w.n_q_heads // w.n_kv_heads, w.n_pseudo, w.head_dim
    ctx.step()                      # rotated pseudo queries
    torch.cuda.synchronize()
    out = {"workload": f"{w.name}: {w.n_layers} layers, N {N}, L_p {ctx.lens[0]}", "reps": args.steps}
    # slices one SIMD runs per pass: (rows / 32) x (keys / 32) x (d / 16) MFMAs over all heads, on 1024 SIMDs
    slices = ctx.key_units * g * N * d / (32 * 32 * 16) / 1024
    out["slices_per_simd_per_pass"] = slices
    out["streams"] = {
        "plain_loads_8192_workgroups": ceiling.stream(ctx.k, 0, 8192, 0, 3, 50),
        "lds_ring_5_slots_1_wave_per_simd": ceiling.stream(ctx.k, 1, 5, 1, 3, 50),
        "lds_ring_2_slots_2_waves_per_simd": ceiling.stream(ctx.k, 1, 2, 2, 3, 50),
    }
    probes = []
    for mix in ceiling.slice_mixes():
        for wps in (1, 2):
            r = ceiling.slice_probe(mix["index"], wps, 400, 3, args.steps)
            r.update({"mix": mix["name"], "waves_per_simd": wps, "ms_per_pass_equivalent": r["ns_per_slice"] * slices * 1e-6})
            probes.append(r)
    out["slice_probes"] = probes
    # the passes themselves, the keys in HBM / in the memory-side cache (every layer reads layer 0's keys: 1/n_layers
    # of the bytes) / in L2 and the memory-side cache (every head reads head 0 of layer 0)
    placements = {"hbm": ctx.shape}
    if w.layout == "hnd":
        one_layer, one_head = type(ctx.shape).from_buffer_copy(ctx.shape), type(ctx.shape).from_buffer_copy(ctx.shape)
        one_layer.k_stride_layer = 0
        one_head.k_stride_layer = 0
        one_head.k_stride_head = 0
        placements["one_layer_of_keys_for_all"] = one_layer
        placements["one_head_of_keys_for_all"] = one_head
    out["passes_ms"] = {name: time_passes(ctx, shape, args.warmup, args.steps) for name, shape in placements.items()}
    out["passes_ns_per_slice"] = {name: {k: r[k] * 1e6 / (slices * n) for k, n in (("score_pass1", 1), ("score_pass2", 1), ("score", 2))}
                                  for name, r in out["passes_ms"].items()}
    # the key slab on chip across the passes: both passes over G layers at a time (G x 64 MiB of keys at C2, against
    # the 256 MB memory-side cache), so that pass 2 finds the keys pass 1 just read; the same kernels, the planner
    # choosing the chunks of each G-layer launch
    if w.layout == "hnd" and w.batch == 1:
        out["both_passes_ms_by_layer_group"] = time_layer_groups(ctx, args.warmup, max(1, args.steps // 6))
    return out


def time_layer_groups(ctx, warm, reps):
    """ms for pass 1 + pass 2 over all layers when they are run G layers at a time (pass 1 then pass 2 of a group,
    then the next group), for several G; G = all layers is the two plain launches."""
    import torch
    D, w, stream = ctx.D, ctx.w, ctx.stream
    res = {}
    for G in (1, 2, 3, 4, 8, 16, w.n_layers):
        if G > w.n_layers:
            continue
        sub = type(ctx.shape).from_buffer_copy(ctx.shape)
        sub.n_layers = G
        last = type(ctx.shape).from_buffer_copy(ctx.shape)
        last.n_layers = w.n_layers % G
        need = max(D.workspace_bytes(sub), D.workspace_bytes(last) if last.n_layers else 0)
        ws = ctx.ws if need <= ctx.ws.numel() else torch.empty(need, dtype=torch.uint8, device=ctx.dev)

        def sweep():
            for l0 in range(0, w.n_layers, G):
                shp = sub if l0 + G <= w.n_layers else last
                l1 = l0 + shp.n_layers
                D.dapq_score_stats(shp, ctx.q[l0:l1], ctx.k[l0:l1], ctx.lse2[l0:l1], ws, stream)
                D.dapq_score_accumulate(shp, ctx.q[l0:l1], ctx.k[l0:l1], ctx.lse2[l0:l1], ctx.S[l0:l1], ws, stream)
        for _ in range(max(1, warm // 4)):
            sweep()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            sweep()
        e1.record(stream)
        torch.cuda.synchronize()
        res[f"{G}_layers_at_a_time"] = e0.elapsed_time(e1) / reps
    return res


class pseudo_query_problem:
    """The queries of the pseudo tokens for the benchmark's workload (Sec. 4.1 upstream of the step): model width
    H_q * d, one N(0, 1/hidden) query weight per layer, 2048 stand-in rows of N(0,1) projection input per layer, and
    pseudo tokens that copy the first 4 and the last N - 4 of them in every sequence."""

    def __init__(self, ctx, rows_per_layer=2048):
        import torch
        D, w, dev = ctx.D, ctx.w, ctx.dev
        d, Hq, N, nl, B = w.head_dim, w.n_q_heads, w.n_pseudo, w.n_layers, w.batch
        self.ctx, self.hidden, self.T = ctx, Hq * d, rows_per_layer
        hidden, T = self.hidden, self.T
        g = torch.Generator(device=dev).manual_seed(2)
        self.x = torch.randn((nl, T, hidden), generator=g, device=dev).to(torch.bfloat16)
        self.w_q = torch.empty((nl, Hq * d, hidden), dtype=torch.bfloat16, device=dev)
        for li in range(nl):
            self.w_q[li].copy_(torch.randn((Hq * d, hidden), generator=g, device=dev) * hidden ** -0.5)
        first = min(4, N)
        self.src = torch.cat([torch.arange(first), torch.arange(T - (N - first), T)]).to(torch.int32).repeat(B).to(dev)
        self.desc = D.Qproj(n_layers=nl, rows=B * N, hidden=hidden, n_q_heads=Hq, head_dim=d, total_tokens=T,
                            x_stride_layer=T * hidden, x_stride_token=hidden, w_stride_layer=Hq * d * hidden,
                            w_stride_row=hidden, q_stride_layer=Hq * B * N * d, q_stride_head=B * N * d, q_stride_row=d)
        self.q = torch.empty((nl, Hq, B, N, d), dtype=torch.bfloat16, device=dev)
        self.pos = ctx.q_pos.reshape(-1).contiguous()
        self.ws = torch.empty(max(D.pseudo_queries_workspace_bytes(self.desc), 16), dtype=torch.uint8, device=dev)

    def run(self, rotate=True):
        ctx = self.ctx
        ctx.D.dapq_pseudo_queries(self.desc, self.x, self.src, self.w_q, self.pos if rotate else None, ctx.w.theta, 0,
                                  self.q, self.ws, ctx.stream)


def time_extras(ctx, reps):
    """Event-timed averages of the entry points that sit around the eviction step, on the step's own outputs."""
    import torch
    D, w, dev, stream = ctx.D, ctx.w, ctx.dev, ctx.stream
    d, Hq, Hkv, N, nl, B = w.head_dim, w.n_q_heads, w.n_kv_heads, w.n_pseudo, w.n_layers, w.batch
    g = torch.Generator(device=dev).manual_seed(1)
    kp = torch.randn((nl, B, Hkv, N, d), generator=g, device=dev).to(torch.bfloat16)
    qd = torch.randn((nl, B, Hq, d), generator=g, device=dev).to(torch.bfloat16)
    dec = torch.empty((nl, B, Hq, d), dtype=torch.float32, device=dev)
    common = torch.empty((nl, B, Hkv), dtype=torch.int32, device=dev)
    rec = torch.empty((nl, B, Hkv), dtype=torch.float32, device=dev)
    D.dapq_score_stats(ctx.shape, ctx.q, ctx.k, ctx.lse2, ctx.ws, stream)   # (a one-kernel step leaves no lse2)
    lse = ctx.lse2.clone()
    calls = {
        "score_stats_extend": lambda: D.dapq_score_stats_extend(ctx.shape, ctx.q, kp, (B * Hkv * N * d, Hkv * N * d, N * d, d),
                                                                lse, stream),
        "recall": lambda: D.dapq_recall(ctx.shape, ctx.idx, ctx.count, w.budget, ctx.idx, ctx.count, w.budget, common, rec,
                                        stream),
    }
    if w.budget <= 8192:
        calls["decode_attention"] = lambda: D.dapq_decode_attention(ctx.shape, qd, ctx.k_out, ctx.v_out, ctx.count, w.budget,
                                                                    dec, stream)
    pq = pseudo_query_problem(ctx)
    calls["pseudo_queries"] = lambda: pq.run(rotate=True)
    calls["pseudo_queries_no_rotation"] = lambda: pq.run(rotate=False)
    res = {}
    for name, fn in calls.items():
        fn()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        evs[0].record(stream)
        for i in range(reps):
            fn()
            evs[i + 1].record(stream)
        torch.cuda.synchronize()
        res[name] = sum(evs[i].elapsed_time(evs[i + 1]) for i in range(reps)) / reps
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 "
              "(the path would shard by layer, KV head or sequence with no communication between the GPUs)",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import workloads as W
    from dataclasses import replace

    w = W.workload(args.workload, args.n_pseudo)
    if args.layers is not None:
        w = replace(w, n_layers=args.layers)
    lens0 = W.seq_lens(w, args.seed)
    # the oracle leg comes first: its worker processes are forked, which has to happen before the GPU is touched
    ncpu = args.cpu_layers
    if ncpu is None:
        ncpu = max(1, min(w.n_layers, int(round(32 * (32768 * 8 * 256) /
                                                 (lens0[0] * w.n_kv_heads * (w.n_q_heads // w.n_kv_heads) * w.n_pseudo)))))
    cpu = cpu_baseline(w, args.seed, min(ncpu, w.n_layers)) if (ncpu > 0 and not args.ceilings) else None

    import torch
    import paper_2603_11564_amd as D
    D.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ctx = Context(w, args.seed, dev, split_passes=args.split_passes)
    lens, tokens = ctx.lens, ctx.tokens
    d, Hq, Hkv, N, nl, B = w.head_dim, w.n_q_heads, w.n_kv_heads, w.n_pseudo, w.n_layers, w.batch
    names = ctx.names
    if args.ceilings:
        print(json.dumps({"ceilings": ceilings(ctx, args)}), flush=True)
        return

    # the first steps after idle, before the clock governor has settled: reported beside the sustained figure
    ms_post_idle = None
    if args.post_idle_steps > 0:
        for _ in range(3):
            ctx.step()
        torch.cuda.synchronize()
        time.sleep(1.0)
        t_idle = time.perf_counter()
        for _ in range(args.post_idle_steps):
            ctx.step()
        torch.cuda.synchronize()
        ms_post_idle = (time.perf_counter() - t_idle) * 1e3 / args.post_idle_steps

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] if s % max(1, args.event_stride) == 0 else None
           for s in range(args.steps)]
    # untimed: let the clock governor settle under this load (after idle it boosts, then throttles deeply, and reaches
    # the sustained clock after some 60 ms), then the W warm-up steps proper
    settle_steps = 0
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(10):
            ctx.step()
        torch.cuda.synchronize()
        settle_steps += 10
    for _ in range(args.warmup):
        ctx.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stride = max(1, args.event_stride)
    for s in range(args.steps):
        ctx.step(evs[s] if s % stride == 0 else None)
    # the host is far ahead of the stream: while it waits for the queued steps, a second thread reads what the driver
    # says about power and clock (the wait itself is the plain synchronize, so the clock stops when the GPU does)
    import threading
    watts, mhz, waiting = [], [], threading.Event()

    def sample():
        while not waiting.is_set():
            watts.append(board_power_watts()[0])
            mhz.append(shader_clock_mhz())
            time.sleep(0.02)
    sampler = threading.Thread(target=sample, daemon=True)
    sampler.start()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    waiting.set()
    sampler.join()
    ms_per_step = dt * 1e3 / args.steps
    per = {n: float(np.mean([evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(0, args.steps, stride)]))
           for i, n in enumerate(names)}

    key_units = ctx.key_units
    value = key_units / (ms_per_step * 1e-3)

    # ---------------------------------------------------------------- roofline of the dominant kernel
    # algorithmic bytes of one score pass: every key row once (2*d bytes) + the 4-byte score (pass 2)
    # or nothing (pass 1), + the pseudo queries once per KV head
    q_bytes = nl * B * Hq * N * d * 2
    flops_one_pass = 2.0 * key_units * (Hq // Hkv) * N * d
    if ctx.single_launch:
        # one kernel walks K twice (pass 1 forward, pass 2 backward), reads the pseudo queries once, writes the scores
        bytes_pass = {"score": key_units * (4 * d + 4) + q_bytes}
        flops_of = {"score": 2 * flops_one_pass}
    else:
        bytes_pass = {"score_pass1": key_units * 2 * d + q_bytes, "score_pass2": key_units * (2 * d + 4) + q_bytes}
        flops_of = {"score_pass1": flops_one_pass, "score_pass2": flops_one_pass}
    dom = max(bytes_pass, key=lambda n: per[n])
    flops_pass = flops_of[dom]
    hbm_gbs = bytes_pass[dom] / (per[dom] * 1e-3) / 1e9
    mfma_tflops = flops_pass / (per[dom] * 1e-3) / 1e12
    # which roof is nearer: a pass runs g*N*d*2 flop per 2*d bytes of K, the machine balances at peak/peak
    if flops_pass / bytes_pass[dom] > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        roofline = {"bound": "mfma", "kernel": dom, "achieved": mfma_tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": mfma_tflops / MFMA_BF16_PEAK_TFLOPS}
    else:
        roofline = {"bound": "hbm", "kernel": dom, "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": hbm_gbs / HBM_PEAK_GBS}
    nrb = 2 if (Hq // Hkv) * N <= 64 else (4 if (Hq // Hkv) * N <= 128 else 8)      # 32-row blocks a wave holds
    roofline.update({
        # the device function behind the kernel_ms entry named by "kernel", as a kernel trace shows it
        "kernel_name": {"score": f"score_fused_kernel<{nrb}, 5>", "score_pass1": f"score_wave_pass1_kernel<{nrb}, ...>",
                        "score_pass2": f"score_wave_pass2_kernel<{nrb}, ...>"}[dom],
        "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, N, dom)),
        "traffic_source": (f"{TRAFFIC_SOURCE['file']}, rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the kernels at commit "
                           f"{TRAFFIC_SOURCE['commit']} (not measured in this run)"
                           if (w.name, N, dom) in MEASURED_TRAFFIC_BYTES else None),
        "algorithmic_bytes_per_launch": bytes_pass[dom], "algorithmic_flops_per_launch": flops_pass,
        "avg_launch_ms": per[dom], "hbm_gbs": hbm_gbs, "mfma_tflops": mfma_tflops,
    })

    # whole step against HBM: bytes the method must move (K once, scores, selection, retained rows) and bytes
    # of the two-pass design (K twice), per step time
    retained = sum(min(w.budget, L) for L in lens) * nl * Hkv
    step_alg = key_units * (2 * d + 16) + retained * (4 + 8 * d)
    step_design = step_alg + key_units * 2 * d
    step_hbm = {
        "algorithmic_bytes": step_alg, "design_bytes": step_design,
        "algorithmic_gbs": step_alg / (ms_per_step * 1e-3) / 1e9, "design_gbs": step_design / (ms_per_step * 1e-3) / 1e9,
        "design_frac_of_peak": step_design / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "mfma_frac_of_peak": {n: flops_of[n] / (per[n] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS for n in bytes_pass},
    }

    # what a read-only stream reaches on this machine, for scale next to the data-sheet peak (outside the timed region)
    streams = read_stream_gbs(dev)
    step_hbm["read_stream_gbs"] = streams
    step_hbm["design_frac_of_read_stream"] = step_hbm["design_gbs"] / streams["lds_ring"]
    roofline["hbm_frac_of_read_stream"] = hbm_gbs / streams["lds_ring"]

    out = {
        "metric": "prompt keys scored+evicted/sec (all layers x KV heads)", "value": value, "unit": "keys/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_steps": settle_steps, "event_stride": stride, "ms_per_step": ms_per_step,
        "ms_per_step_post_idle": ms_post_idle,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {nl} layers, {Hq} q / {Hkv} kv heads, d {d}, batch {B}, "
                               f"L_p {lens if w.ragged else lens[0]}, N {N}, budget {w.budget}, pool {w.pool_width}, "
                               f"K layout {w.layout}"},
        "kernel_ms": per,
        # sampled every 20 ms while the timed steps ran (None where the driver's files cannot be read)
        "board_power_watts": {"mean": float(np.mean([x for x in watts if x])) if any(watts) else None,
                              "max": max([x for x in watts if x], default=None), "cap": board_power_watts()[1],
                              "samples": len(watts)},
        "shader_clock_mhz": float(np.mean([x for x in mhz if x])) if any(mhz) else None,
        "roofline": roofline,
        "step_hbm": step_hbm,
    }
    if args.extras:
        out["extras_ms"] = time_extras(ctx, args.steps)
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
