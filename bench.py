#!/usr/bin/env python3
"""Benchmark of the DapQ eviction step on one MI355X.

A step is one pass of the whole hot path over one synthetic batch, all layers and heads:
  dapq_rope_apply (pseudo queries to positions L_p..L_p+N-1) -> dapq_score_stats (pass 1 over K)
  -> dapq_score_accumulate (pass 2 over K) -> dapq_pool_topk (max-pool + TopK) -> dapq_gather.
Inputs are resident in HBM before the timed region.  Prints one JSON line:
  value     prompt keys scored+evicted per second (layers x KV heads x prompt keys / step time)
  roofline  the dominant kernel against the nearer roof (HBM for up to ~310 query rows per KV head,
            dense bf16 MFMA beyond): algorithmic bytes (flops) of one launch / its average duration,
            timed with events on the launch stream inside the timed region
  cpu_baseline  the float64 oracle on the host cores, on a bounded sample of the same workload
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
# by what the same counter reads for a copy kernel of known size in the same run (the fp32 -> bf16 conversion
# of the input generator: 128 MiB read, 64 MiB written); profiles/score_c2_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = {    # (workload, N, kernel)
    ("C2", 64, "score_pass2"): 2.250e9,   # 2.217 GB fetched (1.032 x the key bytes: Q is re-read per chunk) + 32 MiB written
    ("C2", 64, "score_pass1"): 2.217e9,   # 2.214 GB fetched + 2 MiB of partial row statistics written
}


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
    ap.add_argument("--extras", action="store_true",
                    help="also time the entry points around the step (extended normaliser, decode over the compact "
                         "cache, recall); reported under extras_ms, not part of value")
    return ap.parse_args()


def cpu_baseline(w, seed, n_layers):
    """Times the oracle (rope of the pseudo queries + the eviction step) on n_layers layers of the
    workload, sequence 0 only for ragged batches.  Input generation and the rotation of K are
    preparation and are not timed, as on the GPU side."""
    import numpy as np
    import threadpoolctl
    import workloads as W
    from oracle import dapq_oracle as O

    lens = W.seq_lens(w, seed)
    L = lens[0]
    qs, ks, vs = [], [], []
    for layer in range(n_layers):
        qp = W.q_pre(w, seed, layer, 0)
        k = np.empty((L, w.n_kv_heads, w.head_dim), dtype=np.uint16)
        v = np.empty_like(k)
        for kv in range(w.n_kv_heads):
            k[:, kv] = W.k_pre(w, seed, layer, 0, kv, L, qp)
            v[:, kv] = W.v_rows(w, seed, layer, 0, kv, L)
        qs.append(qp)
        ks.append(O.rope_apply(k, W.k_positions(L), w.theta))
        vs.append(v)
    k = np.stack(ks)
    v = np.stack(vs)
    t0 = time.perf_counter()
    q = np.stack([O.rope_apply(qp.transpose(1, 0, 2), W.q_positions(L, w.n_pseudo), w.theta).transpose(1, 0, 2)
                  for qp in qs])[:, None]
    O.compress(q, k, v, w.n_kv_heads, w.budget, None, w.pool_width, w.scale)
    dt = time.perf_counter() - t0
    keys = n_layers * w.n_kv_heads * L
    blas = [p["num_threads"] for p in threadpoolctl.threadpool_info() if p.get("user_api") == "blas"]
    return {
        "value": keys / dt, "unit": "keys/s", "cores": max(blas) if blas else 1, "kind": "oracle",
        "sample": f"{n_layers} of {w.n_layers} layers x {w.n_kv_heads} KV heads x {L} keys of {w.name} "
                  f"(sequence 0), {dt:.1f} s; matmul on the BLAS threads, the rest single-threaded",
    }


class Context:
    """Everything one benchmark step needs, resident in HBM: inputs, outputs, workspace, and step()."""

    def __init__(self, w, seed, dev, overrides=None, keep_pooled=False):
        """keep_pooled: also write the pooled scores to self.P (the tests look at them); otherwise pooling
        happens inside the selection kernel whenever dapq_pool_topk can fuse the two.
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
        self.lse2 = torch.empty((nl, B, Hq, N), dtype=torch.float32, device=dev)
        self.S = torch.empty((nl, Hkv, tokens), dtype=torch.float32, device=dev)
        # dapq_pool_topk is one kernel for windows up to 9 and heads up to 65536 keys; else it needs P as scratch
        longest = max(lens) if w.ragged is None else tokens
        self.fused_select = w.pool_width <= 9 and longest <= 65536
        self.P = torch.empty_like(self.S) if (keep_pooled or not self.fused_select) else None
        self.idx = torch.zeros((nl, B, Hkv, w.budget), dtype=torch.int32, device=dev)
        self.count = torch.zeros((nl, B, Hkv), dtype=torch.int32, device=dev)
        self.k_out = torch.zeros((nl, B, Hkv, w.budget, d), dtype=torch.bfloat16, device=dev)
        self.v_out = torch.zeros_like(self.k_out)
        self.q_pos = data["q_pos"].reshape(-1).contiguous()
        self.stream = torch.cuda.current_stream()
        self.key_units = nl * Hkv * tokens

    names = ["rope", "score_pass1", "score_pass2", "pool_topk", "gather"]

    def step(self, events=None):
        D, w, stream = self.D, self.w, self.stream
        d, Hq, N, nl = w.head_dim, w.n_q_heads, w.n_pseudo, w.n_layers

        def mark(i):
            if events is not None:
                events[i].record(stream)
        mark(0)
        D.dapq_rope_apply(self.q_pre, self.q, self.q_pos, w.batch * N, nl * Hq, d, d, w.batch * N * d, w.theta, 0, stream)
        mark(1)
        D.dapq_score_stats(self.shape, self.q, self.k, self.lse2, self.ws, stream)
        mark(2)
        D.dapq_score_accumulate(self.shape, self.q, self.k, self.lse2, self.S, self.ws, stream)
        mark(3)
        D.dapq_pool_topk(self.shape, self.S, w.pool_width, w.budget, None, self.idx, self.count, self.P, stream)
        mark(4)
        D.dapq_gather(self.shape, self.k, self.v, self.idx, self.count, w.budget, self.k_out, self.v_out, stream)
        mark(5)


def stream_copy_gbs(dev, n_bytes=1 << 30, reps=10):
    """Bytes per second (read + write) of torch's device-to-device copy of a 1 GiB tensor: the practical ceiling of a
    pure stream on this machine, reported beside the 8 TB/s data-sheet peak."""
    import torch
    a = torch.empty(n_bytes, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    a.zero_()
    b.copy_(a)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n_bytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


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
    import torch
    import paper_2603_11564_amd as D
    import workloads as W
    from dataclasses import replace

    D.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = W.workload(args.workload, args.n_pseudo)
    if args.layers is not None:
        w = replace(w, n_layers=args.layers)
    ctx = Context(w, args.seed, dev)
    lens, tokens = ctx.lens, ctx.tokens
    d, Hq, Hkv, N, nl, B = w.head_dim, w.n_q_heads, w.n_kv_heads, w.n_pseudo, w.n_layers, w.batch
    names = Context.names

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for _ in range(args.steps)]
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
    for s in range(args.steps):
        ctx.step(evs[s])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    per = {n: float(np.mean([evs[s][i].elapsed_time(evs[s][i + 1]) for s in range(args.steps)]))
           for i, n in enumerate(names)}

    key_units = ctx.key_units
    value = key_units / (ms_per_step * 1e-3)

    # ---------------------------------------------------------------- roofline of the dominant kernel
    # algorithmic bytes of one score pass: every key row once (2*d bytes) + the 4-byte score (pass 2)
    # or nothing (pass 1), + the pseudo queries once per KV head
    q_bytes = nl * B * Hq * N * d * 2
    bytes_pass = {"score_pass1": key_units * 2 * d + q_bytes, "score_pass2": key_units * (2 * d + 4) + q_bytes}
    dom = max(bytes_pass, key=lambda n: per[n])
    flops_pass = 2.0 * key_units * (Hq // Hkv) * N * d
    hbm_gbs = bytes_pass[dom] / (per[dom] * 1e-3) / 1e9
    mfma_tflops = flops_pass / (per[dom] * 1e-3) / 1e12
    # which roof is nearer: a pass runs g*N*d*2 flop per 2*d bytes of K, the machine balances at peak/peak
    if flops_pass / bytes_pass[dom] > MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
        roofline = {"bound": "mfma", "kernel": dom, "achieved": mfma_tflops, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": mfma_tflops / MFMA_BF16_PEAK_TFLOPS}
    else:
        roofline = {"bound": "hbm", "kernel": dom, "achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": hbm_gbs / HBM_PEAK_GBS}
    roofline.update({
        "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, N, dom)),
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
        "mfma_frac_of_peak": {n: flops_pass / (per[n] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS for n in bytes_pass},
    }

    # what a plain device copy moves on this machine, for scale next to the data-sheet peak (outside the timed region)
    copy_gbs = stream_copy_gbs(dev)
    step_hbm["stream_copy_gbs"] = copy_gbs
    step_hbm["design_frac_of_stream_copy"] = step_hbm["design_gbs"] / copy_gbs
    roofline["hbm_frac_of_stream_copy"] = hbm_gbs / copy_gbs

    out = {
        "metric": "prompt keys scored+evicted/sec (all layers x KV heads)", "value": value, "unit": "keys/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_steps": settle_steps, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {nl} layers, {Hq} q / {Hkv} kv heads, d {d}, batch {B}, "
                               f"L_p {lens if w.ragged else lens[0]}, N {N}, budget {w.budget}, pool {w.pool_width}, "
                               f"K layout {w.layout}"},
        "kernel_ms": per,
        "roofline": roofline,
        "step_hbm": step_hbm,
    }
    if args.extras:
        out["extras_ms"] = time_extras(ctx, args.steps)
    ncpu = args.cpu_layers
    if ncpu is None:
        ncpu = max(1, min(nl, int(round(24 * (32768 * 8 * 256) / (lens[0] * Hkv * (Hq // Hkv) * N)))))
    if ncpu > 0:
        out["cpu_baseline"] = cpu_baseline(w, args.seed, min(ncpu, nl))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
