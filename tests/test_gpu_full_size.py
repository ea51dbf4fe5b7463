"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The whole workload is built in HBM exactly as bench.py builds it (bench.Context).  A few (layer, KV
head) slices are overwritten with host-generated bits (workloads.k_pre + the oracle's RoPE), so the
float64 oracle can compute those heads one by one on the same inputs; every other head is checked
through properties that hold at any size (mass conservation, ordering, bit-exact gathers, planted
needles retained)."""
import os
import sys

import numpy as np
import pytest
import torch

import workloads as W
from oracle import dapq_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.gpu


def announce(msg):
    print(f"[gpu-case] {msg}", file=sys.__stderr__, flush=True)


@pytest.fixture(scope="module")
def env():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    sys.path.insert(0, ROOT)
    import bench
    import dapq_harness
    return bench, dapq_harness


def host_slice(w, seed, layer, seq, kv, L):
    """Post-RoPE bits of one (layer, sequence, KV head) the way the oracle sees them."""
    qp = W.q_pre(w, seed, layer, seq)
    k = O.rope_apply(W.k_pre(w, seed, layer, seq, kv, L, qp)[:, None, :], W.k_positions(L), w.theta)[:, 0]
    v = W.v_rows(w, seed, layer, seq, kv, L)
    q = O.rope_apply(qp.transpose(1, 0, 2), W.q_positions(L, w.n_pseudo), w.theta).transpose(1, 0, 2)
    return q, k, v


def check_all_heads(ctx, w):
    """Size-independent properties over every head, evaluated on the device."""
    g, N, nl, Hkv = w.group, w.n_pseudo, w.n_layers, w.n_kv_heads
    cu = ctx.cu_host
    S, idx, count = ctx.S, ctx.idx, ctx.count
    assert (ctx.P is None) == ctx.fused_select  # pooled scores exist in HBM only on the two-kernel path
    assert torch.isfinite(S).all() and (S > 0).all()
    for b, L in enumerate(ctx.lens):
        s, e = int(cu[b]), int(cu[b + 1])
        # the pooled scores the selection must have seen, from torch's own max-pool (pads with -inf)
        P_b = torch.nn.functional.max_pool1d(S[:, :, s:e], w.pool_width, 1, w.pool_width // 2)
        mass = S[:, :, s:e].double().sum(dim=2)
        assert (mass - g * N).abs().max().item() < 1e-3 * g * N, "softmax mass is not conserved"
        n = min(w.budget, L)
        assert (count[:, b] == n).all()
        ids = idx[:, b, :, :n].long()
        assert (ids[..., 1:] > ids[..., :-1]).all() and ids.min() >= 0 and ids.max() < L
        # every kept key scores at least as high as every dropped key of its head
        Pb = P_b
        kept = torch.zeros_like(Pb, dtype=torch.bool)
        kept.scatter_(2, ids, True)
        lowest_kept = torch.where(kept, Pb, torch.full_like(Pb, float("inf"))).amin(dim=2)
        highest_dropped = torch.where(kept, torch.full_like(Pb, -1.0), Pb).amax(dim=2)
        assert (lowest_kept >= highest_dropped).all()
        # gathers are bit copies of the rows the indices name
        for name, src, dst in (("k", ctx.k, ctx.k_out), ("v", ctx.v, ctx.v_out)):
            rows = src[:, :, s:e] if w.layout == "hnd" else src[:, s:e].permute(0, 2, 1, 3)
            want = torch.gather(rows.view(torch.int16), 2, ids[..., None].expand(-1, -1, -1, w.head_dim))
            assert torch.equal(dst[:, b, :, :n].view(torch.int16), want), name


@pytest.mark.parametrize("name,layers,samples", [
    ("C2", None, [(0, 0), (3, 2), (9, 6), (17, 5), (22, 1), (27, 4), (31, 3), (31, 7)]),
    # the 70B-class shape at its full 128k prompt, 2 of its 80 layers: 512 query rows per KV head (two row groups)
    # and heads of 131072 keys, which the selection takes in four pieces of 32768 keys (pooling across the piece
    # boundaries) and a merge of their candidates
    ("C5", 2, [(0, 3), (1, 7)]),
    # the same shape as the configuration names it: all 80 layers resident (21.5 GB of keys, as much of values), so
    # that the key, value, score and index offsets of the last layers lie far beyond 4 GiB; heads of the first,
    # middle and last layers against the oracle, every head through the properties
    ("C5", None, [(0, 2), (13, 0), (40, 3), (57, 6), (78, 1), (79, 7)]),
    # the window-size sweep at its 64k prompt, one layer each: 64, 512, 1024 and 2048 query rows per KV head
    ("C4:16", 1, [(0, 1), (0, 5)]),
    ("C4:128", 1, [(0, 3)]),
    ("C4:256", 1, [(0, 4)]),
    ("C4:512", 1, [(0, 6), (0, 2)]),
])
def test_full_size_dense_workload(env, name, layers, samples):
    bench, H = env
    from dataclasses import replace
    w = W.workload(*((name.split(":")[0], int(name.split(":")[1])) if ":" in name else (name,)))
    if layers is not None:
        w = replace(w, n_layers=layers)
    seed = 0
    L = w.seq_len
    announce(f"full size {name}: building the workload")
    host = {(li, kv): host_slice(w, seed, li, 0, kv, L) for (li, kv) in samples}
    ctx = bench.Context(w, seed, torch.device("cuda:0"),
                        {(li, 0, kv): (k, v) for (li, kv), (q, k, v) in host.items()})
    announce(f"full size {name}: one step")
    ctx.step()
    torch.cuda.synchronize()
    check_all_heads(ctx, w)
    if ctx.single_launch:
        # the step ran both passes in one kernel: every score of every head has the bits of the separate passes
        announce(f"full size {name}: the separate passes, bit for bit")
        S_split = torch.empty_like(ctx.S)
        H.D.dapq_score_stats(ctx.shape, ctx.q, ctx.k, ctx.lse2, ctx.ws)
        H.D.dapq_score_accumulate(ctx.shape, ctx.q, ctx.k, ctx.lse2, S_split, ctx.ws)
        torch.cuda.synchronize()
        assert torch.equal(ctx.S, S_split)
        del S_split
    # planted needles survive in every head (the device generator plants the same rows as the host one)
    idx = ctx.idx.cpu().numpy()
    for li in range(w.n_layers):
        for kv in range(w.n_kv_heads):
            pos, _, _ = W.needle_plan(w, seed, li, 0, kv, L)
            assert set(pos.tolist()) <= set(idx[li, 0, kv].tolist()), (li, kv)
    classes = {"exact": 0, "margin": 0}
    for (li, kv), (q, k, v) in host.items():
        announce(f"full size {name}: oracle for layer {li} head {kv}")
        g = w.group
        q_gpu = H.host_bits(ctx.q[li, kv * g:(kv + 1) * g, 0])
        assert np.array_equal(q_gpu, q[kv * g:(kv + 1) * g]), "rotated pseudo queries differ from the oracle's"
        S_ref = O.score_head(O.bf16_bits_to_f64(q[kv * g:(kv + 1) * g]), O.bf16_bits_to_f64(k), w.scale)
        P_ref = O.pool(S_ref, w.pool_width)
        worst = H.assert_scores_close(ctx.S[li, kv].cpu().numpy(), S_ref, f"S[{li},{kv}]")
        classes[H.check_retained(P_ref, idx[li, 0, kv], w.budget)] += 1
        keep = idx[li, 0, kv]
        assert np.array_equal(H.host_bits(ctx.k_out[li, 0, kv]), k[keep])
        assert np.array_equal(H.host_bits(ctx.v_out[li, 0, kv]), v[keep])
        announce(f"full size {name}: layer {li} head {kv}: max rel err {worst:.2e}")
    announce(f"full size {name}: sampled heads {classes}")


def test_full_size_extended_normaliser(env):
    """The normaliser that includes the pseudo tokens' own keys (Sec. 4.1: the extended sequence is prefilled as
    one) at the benchmark's shape, through the benchmark's buffers: pass 1, dapq_score_stats_extend, pass 2.
    Sampled heads against the oracle element by element; every head through what holds at any size: the extra
    keys can only take attention mass away from the prompt keys, and never all of it."""
    bench, H = env
    w = W.workload("C2")
    seed, L = 0, w.seq_len
    samples = [(0, 1), (19, 6), (31, 0)]
    announce("full size C2, extended normaliser: building the workload")
    host = {(li, kv): host_slice(w, seed, li, 0, kv, L) for (li, kv) in samples}
    ctx = bench.Context(w, seed, torch.device("cuda:0"), {(li, 0, kv): (k, v) for (li, kv), (q, k, v) in host.items()})
    D, d, Hq, Hkv, N, nl, g = ctx.D, w.head_dim, w.n_q_heads, w.n_kv_heads, w.n_pseudo, w.n_layers, w.group
    ctx.step()                                           # rotated pseudo queries, and S over the prompt keys alone
    torch.cuda.synchronize()
    S_plain = ctx.S.clone()
    gen = torch.Generator(device="cuda").manual_seed(11)
    kp = torch.randn((nl, 1, Hkv, N, d), generator=gen, device="cuda").to(torch.bfloat16)   # the pseudo tokens' keys
    D.dapq_score_stats(ctx.shape, ctx.q, ctx.k, ctx.lse2, ctx.ws)
    lse_plain = ctx.lse2.clone()
    D.dapq_score_stats_extend(ctx.shape, ctx.q, kp, (Hkv * N * d, Hkv * N * d, N * d, d), ctx.lse2)
    D.dapq_score_accumulate(ctx.shape, ctx.q, ctx.k, ctx.lse2, ctx.S, ctx.ws)
    torch.cuda.synchronize()
    assert torch.isfinite(ctx.S).all() and (ctx.S > 0).all()
    # every row sees at least its own key on top of the prompt (a row whose normaliser a needle dominates may not
    # move by a whole fp32 step)
    assert (ctx.lse2 >= lse_plain).all() and (ctx.lse2 > lse_plain).float().mean().item() > 0.9
    assert (ctx.S <= S_plain * (1 + 1e-6)).all()         # ... so every prompt key gets less
    mass = ctx.S.double().sum(dim=2)
    assert (mass < g * N).all() and (mass > 0).all()
    for (li, kv), (q, k, v) in host.items():
        announce(f"full size C2, extended normaliser: oracle for layer {li} head {kv}")
        assert np.array_equal(H.host_bits(ctx.q[li, kv * g:(kv + 1) * g, 0]), q[kv * g:(kv + 1) * g])
        S_ref = O.score_head(O.bf16_bits_to_f64(q[kv * g:(kv + 1) * g]), O.bf16_bits_to_f64(k), w.scale,
                             O.bf16_bits_to_f64(H.host_bits(kp[li, 0, kv])))
        worst = H.assert_scores_close(ctx.S[li, kv].cpu().numpy(), S_ref, f"extended S[{li},{kv}]")
        announce(f"full size C2, extended normaliser: layer {li} head {kv}: max rel err {worst:.2e}")


def test_full_size_ragged_batch(env):
    """The ragged heavy-hitter batch at its full shape but 4 of the 32 layers (the oracle side of a
    sampled head is then ~1 s); N = 128 and g = 4 give 512 rows per KV head, the multi-slab path."""
    bench, H = env
    from dataclasses import replace
    w = replace(W.workload("C3"), n_layers=4)
    seed = 3
    lens = W.seq_lens(w, seed)
    announce(f"full size C3 (4 layers): lens {lens}")
    samples = [(0, 0, 0), (3, 7, 5), (2, 3, 2)]
    host = {(li, b, kv): host_slice(w, seed, li, b, kv, lens[b]) for (li, b, kv) in samples}
    ctx = bench.Context(w, seed, torch.device("cuda:0"), {key: (k, v) for key, (q, k, v) in host.items()})
    ctx.step()
    torch.cuda.synchronize()
    check_all_heads(ctx, w)
    cu = ctx.cu_host
    idx = ctx.idx.cpu().numpy()
    for (li, b, kv), (q, k, v) in host.items():
        s, e = int(cu[b]), int(cu[b + 1])
        g = w.group
        assert np.array_equal(H.host_bits(ctx.q[li, kv * g:(kv + 1) * g, b]), q[kv * g:(kv + 1) * g])
        S_ref = O.score_head(O.bf16_bits_to_f64(q[kv * g:(kv + 1) * g]), O.bf16_bits_to_f64(k), w.scale)
        P_ref = O.pool(S_ref, w.pool_width)
        worst = H.assert_scores_close(ctx.S[li, kv, s:e].cpu().numpy(), S_ref, f"S[{li},{b},{kv}]")
        cls = H.check_retained(P_ref, idx[li, b, kv], w.budget)
        keep = idx[li, b, kv]
        assert np.array_equal(H.host_bits(ctx.k_out[li, b, kv]), k[keep])
        assert np.array_equal(H.host_bits(ctx.v_out[li, b, kv]), v[keep])
        announce(f"full size C3: layer {li} seq {b} head {kv}: max rel err {worst:.2e}, set {cls}")


def test_full_size_pseudo_queries(env):
    """The queries of the pseudo tokens at the benchmark's shape (32 layers of a 4096-wide model, 64 pseudo tokens),
    in the configuration bench.py times: three layers against the oracle element by element, every layer against
    a property that holds at any size (the rotation keeps each channel pair's norm)."""
    bench, H = env
    w = W.workload("C2")
    announce("full size C2: queries of the pseudo tokens")
    ctx = bench.Context(w, 3, torch.device("cuda:0"))
    pq = bench.pseudo_query_problem(ctx)
    assert H.D.pseudo_queries_workspace_bytes(pq.desc) == 0          # the launch the benchmark times needs no split
    pq.run(rotate=False)
    torch.cuda.synchronize()
    pre = pq.q.clone()
    pq.run(rotate=True)
    torch.cuda.synchronize()
    rot = pq.q
    d, Hq, N = w.head_dim, w.n_q_heads, w.n_pseudo
    src = pq.src.cpu().numpy()
    pos = pq.pos.cpu().numpy()
    assert torch.isfinite(pre.float()).all() and torch.isfinite(rot.float()).all()
    # any size: per channel pair the rotation keeps the norm (up to the two bf16 roundings)
    p, r = pre.float(), rot.float()
    n_p = torch.hypot(p[..., : d // 2], p[..., d // 2:])
    n_r = torch.hypot(r[..., : d // 2], r[..., d // 2:])
    assert ((n_p - n_r).abs() <= 2.0 ** -7 * n_p + 1e-3).all()
    for layer in (0, 13, 31):
        x_bits = H.host_bits(pq.x[layer])
        w_bits = H.host_bits(pq.w_q[layer])
        want_pre = O.pseudo_queries(x_bits, src, w_bits, Hq)                        # [Hq, rows, d]
        got_pre = H.host_bits(pre[layer]).reshape(Hq, -1, d)
        assert (got_pre == want_pre).mean() > 0.99
        g, e = O.bf16_bits_to_f64(got_pre), O.bf16_bits_to_f64(want_pre)
        assert (np.abs(g - e) <= 2.0 ** -7 * np.abs(e) + 1e-4).all()               # one bf16 step at most
        want_rot = O.pseudo_queries(x_bits, src, w_bits, Hq, positions=pos, theta=w.theta)
        got_rot = H.host_bits(rot[layer]).reshape(Hq, -1, d)
        assert (got_rot == want_rot).mean() > 0.98
