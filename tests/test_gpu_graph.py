"""The whole step recorded into a HIP graph and replayed.

The library allocates nothing, clears its counters with kernels of its own and keeps no state between calls
besides the workspaces the caller owns, so a step (rotation of the pseudo queries, both score passes, max-pool +
TopK, gather) can be captured once and replayed by a serving loop.  Each case replays the graph several times, with
eager work of the program and synchronisations between the replays, and compares every replay bit for bit with the
eager step on the same inputs.  One eager step runs before the capture: the first call on a device does the
library's one-time set-up (dynamic-LDS limits, unit counts), which is not stream work.
"""
import os
import sys
from dataclasses import replace

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _cases():
    dense = W.workload("C1")                                                    # one wave per chunk, four to a workgroup
    ragged = replace(W.workload("C3"), n_layers=2, batch=5, ragged=(300, 2500), budget=96)   # teams, work lists, tickets
    empty_mix = replace(W.workload("C3"), n_layers=1, batch=4, ragged=(0, 700), n_pseudo=32, budget=40)
    long_head = replace(W.workload("C5"), n_layers=1, seq_len=70000, budget=1500, needles=8)  # selection in pieces
    one_kernel = replace(W.workload("C1"), seq_len=500, n_layers=3)             # both passes in one kernel
    return [("dense", dense, 3), ("one-kernel", one_kernel, 4), ("ragged", ragged, 5), ("ragged-short", empty_mix, 11),
            ("long-head", long_head, 7)]


@pytest.mark.parametrize("name,w,seed", _cases(), ids=[c[0] for c in _cases()])
def test_step_replays_from_a_graph(name, w, seed):
    import bench
    print(f"graph replay: {name} seed {seed}", flush=True)
    dev = torch.device("cuda:0")
    ctx = bench.Context(w, seed, dev)
    other = bench.Context(W.workload("C1"), seed + 1, dev)      # the program's own eager work between replays
    outs = {"q": ctx.q, "scores": ctx.S, "idx": ctx.idx, "count": ctx.count, "k_out": ctx.k_out, "v_out": ctx.v_out}
    if not ctx.single_launch:                                   # (a one-kernel score call writes no row statistics)
        outs["lse2"] = ctx.lse2

    ctx.step()
    torch.cuda.synchronize()
    want = {n: t.clone() for n, t in outs.items()}
    # every replay starts from scribbled intermediates and workspaces; what a step leaves untouched (index and cache
    # slots beyond a head's count) is not scribbled and is compared as the eager step left it
    def scribble():
        ctx.q.fill_(0)
        ctx.lse2.fill_(float("nan"))
        ctx.S.fill_(-1.0)
        ctx.ws.fill_(0xA5)
        if ctx.topk_ws is not None:
            ctx.topk_ws.fill_(0x5A)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    eager_stream = ctx.stream
    with torch.cuda.graph(graph, stream=side):
        ctx.stream = torch.cuda.current_stream()
        ctx.step()
    ctx.stream = eager_stream

    for replay in range(4):
        scribble()
        other.step()
        torch.cuda.synchronize()
        graph.replay()
        if replay % 2:
            other.step()                                         # eager work queued right behind a replay as well
        torch.cuda.synchronize()
        for what, t in outs.items():
            a, b = t.view(torch.uint8).reshape(-1), want[what].view(torch.uint8).reshape(-1)
            assert torch.equal(a, b), f"{name}: replay {replay}: {what} differs from the eager step"
    counts = ctx.count.cpu().numpy()
    lens = np.asarray(ctx.lens)
    assert (counts == np.minimum(lens, w.budget)[None, :, None]).all()


def test_static_scores_replay_from_a_graph():
    """dapq_score_static is the entry point for callers under capture: recorded once (after an ordinary first call, which
    looks up the address of the built-in scratch array), replayed between other users of the same array."""
    import paper_2603_11564_amd as D
    from dapq_harness import Problem
    print("graph replay: dapq_score_static", flush=True)
    rng = np.random.default_rng(21)
    lens = [900, 0, 37, 2100]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q = W.to_bf16_bits(rng.standard_normal((2, len(lens), 8, 32, 128)))
    k = W.to_bf16_bits(rng.standard_normal((2, int(cu[-1]), 2, 128)))
    ragged = Problem(q, k, k, 2, cu, "thd", 128 ** -0.5)
    qd = W.to_bf16_bits(rng.standard_normal((1, 1, 8, 64, 128)))
    kd = W.to_bf16_bits(rng.standard_normal((1, 3000, 2, 128)))
    dense = Problem(qd, kd, kd, 2, None, "thd", 128 ** -0.5)
    want_ragged, want_dense = ragged.score(), dense.score()
    S_ragged = torch.empty_like(want_ragged)
    S_dense = torch.empty_like(want_dense)
    D.dapq_score_static(dense.shape, dense.q, dense.k, S_dense)          # first call on the device: set-up
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        D.dapq_score_static(ragged.shape, ragged.q, ragged.k, S_ragged, torch.cuda.current_stream())
    for replay in range(3):
        S_ragged.fill_(float("nan"))
        S_dense.fill_(float("nan"))
        D.dapq_score_static(dense.shape, dense.q, dense.k, S_dense)      # another user of the scratch array, in order
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(S_dense, want_dense), f"replay {replay}: eager call between replays"
        assert torch.equal(S_ragged, want_ragged), f"replay {replay}: captured call"
