"""GPU parity: every C-ABI entry point of libdapq.so against the float64 oracle, element by element,
on seeded inputs that span several tiles and ragged tails, plus the degenerate cases."""
import sys
import zlib

import numpy as np
import pytest
import torch

import workloads as W
from oracle import dapq_oracle as O

pytestmark = pytest.mark.gpu


def announce(msg):
    print(f"[gpu-case] {msg}", file=sys.__stderr__, flush=True)


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import dapq_harness
    return dapq_harness


def random_problem(seed, layers, lens, Hq, Hkv, N, d=128, gain=1.0):
    r = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q = W.to_bf16_bits(r.standard_normal((layers, len(lens), Hq, N, d)) * gain)
    k = W.to_bf16_bits(r.standard_normal((layers, int(cu[-1]), Hkv, d)) * gain)
    v = r.integers(0, 65536, size=k.shape, dtype=np.uint16)
    return q, k, v, cu


# ----------------------------------------------------------------------------------------- rope
@pytest.mark.parametrize("pairing", [0, 1])
def test_rope_matches_oracle_bits(H, pairing):
    announce(f"rope pairing={pairing}")
    r = np.random.default_rng(100 + pairing)
    bits = W.to_bf16_bits(r.standard_normal((777, 5, 128)))
    pos = r.integers(0, 140000, size=777).astype(np.int32)
    pos[:3] = [0, 1, 131071 + 63]
    got = H.rope_gpu(bits, pos, 500000.0, pairing)
    want = O.rope_apply(bits, pos, 500000.0, "half" if pairing == 0 else "interleaved")
    diff = got.astype(np.int32) - want.astype(np.int32)
    mism = np.count_nonzero(diff)
    # both sides evaluate the rotation in fp64 and round once: a mismatch needs an fp64 last-bit
    # difference to straddle a bf16 rounding boundary
    assert np.abs(diff).max() <= 1 and mism <= 2, f"{mism} of {diff.size} elements differ"
    assert np.array_equal(got[0], bits[0])                     # position 0 is the identity


@pytest.mark.parametrize("pairing", [0, 1])
def test_rope_unaligned_buffers_and_small_head_dims(H, pairing):
    """Buffers that are only 2-byte aligned give the bits of aligned ones (and the oracle's); head_dim 2, 4 and 6 (one
    channel pair, two, an odd number)."""
    announce(f"rope unaligned / small head_dim, pairing={pairing}")
    import paper_2603_11564_amd as D
    r = np.random.default_rng(300 + pairing)
    rows, heads, d = 130, 11, 128
    bits = W.to_bf16_bits(r.standard_normal((rows, heads, d)))
    pos = r.integers(0, 200000, size=rows).astype(np.int32)
    want = O.rope_apply(bits, pos, 500000.0, "half" if pairing == 0 else "interleaved")
    wide = H.rope_gpu(bits, pos, 500000.0, pairing)
    flat_in = torch.zeros(bits.size + 1, dtype=torch.bfloat16, device="cuda")
    flat_out = torch.zeros_like(flat_in)
    x, y = flat_in[1:].view(rows, heads, d), flat_out[1:].view(rows, heads, d)
    assert x.data_ptr() % 4 == 2
    x.copy_(H.dev_bf16(bits))
    D.dapq_rope_apply(x, y, torch.from_numpy(pos).cuda(), rows, heads, d, heads * d, d, 500000.0, pairing)
    narrow = H.host_bits(y)
    assert np.array_equal(narrow, wide)
    diff = wide.astype(np.int32) - want.astype(np.int32)
    assert np.abs(diff).max() <= 1 and np.count_nonzero(diff) <= 2
    for small_d in (2, 6, 4):
        b = W.to_bf16_bits(r.standard_normal((37, 3, small_d)))
        ps = r.integers(0, 5000, size=37).astype(np.int32)
        got = H.rope_gpu(b, ps, 10000.0, pairing)
        ref = O.rope_apply(b, ps, 10000.0, "half" if pairing == 0 else "interleaved")
        dd = got.astype(np.int32) - ref.astype(np.int32)
        assert np.abs(dd).max() <= 1 and np.count_nonzero(dd) <= 1, f"head_dim {small_d}"


def test_rope_in_place_and_pseudo_query_positions(H):
    announce("rope in place, C1 pseudo queries")
    w = W.workload("C1")
    p = W.host_problem(w, 5)
    q_rows = np.ascontiguousarray(p["q"][0, 0].transpose(1, 0, 2))          # [N, Hq, d]
    x = H.dev_bf16(q_rows)
    pos = torch.from_numpy(p["q_pos"][0]).cuda()
    import paper_2603_11564_amd as D
    D.dapq_rope_apply(x, x, pos, w.n_pseudo, w.n_q_heads, 128, w.n_q_heads * 128, 128, w.theta, 0)
    want = O.rope_apply(q_rows, p["q_pos"][0], w.theta)
    assert np.array_equal(H.host_bits(x), want)


# ----------------------------------------------------------------------------------------- score
SCORE_CASES = [
    # name, layers, lens, Hq, Hkv, N, layout
    ("c1-like hnd", 1, [1024], 32, 8, 64, "hnd"),
    ("ragged tail thd", 2, [1000], 8, 2, 64, "thd"),
    ("tiny lengths", 1, [1, 5, 31, 33, 129, 2], 4, 2, 8, "thd"),
    ("N=1 g=1", 1, [300], 2, 2, 1, "thd"),
    ("N=3 g=4 (12 rows)", 1, [700], 8, 2, 3, "hnd"),
    ("R=64", 1, [513], 4, 1, 64, "thd"),
    ("R=128", 1, [515], 8, 2, 32, "thd"),
    ("R=512 two super-groups", 1, [400, 260], 8, 2, 128, "thd"),
    ("R=640 g=5", 1, [257], 5, 1, 128, "thd"),
    ("R=2048 eight row groups", 1, [300], 4, 1, 512, "thd"),
    ("R=512 several chunks", 1, [5000], 8, 2, 128, "hnd"),
    ("long chunked", 1, [9000], 4, 1, 64, "hnd"),
    ("ragged with empty", 1, [130, 0, 64, 0], 4, 2, 16, "thd"),
]


@pytest.mark.parametrize("case", SCORE_CASES, ids=[c[0] for c in SCORE_CASES])
def test_score_matches_oracle(H, case):
    name, layers, lens, Hq, Hkv, N, layout = case
    announce(f"score {name}")
    q, k, v, cu = random_problem(zlib.crc32(name.encode()) % 1000, layers, lens, Hq, Hkv, N)
    ragged = len(lens) > 1
    prob = H.Problem(q, k, v, Hkv, cu if ragged else None, layout)
    S = prob.score().cpu().numpy()
    lse = prob.stats().cpu().numpy()
    want = O.score(q, k, Hkv, cu if ragged else None)
    worst = H.assert_scores_close(S, want, name)
    # every row's normaliser: log2 sum_j exp(l_j)
    g = Hq // Hkv
    for l in range(layers):
        for b, (s, e) in enumerate(prob.seq_bounds()):
            if e == s:
                continue
            for h in range(Hq):
                logits = O.bf16_bits_to_f64(q[l, b, h]) @ O.bf16_bits_to_f64(k[l, s:e, h // g]).T / np.sqrt(128)
                m = logits.max(axis=1)
                ref = (m + np.log(np.exp(logits - m[:, None]).sum(axis=1))) / np.log(2)
                assert np.abs(lse[l, b, h] - ref).max() < 2e-4, name
    for l in range(layers):
        for kv in range(Hkv):
            for b, (s, e) in enumerate(prob.seq_bounds()):
                if e > s:
                    assert abs(S[l, kv, s:e].sum() - g * N) < 1e-3 * g * N
    announce(f"score {name}: max rel err {worst:.2e}")


# dense batches whose sequences are at most 4 chunks of keys and whose KV heads have at most 256 query rows: dapq_score
# runs both passes in one kernel.  name, layers, batch, L, Hq, Hkv, N, layout
FUSED_CASES = [
    ("one chunk", 1, 1, 100, 4, 2, 16, "thd"),
    ("two chunks", 2, 1, 200, 8, 2, 32, "thd"),
    ("three chunks", 2, 1, 300, 4, 2, 32, "thd"),
    ("batch of four, three chunks each", 1, 4, 333, 8, 2, 64, "thd"),
    ("batch of seven, two chunks each", 1, 7, 190, 4, 1, 16, "thd"),
    ("four chunks, ragged tail", 1, 1, 450, 8, 2, 64, "hnd"),
    ("four full chunks", 1, 1, 512, 4, 1, 64, "thd"),
    ("batch of three, four chunks each", 1, 3, 400, 8, 2, 16, "thd"),
    ("batch of five, one chunk each", 2, 5, 77, 4, 2, 8, "thd"),
    ("few rows (N=3, g=4)", 1, 1, 256, 8, 2, 3, "thd"),
    ("many heads, 512-key chunks", 32, 1, 2048, 16, 8, 64, "hnd"),
]


@pytest.mark.parametrize("case", FUSED_CASES, ids=[c[0] for c in FUSED_CASES])
def test_fused_score_equals_the_separate_passes(H, case):
    """One kernel for both passes gives the bits of pass 1 + merge + pass 2 (same arithmetic in the same order), and the
    oracle's scores."""
    name, layers, batch, L, Hq, Hkv, N, layout = case
    announce(f"fused score: {name}")
    q, k, v, cu = random_problem(zlib.crc32(name.encode()) % 1000, layers, [L] * batch, Hq, Hkv, N)
    prob = H.Problem(q, k, v, Hkv, None, layout)
    assert H.D.score_single_launch(prob.shape), name
    S = prob.score()
    S_split = prob.score_split()
    assert torch.equal(S, S_split), name
    if layers <= 2:
        H.assert_scores_close(S.cpu().numpy(), O.score(q, k, Hkv, cu if batch > 1 else None), name)
    else:                                                           # the oracle on a sample of the heads
        Sh = S.cpu().numpy()
        g = Hq // Hkv
        for l, kv in ((0, 0), (17, 3), (31, 7)):
            want = O.score(q[l:l + 1, :, kv * g:(kv + 1) * g], k[l:l + 1, :, kv:kv + 1], 1)
            H.assert_scores_close(Sh[l:l + 1, kv:kv + 1], want, f"{name} layer {l} head {kv}")


def test_fused_score_dominant_late_key(H):
    """The overflow path of pass 1 (a chunk redone with a running maximum) inside the one-kernel form."""
    announce("fused score: dominant late key")
    q, k, v, cu = random_problem(17, 1, [500], 4, 1, 16)
    qf = O.bf16_bits_to_f64(q[0, 0, 0, 0])
    k[0, 430, 0] = W.to_bf16_bits(40.0 * qf)
    k[0, 17, 0] = W.to_bf16_bits(-40.0 * qf)
    prob = H.Problem(q, k, v, 1, None, "thd")
    assert H.D.score_single_launch(prob.shape)
    S = prob.score()
    assert torch.equal(S, prob.score_split())
    H.assert_scores_close(S.cpu().numpy(), O.score(q, k, 1), "fused dominant key")
    assert S[0, 0, 430].item() > 1.0


def test_score_c1_workload_with_needles(H):
    announce("score C1 workload")
    w = W.workload("C1")
    p = W.host_problem(w, 0)
    q, k = H.rope_problem_oracle(p, w.theta)
    prob = H.Problem(q, k, p["v"], w.n_kv_heads, None, "hnd", w.scale)
    S = prob.score().cpu().numpy()
    H.assert_scores_close(S, O.score(q, k, w.n_kv_heads), "C1")
    S2 = prob.score().cpu().numpy()
    assert np.array_equal(S, S2), "two runs differ bit for bit"


def test_score_dominant_late_key_takes_overflow_path(H):
    # one key far above the reference logit of the first sub-block: the fast pass overflows and the
    # chunk is redone with a running maximum; all mass must land on that key
    announce("score dominant late key")
    q, k, v, cu = random_problem(7, 1, [3000], 4, 1, 16)
    qf = O.bf16_bits_to_f64(q[0, 0, 0, 0])
    k[0, 2500, 0] = W.to_bf16_bits(40.0 * qf)             # logit ~ 40*128/11.3 ~ 450 for that row
    k[0, 17, 0] = W.to_bf16_bits(-40.0 * qf)
    prob = H.Problem(q, k, v, 1, None, "thd")
    S = prob.score().cpu().numpy()
    want = O.score(q, k, 1)
    H.assert_scores_close(S, want, "dominant key")
    assert S[0, 0, 2500] > 1.0


def test_score_all_equal_keys_uniform(H):
    announce("score all-equal keys")
    q, k, v, cu = random_problem(8, 1, [517], 8, 2, 8)
    k[:] = k[:, :1]
    prob = H.Problem(q, k, v, 2, None, "thd")
    S = prob.score().cpu().numpy()
    assert np.allclose(S, 4 * 8 / 517, rtol=1e-5)


def test_score_scale_and_large_gain(H):
    announce("score custom scale / heavy keys")
    q, k, v, cu = random_problem(9, 1, [640], 4, 2, 32, gain=1.0)
    k[0, ::10] = W.to_bf16_bits(4.0 * W.from_bf16_bits(k[0, ::10]))        # heavy-hitter tail
    prob = H.Problem(q, k, v, 2, None, "thd", scale=0.2)
    S = prob.score().cpu().numpy()
    H.assert_scores_close(S, O.score(q, k, 2, None, 0.2), "scale 0.2")


EXTENDED_CASES = [
    # name, layers, lens, Hq, Hkv, N, gain
    ("N64 g4 one sequence", 1, [700], 8, 2, 64, 1.0),
    ("N1 g1: a single pseudo key", 1, [33], 2, 2, 1, 1.0),
    ("N5 g2 ragged, short prompts", 2, [3, 40, 0, 129], 4, 2, 5, 1.0),
    ("N128 g4: two row groups", 1, [300], 4, 1, 128, 1.0),
    ("N40 g3: rows not a multiple of 32, sharp logits", 1, [257], 6, 2, 40, 3.0),
]


@pytest.mark.parametrize("case", EXTENDED_CASES, ids=[c[0] for c in EXTENDED_CASES])
def test_score_extended_normaliser_matches_oracle(H, case):
    """Sec. 4.1 prefills the pseudo tokens in-sequence: the causal block of their own keys joins
    every row's normaliser (dapq_score_stats_extend between the two passes)."""
    name, layers, lens, Hq, Hkv, N, gain = case
    announce(f"score, extended normaliser: {name}")
    q, k, v, cu = random_problem(31, layers, lens, Hq, Hkv, N, gain=gain)
    kp = W.to_bf16_bits(np.random.default_rng(32).standard_normal((layers, len(lens), Hkv, N, 128)) * gain)
    prob = H.Problem(q, k, v, Hkv, cu if len(lens) > 1 else None, "thd")
    S = prob.score_extended(kp).cpu().numpy()
    want = O.score(q, k, Hkv, cu, None, kp)
    H.assert_scores_close(S, want, name)
    # the pseudo keys only take mass away from the prompt keys
    plain = prob.score().cpu().numpy()
    assert (S <= plain * (1 + 1e-6)).all()


# ----------------------------------------------------------------------------------------- pool
@pytest.mark.parametrize("width", [1, 3, 7, 9, 11, 63])
def test_pool_bit_exact(H, width):
    announce(f"pool width={width}")
    r = np.random.default_rng(width)
    lens = [1, 2, 6, 7, 8, 255, 256, 257, 1000, 3, 0, 1029]
    q, k, v, cu = random_problem(1, 2, lens, 2, 2, 1)
    prob = H.Problem(q, k, v, 2, cu, "thd")
    S = r.random((2, 2, int(cu[-1]))).astype(np.float32)
    S[0, 0, ::5] = S[0, 0, 1]                                   # ties
    P = prob.pool(torch.from_numpy(S).cuda(), width).cpu().numpy()
    for l in range(2):
        for kv in range(2):
            for b in range(len(lens)):
                s, e = cu[b], cu[b + 1]
                want = O.pool(S[l, kv, s:e].astype(np.float64), width)
                assert np.array_equal(P[l, kv, s:e].astype(np.float64), want), (width, l, kv, b)


def test_pool_dense_batch_unaligned_total(H):
    announce("pool dense, total % 4 != 0")
    q, k, v, cu = random_problem(2, 1, [333, 333, 333], 2, 1, 1)
    prob = H.Problem(q, k, v, 1, None, "thd")
    S = np.random.default_rng(3).random((1, 1, 999)).astype(np.float32)
    P = prob.pool(torch.from_numpy(S).cuda(), 7).cpu().numpy()
    for b in range(3):
        want = O.pool(S[0, 0, 333 * b:333 * (b + 1)].astype(np.float64), 7)
        assert np.array_equal(P[0, 0, 333 * b:333 * (b + 1)].astype(np.float64), want)


# ----------------------------------------------------------------------------------------- top-K
def _topk_case(H, lens, budget, P, per_seq=None, layers=1, Hkv=2, dense=False, pieces=True):
    q, k, v, cu = random_problem(4, layers, lens, Hkv, Hkv, 1)
    prob = H.Problem(q, k, v, Hkv, None if dense else cu, "thd")
    idx, count = prob.topk(torch.from_numpy(P).cuda(), budget, per_seq, pieces)
    idx, count = idx.cpu().numpy(), count.cpu().numpy()
    for l in range(layers):
        for b in range(len(lens)):
            kb = budget if per_seq is None else max(0, min(budget, per_seq[b]))
            n = min(kb, lens[b])
            for kv in range(Hkv):
                assert count[l, b, kv] == n
                want = O.topk(P[l, kv, cu[b]:cu[b + 1]].astype(np.float64), kb)
                assert np.array_equal(idx[l, b, kv, :n], want), (l, b, kv)
                assert (idx[l, b, kv, n:] == -7).all()          # slots past count untouched


def test_topk_bit_exact_with_ties_and_plateaus(H):
    announce("topk ties / plateaus")
    r = np.random.default_rng(5)
    lens = [1, 7, 100, 1023, 1024, 1025, 5000, 0, 40000]
    tot = sum(lens)
    P = r.random((1, 2, tot)).astype(np.float32)
    P[0, 0] = np.round(P[0, 0] * 8) / 8                         # 9 distinct values: huge ties
    P[0, 1, 10000:30000] = 0.5                                  # plateau straddling the boundary
    for budget in (1, 64, 983, 5000):
        _topk_case(H, lens, budget, P)


def test_topk_pooled_scores_and_per_sequence_budgets(H):
    announce("topk on pooled scores, per-sequence budgets")
    r = np.random.default_rng(6)
    lens = [3000, 50, 2048]
    S = (r.random((2, 2, sum(lens))) ** 8).astype(np.float64)
    cu = np.concatenate([[0], np.cumsum(lens)])
    P = np.zeros_like(S)
    for l in range(2):
        for kv in range(2):
            for b in range(3):
                P[l, kv, cu[b]:cu[b + 1]] = O.pool(S[l, kv, cu[b]:cu[b + 1]], 7)
    _topk_case(H, lens, 300, P.astype(np.float32), per_seq=[300, 0, 10000], layers=2)


def test_topk_all_equal_and_tiny_values(H):
    announce("topk all equal / denormal-scale values")
    lens = [777]
    P = np.full((1, 2, 777), 0.25, dtype=np.float32)
    P[0, 1] = (np.arange(777) % 13).astype(np.float32) * np.float32(1e-41)   # subnormals and zeros
    _topk_case(H, lens, 100, P)


@pytest.mark.parametrize("L", [3000, 12000, 30000, 60000])
def test_topk_both_signs_over_many_binades(H, L):
    """Scores of both signs from 1e-30 to 1e30, with infinities: the first radix digit (sign and exponent) spreads
    over the whole histogram, which takes the selection off its packed first-pass counting, in every kernel variant."""
    announce(f"topk both signs, wide range, L={L}")
    r = np.random.default_rng(L + 1)
    P = (r.standard_normal((1, 2, L)) * 10.0 ** r.uniform(-30, 30, (1, 2, L))).astype(np.float32)
    P[0, 0, 17] = np.inf
    P[0, 0, 1000] = -np.inf
    P[0, 1, ::7] = P[0, 1, 3]                                   # ties
    for budget in (5, 983, L - 1):
        _topk_case(H, [L], budget, P, dense=True)


@pytest.mark.parametrize("pieces", [False, True])
def test_topk_long_sequence_not_staged_in_lds(H, pieces):
    """A head longer than a workgroup's registers hold: streamed from memory (no workspace) or selected in pieces of
    32768 keys whose candidates are then selected among (with the workspace)."""
    announce(f"topk L=70000 pieces={pieces}")
    r = np.random.default_rng(7)
    P = r.random((1, 1, 70000)).astype(np.float32)
    P[0, 0, 5000:5100] = 2.0
    _topk_case(H, [70000], 2048, P, Hkv=1, pieces=pieces)


@pytest.mark.parametrize("lens,dense,budget", [([131072], True, 3932), ([200001], True, 983), ([65537] * 2, True, 5),
                                               ([70000, 3, 0, 140001, 9000], False, 2048),
                                               ([98304], True, 40000)])
def test_topk_long_heads_in_pieces(H, lens, dense, budget):
    """Long heads through the candidate lists: the 70B-class length, a length that is no multiple of anything, a
    ragged batch that mixes heads of every kind, ties that straddle the piece boundaries, a plateau over a whole
    piece, and a budget larger than a piece (every piece survives whole)."""
    announce(f"topk in pieces lens={lens} budget={budget}")
    r = np.random.default_rng(sum(lens) + budget)
    tot = sum(lens)
    P = (r.random((1, 2, tot)) ** 5).astype(np.float32)
    P[0, 0] = np.round(P[0, 0] * 16) / 16                       # 17 distinct values: ties across every boundary
    P[0, 1, 30000:66000] = 0.5                                  # plateau over all of the second piece
    if budget * ((max(lens) + 32767) // 32768) > 65536:
        q, k, v, cu = random_problem(4, 1, lens, 2, 2, 1)
        prob = H.Problem(q, k, v, 2, None if dense else cu, "thd")
        assert H.D.topk_workspace_bytes(prob.shape, budget) == 0   # too many candidates: the streaming kernel serves
    _topk_case(H, lens, budget, P, dense=dense, pieces=True)
    if not dense:   # per-sequence budgets, one of them 0, one larger than the common budget
        _topk_case(H, lens, budget, P, per_seq=[100, 5, 0, 10 * budget, 0][:len(lens)], dense=False, pieces=True)


@pytest.mark.parametrize("L,batch", [(8192, 1), (8193, 3), (16384, 2), (16385, 1), (20001, 2), (32767, 3), (32768, 1),
                                     (32769, 2), (50001, 1), (65536, 1), (65537, 1)])
def test_topk_dense_lengths_around_the_variant_limits(H, L, batch):
    """Dense batches at the lengths where the kernel variant changes (256, 512 or 1024 threads with 32 keys each, 1024
    with 64, then pieces or streaming), with sequence starts that are not 16-byte aligned, heavy ties and a plateau
    across the threshold."""
    announce(f"topk dense L={L} batch={batch}")
    r = np.random.default_rng(L)
    P = (r.random((1, 1, L * batch)) ** 6).astype(np.float32)
    P[0, 0, : L // 2] = np.round(P[0, 0, : L // 2] * 64) / 64
    P[0, 0, L // 3: L // 3 + 3000] = 0.75
    for budget in (7, 983, 3932):
        _topk_case(H, [L] * batch, budget, P, Hkv=1, dense=True)


_POOL_TOPK_SHAPES = [([5000], True), ([8193] * 2, True), ([20001] * 2, True), ([40000], True), ([70000], True),
                     ([131072], True), ([1, 6, 100, 1025, 0, 4097], False), ([70000, 3, 0, 40000], False)]
# long heads (more than 32768 keys; a ragged batch counts with its total) also go in pieces through the workspace
_POOL_TOPK_CASES = [(lens, dense, pieces) for lens, dense in _POOL_TOPK_SHAPES
                    for pieces in ([False, True] if (max(lens) if dense else sum(lens)) > 32768 else [False])]


@pytest.mark.parametrize("width", [1, 3, 5, 7, 9, 11])
@pytest.mark.parametrize("lens,dense,pieces", _POOL_TOPK_CASES)
def test_pool_topk_one_call_equals_the_two(H, width, lens, dense, pieces):
    """dapq_pool_topk against the oracle's pool followed by its top-K, for windows the selection kernel
    pools itself (<= 9), a window it does not (11), head lengths of every kernel variant and a ragged
    batch (sequence ends clip the window); with and without the pooled output."""
    announce(f"pool+topk width={width} lens={lens} dense={dense} pieces={pieces}")
    r = np.random.default_rng(width * 1000 + len(lens))
    tot = sum(lens)
    S = (r.random((1, 2, tot)) ** 4).astype(np.float32)
    S[0, 0] = np.round(S[0, 0] * 32) / 32                       # ties before pooling: longer plateaus after
    q, k, v, cu = random_problem(4, 1, lens, 2, 2, 1)
    prob = H.Problem(q, k, v, 2, None if dense else cu, "thd")
    Sd = torch.from_numpy(S).cuda()
    fusable = width <= 9 and ((max(lens) if dense else tot) <= 65536 or pieces)
    for budget, want_pooled in ((983, True), (64, False)):
        if not want_pooled and not fusable:
            with pytest.raises(H.D.DapqError):
                prob.pool_topk(Sd, width, budget, None, False, pieces)
            continue
        idx, count, P = prob.pool_topk(Sd, width, budget, None, want_pooled, pieces)
        idx, count = idx.cpu().numpy(), count.cpu().numpy()
        for b in range(len(lens)):
            for kv in range(2):
                Pw = O.pool(S[0, kv, cu[b]:cu[b + 1]].astype(np.float64), width)
                if want_pooled:
                    assert np.array_equal(P[0, kv, cu[b]:cu[b + 1]].cpu().numpy().astype(np.float64), Pw), (b, kv)
                n = min(budget, lens[b])
                assert count[0, b, kv] == n
                assert np.array_equal(idx[0, b, kv, :n], O.topk(Pw, budget)), (b, kv)


# ----------------------------------------------------------------------------------------- gather
@pytest.mark.parametrize("layout", ["thd", "hnd"])
def test_gather_bit_exact(H, layout):
    announce(f"gather {layout}")
    lens = [300, 5, 64] if layout == "thd" else [400]
    q, k, v, cu = random_problem(11, 2, lens, 4, 2, 1)
    prob = H.Problem(q, k, v, 2, cu if len(lens) > 1 else None, layout)
    r = np.random.default_rng(12)
    budget = 40
    idx = np.full((2, len(lens), 2, budget), -1, dtype=np.int32)
    count = np.zeros((2, len(lens), 2), dtype=np.int32)
    for l in range(2):
        for b, L in enumerate(lens):
            for kv in range(2):
                n = min(budget, L) if (l + b + kv) % 3 else min(budget, L) // 2
                count[l, b, kv] = n
                idx[l, b, kv, :n] = np.sort(r.choice(L, size=n, replace=False))
    ko, vo = prob.gather(torch.from_numpy(idx).cuda(), torch.from_numpy(count).cuda(), budget)
    ko, vo = H.host_bits(ko), H.host_bits(vo)
    for l in range(2):
        for b in range(len(lens)):
            for kv in range(2):
                n = count[l, b, kv]
                rows = idx[l, b, kv, :n]
                assert np.array_equal(ko[l, b, kv, :n], O.gather(k[l, cu[b]:cu[b + 1], kv], rows))
                assert np.array_equal(vo[l, b, kv, :n], O.gather(v[l, cu[b]:cu[b + 1], kv], rows))
                assert (ko[l, b, kv, n:] == 0).all() and (vo[l, b, kv, n:] == 0).all()


# ----------------------------------------------------------------------------------------- chain
def run_chain(H, prob, budget, width, per_seq=None):
    S = prob.score()
    P = prob.pool(S, width)
    idx, count = prob.topk(P, budget, per_seq)
    ko, vo = prob.gather(idx, count, budget)
    return S.cpu().numpy(), P.cpu().numpy(), idx.cpu().numpy(), count.cpu().numpy(), H.host_bits(ko), H.host_bits(vo)


def compare_chain(H, prob, q, k, v, budget, width, per_seq=None, scale=None):
    cu = prob.cu_host
    S, P, idx, count, ko, vo = run_chain(H, prob, budget, width, per_seq)
    ref = O.compress(q, k, v, prob.Hkv, budget if per_seq is None else per_seq, cu, width, scale)
    H.assert_scores_close(S, ref["S"], "S")
    H.assert_scores_close(P, ref["P"], "P")
    classes = {"exact": 0, "margin": 0}
    for l in range(prob.layers):
        for b, (s, e) in enumerate(prob.seq_bounds()):
            kb = budget if per_seq is None else per_seq[b]
            for kv in range(prob.Hkv):
                n = min(kb, e - s)
                assert count[l, b, kv] == n == ref["count"][l, b, kv]
                classes[H.check_retained(ref["P"][l, kv, s:e], idx[l, b, kv], kb)] += 1
                rows = idx[l, b, kv, :n]
                assert np.array_equal(ko[l, b, kv, :n], k[l, s:e, kv][rows])
                assert np.array_equal(vo[l, b, kv, :n], v[l, s:e, kv][rows])
    return classes, idx


def test_chain_c1_workload_keeps_needles(H):
    announce("chain C1")
    w = W.workload("C1")
    for seed in (0, 1):
        p = W.host_problem(w, seed)
        # the GPU rotates its own inputs; the oracle rotates its own
        q_gpu = np.stack([H.rope_gpu(np.ascontiguousarray(p["q"][0, 0].transpose(1, 0, 2)), p["q_pos"][0],
                                     w.theta).transpose(1, 0, 2)])[None]
        k_gpu = H.rope_gpu(p["k"][0], p["k_pos"], w.theta)[None]
        q_ref, k_ref = H.rope_problem_oracle(p, w.theta)
        assert np.array_equal(q_gpu, q_ref) and np.array_equal(k_gpu, k_ref)
        prob = H.Problem(q_gpu, k_gpu, p["v"], w.n_kv_heads, None, "hnd", w.scale)
        classes, idx = compare_chain(H, prob, q_ref, k_ref, p["v"], w.budget, w.pool_width)
        for kv in range(w.n_kv_heads):
            pos, _, _ = W.needle_plan(w, seed, 0, 0, kv, w.seq_len)
            assert set(pos.tolist()) <= set(idx[0, 0, kv].tolist())
        announce(f"chain C1 seed {seed}: {classes}")


def test_chain_ragged_batch_heavy_hitters(H):
    announce("chain ragged heavy hitters (C3-like, small)")
    w = W.workload("C3")
    lens = [700, 1, 2500, 130]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    layers, N = 2, 128
    q = np.empty((layers, len(lens), w.n_q_heads, N, 128), dtype=np.uint16)
    k = np.empty((layers, int(cu[-1]), w.n_kv_heads, 128), dtype=np.uint16)
    v = np.empty_like(k)
    for l in range(layers):
        for b, L in enumerate(lens):
            qb = W.q_pre(w, 21, l, b)
            q[l, b] = O.rope_apply(qb.transpose(1, 0, 2), W.q_positions(L, N), w.theta).transpose(1, 0, 2)
            for kv in range(w.n_kv_heads):
                kb = W.k_pre(w, 21, l, b, kv, L)
                k[l, cu[b]:cu[b + 1], kv] = O.rope_apply(kb[:, None, :], W.k_positions(L), w.theta)[:, 0]
                v[l, cu[b]:cu[b + 1], kv] = W.v_rows(w, 21, l, b, kv, L)
    prob = H.Problem(q, k, v, w.n_kv_heads, cu, "thd", w.scale)
    classes, _ = compare_chain(H, prob, q, k, v, 512, 7)
    announce(f"chain ragged: {classes}")


def test_chain_budget_edges(H):
    announce("chain budget >= L, budget 1, L < pool width")
    q, k, v, cu = random_problem(31, 1, [5, 900, 64], 8, 2, 16)
    prob = H.Problem(q, k, v, 2, cu, "thd")
    compare_chain(H, prob, q, k, v, 64, 7)
    compare_chain(H, prob, q, k, v, 1, 7)
    compare_chain(H, prob, q, k, v, 1000, 7, per_seq=[2, 1000, 0])


# ----------------------------------------------------------------------------------------- recall, observation window
def test_recall_counts_match_oracle(H):
    """dapq_recall on index sets in dapq_topk's format against the set definition of Sec. 3.3."""
    announce("recall of retained sets")
    r = np.random.default_rng(21)
    layers, B, Hkv, L = 2, 3, 2, 5000
    bg, bp = 700, 300
    q, k, v, cu = random_problem(22, layers, [L] * B, Hkv, Hkv, 1)
    prob = H.Problem(q, k, v, Hkv, None, "thd")
    idx_g = np.full((layers, B, Hkv, bg), -3, dtype=np.int32)
    idx_p = np.full((layers, B, Hkv, bp), -3, dtype=np.int32)
    cnt_g = np.zeros((layers, B, Hkv), dtype=np.int32)
    cnt_p = np.zeros_like(cnt_g)
    for l in range(layers):
        for b in range(B):
            for kv in range(Hkv):
                ng = [bg, 1, 257, 0][(l + b + kv) % 4]
                npred = [bp, 0, 64][(l + 2 * b + kv) % 3]
                pool_ = r.choice(L, size=900, replace=False)             # both sets drawn from 900 positions: they overlap
                cnt_g[l, b, kv], cnt_p[l, b, kv] = ng, npred
                idx_g[l, b, kv, :ng] = np.sort(r.choice(pool_, size=ng, replace=False))
                idx_p[l, b, kv, :npred] = np.sort(r.choice(pool_, size=npred, replace=False))
    common = torch.full((layers, B, Hkv), -1, dtype=torch.int32, device="cuda")
    rec = torch.full((layers, B, Hkv), float("nan"), dtype=torch.float32, device="cuda")
    H.D.dapq_recall(prob.shape, torch.from_numpy(idx_g).cuda(), torch.from_numpy(cnt_g).cuda(), bg,
                    torch.from_numpy(idx_p).cuda(), torch.from_numpy(cnt_p).cuda(), bp, common, rec)
    common, rec = common.cpu().numpy(), rec.cpu().numpy()
    for l in range(layers):
        for b in range(B):
            for kv in range(Hkv):
                ng, npred = cnt_g[l, b, kv], cnt_p[l, b, kv]
                want = len(set(idx_g[l, b, kv, :ng].tolist()) & set(idx_p[l, b, kv, :npred].tolist()))
                assert common[l, b, kv] == want
                if ng > 0:
                    assert rec[l, b, kv] == np.float32(want) / np.float32(ng)
                    assert abs(rec[l, b, kv] - O.recall(idx_g[l, b, kv, :ng], idx_p[l, b, kv, :npred])) < 1e-6
                else:
                    assert rec[l, b, kv] == 0.0


def test_observation_window_scores_by_composition(H):
    """The observation window of Sec. 1 / Sec. 3.3 (the last N prompt tokens as queries, causal inside the
    window) needs no kernel of its own: pass 1 over the keys before the window, the causal block of the
    window's own keys via dapq_score_stats_extend, pass 2 over the keys before the window.  The result is
    the accumulated attention the window pays to every earlier key."""
    announce("observation window by composition")
    layers, B, Hq, Hkv, N, L, d = 2, 2, 4, 2, 16, 300, 128
    r = np.random.default_rng(23)
    k_bits = W.to_bf16_bits(r.standard_normal((layers, B * L, Hkv, d)))
    q_bits = W.to_bf16_bits(r.standard_normal((layers, B, Hq, N, d)))          # queries of the last N tokens
    k = H.dev_bf16(k_bits)
    q = H.dev_bf16(q_bits)
    Lp = L - N                                                                   # keys before the window
    tok, seq, lay = Hkv * d, L * Hkv * d, B * L * Hkv * d
    # the batch as the library sees it: B sequences of Lp keys, each followed by N rows (the window) it skips
    shape = H.D.make_shape(n_layers=layers, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, n_pseudo=N, total_tokens=B * Lp,
                           k_strides=(lay, N * tok, d, tok), v_strides=(lay, N * tok, d, tok),
                           q_strides=(B * Hq * N * d, Hq * N * d, N * d, d), scale=d ** -0.5)
    ws = torch.empty(max(H.D.workspace_bytes(shape), 256), dtype=torch.uint8, device="cuda")
    lse = torch.empty((layers, B, Hq, N), dtype=torch.float32, device="cuda")
    S = torch.full((layers, Hkv, B * Lp), float("nan"), dtype=torch.float32, device="cuda")
    H.D.dapq_score_stats(shape, q, k, lse, ws)
    window_keys = k.view(layers, B, L, Hkv, d)[:, :, Lp:]                       # a view: same memory, offset Lp tokens
    H.D.dapq_score_stats_extend(shape, q, window_keys, (lay, seq, d, tok), lse)
    H.D.dapq_score_accumulate(shape, q, k, lse, S, ws)
    S = S.cpu().numpy()
    g = Hq // Hkv
    kf = O.bf16_bits_to_f64(k_bits).reshape(layers, B, L, Hkv, d)
    for l in range(layers):
        for b in range(B):
            for kv in range(Hkv):
                want = O.score_head(O.bf16_bits_to_f64(q_bits[l, b, kv * g:(kv + 1) * g]), kf[l, b, :Lp, kv], None,
                                    kf[l, b, Lp:, kv])
                H.assert_scores_close(S[l, kv, b * Lp:(b + 1) * Lp], want, f"window S[{l},{b},{kv}]")


# ----------------------------------------------------------------------------------------- decode over the compact cache
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (5, 1), (2, 2)])
def test_decode_step_over_the_compact_cache(H, Hq, Hkv):
    """Sec. 4.2, last paragraph: decoding uses only the compressed cache.  Eviction chain on the GPU, then one
    decode step of attention over the compact cache, against the oracle's attention over the same retained
    rows; and the distance to attention over the full cache stays inside the dropped-mass bound 2 m max|v|."""
    announce(f"decode step over the compact cache, {Hq} query / {Hkv} KV heads")
    layers, lens, N, budget = 2, [700, 40, 0, 300], 16, 64
    q, k, v_raw, cu = random_problem(41, layers, lens, Hq, Hkv, N)
    r = np.random.default_rng(42)
    v = W.to_bf16_bits(r.standard_normal(v_raw.shape))                          # values that are real numbers
    prob = H.Problem(q, k, v, Hkv, cu, "thd")
    idx, count, _ = prob.pool_topk(prob.score(), 7, budget, None, False)
    ko, vo = prob.gather(idx, count, budget)
    qd_bits = W.to_bf16_bits(r.standard_normal((layers, len(lens), Hq, 128)) * 2.0)
    out = torch.full((layers, len(lens), Hq, 128), float("nan"), dtype=torch.float32, device="cuda")
    H.D.dapq_decode_attention(prob.shape, H.dev_bf16(qd_bits), ko, vo, count, budget, out)
    out = out.cpu().numpy().astype(np.float64)
    idx, count = idx.cpu().numpy(), count.cpu().numpy()
    g = Hq // Hkv
    kf, vf, qd = O.bf16_bits_to_f64(k), O.bf16_bits_to_f64(v), O.bf16_bits_to_f64(qd_bits)
    for l in range(layers):
        for b, L in enumerate(lens):
            for hq in range(Hq):
                kv = hq // g
                n = count[l, b, kv]
                assert n == min(budget, L)
                if n == 0:
                    assert np.all(out[l, b, hq] == 0.0)
                    continue
                keep = idx[l, b, kv, :n]
                kk, vv = kf[l, cu[b]:cu[b + 1], kv], vf[l, cu[b]:cu[b + 1], kv]
                want = O.decode_attention(qd[l, b, hq][None], kk[keep], vv[keep])[0]
                vmax = np.abs(vv).max()
                assert np.all(np.abs(out[l, b, hq] - want) <= 1e-5 * vmax + 1e-4 * np.abs(want)), (l, b, hq)
                # against the full cache: bounded by the attention mass of the dropped keys
                alpha = O.attention(qd[l, b, hq][None], kk)[0]
                m = 1.0 - alpha[keep].sum()
                full = O.decode_attention(qd[l, b, hq][None], kk, vv)[0]
                assert np.abs(out[l, b, hq] - full).max() <= 2 * m * vmax + 1e-5 * vmax


@pytest.mark.parametrize("budget", [983, 2048, 8192])
def test_decode_attention_large_caches(H, budget):
    """The decode step on compact caches of the sizes the budgets of the workloads give (and the largest the entry
    point takes), filled directly: full, partly filled, one-row and empty heads."""
    announce(f"decode attention over caches of {budget} rows")
    layers, batch, Hq, Hkv, d = 1, 2, 8, 2, 128
    r = np.random.default_rng(budget)
    kc = W.to_bf16_bits(r.standard_normal((layers, batch, Hkv, budget, d)))
    vc = W.to_bf16_bits(r.standard_normal((layers, batch, Hkv, budget, d)))
    qd = W.to_bf16_bits(r.standard_normal((layers, batch, Hq, d)) * 2.0)
    count = np.array([[[budget, budget // 3], [1, 0]]], dtype=np.int32)
    q0, k0, v0, cu = random_problem(1, layers, [8] * batch, Hq, Hkv, 4)
    prob = H.Problem(q0, k0, v0, Hkv, cu, "thd")                                  # only the head counts and the scale are used
    out = torch.full((layers, batch, Hq, d), float("nan"), dtype=torch.float32, device="cuda")
    H.D.dapq_decode_attention(prob.shape, H.dev_bf16(qd), H.dev_bf16(kc), H.dev_bf16(vc),
                              torch.from_numpy(count).cuda(), budget, out)
    out = out.cpu().numpy().astype(np.float64)
    kf, vf, qf = O.bf16_bits_to_f64(kc), O.bf16_bits_to_f64(vc), O.bf16_bits_to_f64(qd)
    for b in range(batch):
        for hq in range(Hq):
            kv = hq // (Hq // Hkv)
            n = int(count[0, b, kv])
            if n == 0:
                assert np.all(out[0, b, hq] == 0.0)
                continue
            want = O.decode_attention(qf[0, b, hq][None], kf[0, b, kv, :n], vf[0, b, kv, :n])[0]
            assert np.all(np.abs(out[0, b, hq] - want) <= 1e-5 * np.abs(vf[0, b, kv, :n]).max() + 1e-4 * np.abs(want)), (b, hq)


def test_pseudo_tokens_and_positions(H):
    """Sec. 4.1 positions and the first-m / last-n content choice, for a ragged and a dense batch."""
    announce("pseudo tokens (first m + last n) and their positions")
    for lens, dense in (([1000, 3, 0, 50, 4097], False), ([777] * 3, True)):
        for m, n in ((4, 28), (2, 30), (0, 16), (8, 0)):
            q, k, v, cu = random_problem(5, 1, lens, 2, 2, m + n)
            prob = H.Problem(q, k, v, 2, None if dense else cu, "thd")
            tok = torch.full((len(lens), m + n), -9, dtype=torch.int32, device="cuda")
            pos = torch.full((len(lens), m + n), -9, dtype=torch.int32, device="cuda")
            H.D.dapq_pseudo_tokens(prob.shape, m, n, tok, pos)
            tok, pos = tok.cpu().numpy(), pos.cpu().numpy()
            for b, L in enumerate(lens):
                src, want_pos = O.pseudo_tokens(L, m, n)
                assert np.array_equal(pos[b], want_pos)
                assert np.array_equal(tok[b], np.where(src >= 0, src + cu[b], -1))


# ----------------------------------------------------------------------------------------- random shapes
@pytest.mark.parametrize("seed", range(100))
def test_chain_random_shapes(H, seed):
    """The whole step on seeded random shapes (head counts, pseudo-query counts, ragged or dense lengths
    with chunk-boundary values, both K layouts, window widths, budgets), both ways of selecting (two calls /
    one call), against the oracle's compress()."""
    r = np.random.default_rng(1000 + seed)
    layers = int(r.integers(1, 3))
    Hkv = int(r.choice([1, 2, 3]))
    g = int(r.choice([1, 2, 4, 5, 8]))
    N = int(r.choice([1, 7, 16, 32, 33, 64, 100, 128]))
    while g * N > 640:
        N //= 2
    dense = bool(r.integers(0, 2))
    special = [1, 31, 32, 33, 127, 128, 129, 255, 256, 257, 1023, 1024, 1025, 2047, 2048, 2049, 4100]
    if dense:
        lens = [int(r.choice(special + [int(r.integers(1, 3000))]))] * int(r.integers(1, 4))
    else:
        lens = [int(r.choice(special + [0, int(r.integers(1, 3000))])) for _ in range(int(r.integers(1, 5)))]
        if sum(lens) == 0:
            lens[0] = 77
    layout = "thd" if (not dense or len(lens) > 1 or r.integers(0, 2)) else "hnd"
    width = int(r.choice([1, 3, 7, 7, 7, 9, 13]))
    budget = int(r.choice([1, 5, 64, 300, 983]))
    gain = float(r.choice([0.5, 1.0, 2.5]))
    announce(f"random shape {seed}: layers {layers} Hkv {Hkv} g {g} N {N} lens {lens} dense {dense} {layout} "
             f"width {width} budget {budget} gain {gain}")
    q, k, v, cu = random_problem(2000 + seed, layers, lens, Hkv * g, Hkv, N, gain=gain)
    prob = H.Problem(q, k, v, Hkv, None if dense else cu, layout)
    classes, idx = compare_chain(H, prob, q, k, v, budget, width)
    # the one-call selection gives the same indices as the two calls
    idx2, count2, _ = prob.pool_topk(prob.score(), width, budget, None, True)
    assert np.array_equal(idx2.cpu().numpy(), idx)


def test_score_keys_with_a_huge_row_stride(H):
    """Keys that sit 2 MiB apart (a strided view of a wide buffer): the transfers' scalar and lane offsets
    reach into the gigabytes."""
    announce("score with k_stride_token = 2^20 elements")
    L, N, Hq, d, stride = 70, 8, 2, 128, 1 << 20
    r = np.random.default_rng(51)
    k_bits = W.to_bf16_bits(r.standard_normal((1, L, 1, d)))
    q_bits = W.to_bf16_bits(r.standard_normal((1, 1, Hq, N, d)))
    wide = torch.zeros((L, stride), dtype=torch.bfloat16, device="cuda")            # 140 MiB
    wide[:, :d] = H.dev_bf16(k_bits[0, :, 0])
    q = H.dev_bf16(q_bits)
    shape = H.D.make_shape(n_layers=1, batch=1, n_q_heads=Hq, n_kv_heads=1, n_pseudo=N, total_tokens=L,
                           k_strides=(0, 0, 0, stride), v_strides=(0, 0, 0, stride),
                           q_strides=(Hq * N * d, Hq * N * d, N * d, d), scale=d ** -0.5)
    ws = torch.empty(max(H.D.workspace_bytes(shape), 256), dtype=torch.uint8, device="cuda")
    S = torch.full((1, 1, L), float("nan"), dtype=torch.float32, device="cuda")
    H.D.dapq_score(shape, q, wide, S, ws)
    H.assert_scores_close(S.cpu().numpy(), O.score(q_bits, k_bits, 1), "S, strided keys")


# ----------------------------------------------------------------------------------------- several streams
def test_calls_on_two_streams_do_not_disturb_each_other(H):
    """Two problems scored at the same time on two streams, each with its own workspace and outputs, give the
    bits they give when run one after the other (the library keeps no state between or across calls)."""
    announce("two streams at once")
    D = H.D
    probs = []
    for seed, lens in ((201, [3000, 700]), (202, [2500, 2500])):
        q, k, v, cu = random_problem(seed, 2, lens, 8, 2, 32)
        probs.append(H.Problem(q, k, v, 2, cu, "thd"))
    alone = [p.score().clone() for p in probs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.zeros_like(a) for a in alone]
    for rep in range(3):
        for p, s, o in zip(probs, streams, outs):
            o.zero_()
            s.wait_stream(torch.cuda.current_stream())
        for p, s, o in zip(probs, streams, outs):
            D.dapq_score(p.shape, p.q, p.k, o, p.ws, s)
        torch.cuda.synchronize()
        for a, o in zip(alone, outs):
            assert torch.equal(a, o), rep


@pytest.mark.parametrize("ragged", [False, True])
def test_batch_of_empty_prompts(H, ragged):
    """total_tokens = 0: every entry point accepts the shape, writes count = 0 and lse2 = 0, and touches nothing else
    (the buffers that would hold keys are one dummy row, never read)."""
    announce(f"all prompts empty, ragged={ragged}")
    D = H.D
    layers, B, Hq, Hkv, N, d, budget = 2, 2, 4, 2, 8, 128, 5
    cu = torch.zeros(B + 1, dtype=torch.int32, device="cuda") if ragged else None
    shape = D.make_shape(n_layers=layers, batch=B, n_q_heads=Hq, n_kv_heads=Hkv, n_pseudo=N, total_tokens=0, cu_seqlens=cu,
                         k_strides=(0, 0, d, Hkv * d), v_strides=(0, 0, d, Hkv * d),
                         q_strides=(B * Hq * N * d, Hq * N * d, N * d, d), scale=d ** -0.5)
    q = torch.randn((layers, B, Hq, N, d), device="cuda").to(torch.bfloat16)
    k = torch.full((1, Hkv, d), float("nan"), device="cuda").to(torch.bfloat16)
    ws = torch.empty(max(D.workspace_bytes(shape), 256), dtype=torch.uint8, device="cuda")
    S = torch.full((layers, Hkv, 1), 7.0, dtype=torch.float32, device="cuda")
    lse = torch.full((layers, B, Hq, N), 7.0, dtype=torch.float32, device="cuda")
    D.dapq_score_stats(shape, q, k, lse, ws)
    D.dapq_score(shape, q, k, S, ws)
    idx = torch.full((layers, B, Hkv, budget), -7, dtype=torch.int32, device="cuda")
    count = torch.full((layers, B, Hkv), -7, dtype=torch.int32, device="cuda")
    D.dapq_pool_topk(shape, S, 7, budget, None, idx, count, None)
    ko = torch.full((layers, B, Hkv, budget, d), 3.0, device="cuda").to(torch.bfloat16)
    vo = ko.clone()
    D.dapq_gather(shape, k, k, idx, count, budget, ko, vo)
    torch.cuda.synchronize()
    assert (lse == 0).all() and (count == 0).all()
    assert (S == 7.0).all() and (idx == -7).all() and (ko == 3.0).all() and (vo == 3.0).all()


def test_chain_many_short_sequences(H):
    """A ragged batch of 300 short prompts (0 to 200 keys): per-sequence chunking, pooling that never crosses a
    sequence boundary, budgets clipped to the prompt lengths."""
    announce("300 short sequences")
    r = np.random.default_rng(77)
    lens = [int(v) for v in r.integers(0, 200, 300)]
    lens[5], lens[17] = 0, 1
    q, k, v, cu = random_problem(78, 1, lens, 4, 2, 8)
    prob = H.Problem(q, k, v, 2, cu, "thd")
    budget = 24
    S = prob.score()
    idx, count, _ = prob.pool_topk(S, 7, budget, None, False)
    ko, vo = prob.gather(idx, count, budget)
    want = O.compress(q, k, v, 2, budget, cu, 7)
    H.assert_scores_close(S.cpu().numpy(), want["S"], "many sequences")
    idx, count = idx.cpu().numpy(), count.cpu().numpy()
    assert np.array_equal(count, want["count"])
    kob, vob = H.host_bits(ko), H.host_bits(vo)
    exact = 0
    for b, L in enumerate(lens):
        for kv in range(2):
            n = count[0, b, kv]
            res = H.check_retained(want["P"][0, kv, cu[b]:cu[b + 1]], idx[0, b, kv], budget) if L > 0 else "exact"
            exact += res == "exact"
            keep = idx[0, b, kv, :n]
            assert np.array_equal(kob[0, b, kv, :n], k[0, cu[b]:cu[b + 1], kv][keep])
            assert np.array_equal(vob[0, b, kv, :n], v[0, cu[b]:cu[b + 1], kv][keep])
    assert exact > 500
