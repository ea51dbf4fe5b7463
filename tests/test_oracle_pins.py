"""Pins for the CPU oracle: closed forms, hand-worked fixtures, invariants, brute force and
independent library routines (scipy / torch on the CPU).  None of the expected values comes from
the oracle itself or from the GPU path."""
import math

import numpy as np
import pytest
import scipy.ndimage
import scipy.special
import torch

from oracle import dapq_oracle as O
import workloads as W


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ bf16 codec
def test_bf16_decode_known_patterns():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x3DCD, 0x7F7F, 0x0080], dtype=np.uint16)
    want = [1.0, -2.0, 0.0, -0.0, 0.10009765625, (2 - 2 ** -7) * 2.0 ** 127, 2.0 ** -126]
    got = O.bf16_bits_to_f64(bits)
    assert got.tolist() == want
    assert np.signbit(got[3])


def test_bf16_encode_ties_and_edges():
    # 8 significant bits: spacing at 1.0 is 2**-7; halfway cases go to the even mantissa
    x = np.array([1.0, 1 + 2 ** -8, 1 + 3 * 2 ** -8, 1 + 2 ** -8 + 2 ** -30, -(1 + 2 ** -8), 0.1,
                  2.0 ** -126, 2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -134, -0.0])
    want = np.array([0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xBF80, 0x3DCD,
                     0x0080, 0x0001, 0x0000, 0x0002, 0x8000], dtype=np.uint16)
    assert O.f64_to_bf16_bits(x).tolist() == want.tolist()


def test_bf16_encode_matches_torch_on_float32_inputs():
    x = rng(0).standard_normal(20000).astype(np.float32) * np.float32(7.0)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.f64_to_bf16_bits(x.astype(np.float64)), want)
    # and the round trip is the identity on bf16 values
    assert np.array_equal(O.f64_to_bf16_bits(O.bf16_bits_to_f64(want)), want)


def test_workload_codec_agrees_with_oracle_codec():
    x = rng(1).standard_normal(5000).astype(np.float32)
    assert np.array_equal(W.to_bf16_bits(x), O.f64_to_bf16_bits(x.astype(np.float64)))


# ------------------------------------------------------------------ attention (App. C.1 Step 1)
def test_attention_golden_three_keys(golden):
    g = golden("attention_three_keys.txt")
    q = np.array([g["q"]])
    k = np.array([g["k1"], g["k2"], g["k3"]])
    a = O.attention(q, k)
    assert np.allclose(a[0], g["alpha"], rtol=0, atol=1e-15)


def test_attention_two_keys_is_logistic():
    # L = 2: alpha_1 = 1/(1+exp(-(s1-s2))), with s = q.k/sqrt(d)
    r = rng(2)
    for d in (2, 8, 128):
        q = r.standard_normal((5, d))
        k = r.standard_normal((2, d))
        a = O.attention(q, k)
        s = (q @ k.T) / math.sqrt(d)
        want = 1.0 / (1.0 + np.exp(-(s[:, 0] - s[:, 1])))
        assert np.allclose(a[:, 0], want, rtol=1e-13)
        assert np.allclose(a[:, 1], 1 - want, rtol=1e-12, atol=1e-15)


def test_attention_rows_sum_to_one_and_nonnegative():
    r = rng(3)
    a = O.attention(r.standard_normal((17, 32)) * 3, r.standard_normal((301, 32)) * 3)
    assert (a >= 0).all()
    assert np.allclose(a.sum(axis=1), 1.0, rtol=0, atol=1e-13)


def test_attention_matches_scipy_softmax():
    r = rng(4)
    q, k = r.standard_normal((9, 64)), r.standard_normal((200, 64))
    want = scipy.special.softmax((q @ k.T) / 8.0, axis=1)
    assert np.allclose(O.attention(q, k), want, rtol=1e-12, atol=1e-300)


def test_attention_explicit_scale_and_large_logits():
    # shift invariance keeps huge logits finite; a custom scale is honoured
    q = np.array([[1000.0, 0.0]])
    k = np.array([[1.0, 0.0], [0.0, 1.0], [0.5, 0.0]])
    a = O.attention(q, k, scale=1.0)
    assert np.isfinite(a).all() and abs(a[0, 0] - 1.0) < 1e-200 + 1e-15
    a2 = O.attention(np.array([[2.0, 0.0]]), k, scale=0.5)       # logits (1, 0, .5)
    z = math.e + 1 + math.exp(0.5)
    assert np.allclose(a2[0], [math.e / z, 1 / z, math.exp(0.5) / z], rtol=1e-14)


def test_theorem_bounds_hold_and_are_nearly_tight():
    # App. C.1 ineq. (5): ||alpha - alpha'||_1 <= Kmax sqrt(2(1-sim)) / sqrt(d) for unit q, q'
    r = rng(5)
    d = 16
    for _ in range(50):
        q = r.standard_normal(d); q /= np.linalg.norm(q)
        q2 = q + 0.3 * r.standard_normal(d); q2 /= np.linalg.norm(q2)
        k = r.standard_normal((40, d)) * 2
        a, a2 = O.attention(q[None], k)[0], O.attention(q2[None], k)[0]
        bound = np.linalg.norm(k, axis=1).max() * math.sqrt(2 * (1 - q @ q2)) / math.sqrt(d)
        assert np.abs(a - a2).sum() <= bound
        assert 1 - 0.5 * np.abs(a - a2).sum() >= 1 - bound / 2            # ineq. (6)
    # two opposite keys along q - q' make the bound tight to first order; a missing or squared
    # 1/sqrt(d) factor in the oracle would land far outside [0.98, 1] x bound
    q = np.zeros(d); q[0] = 1.0
    q2 = np.zeros(d); q2[0], q2[1] = math.cos(0.02), math.sin(0.02)
    u = (q - q2) / np.linalg.norm(q - q2)
    k = np.stack([u, -u]) * 1.5
    a, a2 = O.attention(q[None], k)[0], O.attention(q2[None], k)[0]
    bound = 1.5 * math.sqrt(2 * (1 - q @ q2)) / math.sqrt(d)
    ratio = np.abs(a - a2).sum() / bound
    assert 0.98 < ratio <= 1.0


# ------------------------------------------------------------------ S(j) (Sec. 4.2)
def test_score_golden_two_heads(golden):
    g = golden("score_two_heads.txt")
    k = np.array(g["keys"])[:, None]
    q = np.array([g["head0"], g["head1"]])[:, :, None]           # [g=2, N=2, d=1]
    S = O.score_head(q, k)
    assert np.allclose(S, g["S"], rtol=1e-14)


def test_score_sums_to_N_times_group():
    r = rng(6)
    for g_, N, L, d in ((1, 1, 5, 8), (4, 8, 333, 32), (8, 3, 64, 128)):
        S = O.score_head(r.standard_normal((g_, N, d)), r.standard_normal((L, d)))
        assert abs(S.sum() - g_ * N) < 1e-11 * g_ * N
        assert (S > 0).all()


def test_score_identical_keys_uniform():
    r = rng(7)
    k = np.tile(r.standard_normal((1, 16)), (37, 1))
    S = O.score_head(r.standard_normal((2, 5, 16)), k)
    assert np.allclose(S, 2 * 5 / 37, rtol=1e-13)


def test_score_dominant_key_takes_everything():
    d = 8
    q = np.ones((2, 3, d))
    k = np.zeros((10, d)); k[4] = 50.0
    S = O.score_head(q, k)
    assert abs(S[4] - 6.0) < 1e-12 and S.sum() - S[4] < 1e-12


def test_score_permutation_equivariance_and_head_duplication():
    r = rng(8)
    q, k = r.standard_normal((2, 4, 16)), r.standard_normal((50, 16))
    perm = r.permutation(50)
    assert np.allclose(O.score_head(q, k[perm]), O.score_head(q, k)[perm], rtol=1e-13)
    q_dup = np.concatenate([q, q[:1]], axis=0)                    # head 0 counted twice
    want = O.score_head(q, k) + O.score_head(q[:1], k)
    assert np.allclose(O.score_head(q_dup, k), want, rtol=1e-13)


def test_score_matches_torch_float64():
    r = rng(9)
    q, k = r.standard_normal((4, 6, 128)), r.standard_normal((257, 128))
    tq, tk = torch.from_numpy(q.reshape(24, 128)), torch.from_numpy(k)
    want = torch.softmax(tq @ tk.T / math.sqrt(128), dim=-1).sum(0).numpy()
    assert np.allclose(O.score_head(q, k), want, rtol=1e-12)


def test_score_batch_layout_group_mapping_and_ragged():
    # query head h scores against KV head h // g; sequences are scored separately
    r = rng(10)
    Hq, Hkv, N, d = 4, 2, 3, 16
    lens = [5, 1, 9]
    cu = np.concatenate([[0], np.cumsum(lens)])
    qb = W.to_bf16_bits(r.standard_normal((2, 3, Hq, N, d)))
    kb = W.to_bf16_bits(r.standard_normal((2, cu[-1], Hkv, d)))
    S = O.score(qb, kb, Hkv, cu)
    q, k = O.bf16_bits_to_f64(qb), O.bf16_bits_to_f64(kb)
    for l in range(2):
        for b in range(3):
            for kv in range(Hkv):
                logits = np.einsum("hnd,jd->hnj", q[l, b, 2 * kv:2 * kv + 2], k[l, cu[b]:cu[b + 1], kv]) / 4.0
                want = scipy.special.softmax(logits, axis=2).sum(axis=(0, 1))
                assert np.allclose(S[l, kv, cu[b]:cu[b + 1]], want, rtol=1e-12)
    assert np.allclose(S[:, :, cu[1]:cu[2]], Hq // Hkv * N)       # length-1 sequence: all mass on its key
    # dense form: cu_seqlens None means equal lengths
    S_dense = O.score(qb[:, :1], kb[:, :5], Hkv, None)
    assert np.allclose(S_dense, S[:, :, :5], rtol=1e-14)


# ------------------------------------------------------------------ RoPE (Sec. 4.1)
def test_rope_closed_form_pairs():
    d, theta = 4, 10000.0                       # omega = (1, 0.01)
    x = np.array([[[1.0, 0.0, 0.0, 1.0]]])      # half pairing: (x0,x2)=(1,0), (x1,x3)=(0,1)
    y = O.rope_rotate(x, [3], theta, "half")[0, 0]
    want = [math.cos(3.0), -math.sin(0.03), math.sin(3.0), math.cos(0.03)]
    assert np.allclose(y, want, rtol=1e-15, atol=1e-17)
    yi = O.rope_rotate(x, [3], theta, "interleaved")[0, 0]   # pairs (x0,x1)=(1,0), (x2,x3)=(0,1)
    want_i = [math.cos(3.0), math.sin(3.0), -math.sin(0.03), math.cos(0.03)]
    assert np.allclose(yi, want_i, rtol=1e-15, atol=1e-17)


def test_rope_frequency_ladder():
    # channel pair c turns by pos * theta**(-2c/d): read the angle back from a unit vector
    d, theta, pos = 128, 500000.0, 7
    x = np.zeros((1, 1, d)); x[0, 0, :d // 2] = 1.0
    y = O.rope_rotate(x, [pos], theta)[0, 0]
    ang = np.arctan2(y[d // 2:], y[:d // 2])
    want = pos * theta ** (-np.arange(d // 2) / (d / 2))
    assert np.allclose(np.angle(np.exp(1j * want)), ang, rtol=1e-12, atol=1e-14)


def test_rope_identity_norm_and_bf16_rounding():
    r = rng(11)
    xb = W.to_bf16_bits(r.standard_normal((6, 3, 128)))
    assert np.array_equal(O.rope_apply(xb, np.zeros(6, dtype=np.int64)), xb)      # position 0
    x = O.bf16_bits_to_f64(xb)
    pos = np.array([1, 17, 1024, 32768, 131071, 5])
    y = O.rope_rotate(x, pos)
    h = 64
    assert np.allclose(x[..., :h] ** 2 + x[..., h:] ** 2, y[..., :h] ** 2 + y[..., h:] ** 2, rtol=1e-13)
    yb = O.bf16_bits_to_f64(O.rope_apply(xb, pos))
    assert (np.abs(yb - y) <= np.abs(y) * 2.0 ** -8 + 1e-40).all()                # one rounding to bf16


def test_rope_scores_depend_only_on_relative_offset():
    r = rng(12)
    N, L, d, g_ = 4, 40, 128, 2
    q = r.standard_normal((N, g_, d))
    k = r.standard_normal((L, 1, d))

    def S(shift, q_start=L):
        qr = O.rope_rotate(q, np.arange(q_start, q_start + N) + shift)
        kr = O.rope_rotate(k, np.arange(L) + shift)
        return O.score_head(qr.transpose(1, 0, 2), kr[:, 0])

    base = S(0)
    assert np.allclose(S(1000), base, rtol=1e-9)
    assert np.allclose(S(100000), base, rtol=1e-7)
    # pseudo queries placed at 0..N-1 instead of L_p.. give a different importance profile
    # (Sec. 3.1, Table 1: same content at the wrong position is a poor stand-in)
    assert np.abs(S(0, q_start=0) - base).max() > 1e-3


# ------------------------------------------------------------------ pooling
def test_pool_golden_and_topk_golden(golden):
    g = golden("pool_topk_example.txt")
    P = O.pool(np.array(g["S"]), 7)
    assert P.tolist() == g["P"]
    assert O.topk(P, 4).tolist() == g["top4"]
    assert O.topk(P, 8).tolist() == g["top8"]
    assert O.topk(P, 11).tolist() == g["top11"]


def test_pool_matches_scipy_maximum_filter_and_properties():
    r = rng(13)
    for L in (1, 2, 3, 6, 7, 8, 100):
        S = r.random(L)
        for width in (1, 3, 7):
            P = O.pool(S, width)
            want = scipy.ndimage.maximum_filter1d(S, size=width, mode="constant", cval=-np.inf)
            assert np.array_equal(P, want)
            assert (P >= S).all()
        assert np.array_equal(O.pool(S, 1), S)
    assert np.array_equal(O.pool(np.full(20, 0.25), 7), np.full(20, 0.25))


# ------------------------------------------------------------------ TopK (Sec. 4.2)
def test_topk_brute_force_and_ties():
    r = rng(14)
    for L, Kb in ((1, 1), (10, 3), (50, 50), (50, 70), (200, 17)):
        P = r.integers(0, 6, size=L).astype(np.float64)          # many ties
        got = O.topk(P, Kb)
        n = min(Kb, L)
        want = np.sort(np.argsort(-P, kind="stable")[:n])        # stable sort: ties keep index order
        assert got.tolist() == want.tolist()
        assert len(set(got.tolist())) == n and (np.diff(got) > 0).all()
        dropped = np.setdiff1d(np.arange(L), got)
        if dropped.size and n:
            assert P[got].min() >= P[dropped].max()
    assert O.topk(np.full(9, 0.5), 4).tolist() == [0, 1, 2, 3]
    assert O.topk(np.array([3.0, 1.0, 2.0]), 0).tolist() == []


def test_topk_margin_uses_distinct_values():
    P = np.array([5.0, 5.0, 5.0, 4.0, 1.0])
    v, gap = O.topk_margin(P, 2)                 # boundary inside the plateau of 5s
    assert v == 5.0 and abs(gap - 0.2) < 1e-15
    v, gap = O.topk_margin(P, 4)
    assert v == 4.0 and abs(gap - 0.25) < 1e-15
    assert O.topk_margin(P, 5)[1] == np.inf
    # the nearest distinct value on each side counts, not the farthest: 5.001 sits 2e-4 above the boundary 5
    v, gap = O.topk_margin(np.array([10.0, 5.001, 5.0, 1.0]), 3)
    assert v == 5.0 and abs(gap - 0.001 / 5.0) < 1e-12
    v, gap = O.topk_margin(np.array([10.0, 5.0, 4.999, 1.0]), 2)
    assert v == 5.0 and abs(gap - 0.001 / 5.0) < 1e-12


# ------------------------------------------------------------------ gather / whole step
def test_gather_is_a_bit_copy():
    r = rng(15)
    bits = r.integers(0, 65536, size=(30, 8), dtype=np.uint16)
    idx = np.array([0, 3, 29])
    out = O.gather(bits, idx)
    assert out.dtype == np.uint16 and np.array_equal(out, bits[[0, 3, 29]])
    out[0, 0] ^= 1
    assert bits[0, 0] != out[0, 0]               # a copy, not a view


def test_compress_ragged_batch_is_per_sequence_and_clipped():
    r = rng(16)
    Hq, Hkv, N, d = 4, 2, 4, 32
    lens = [20, 3, 11]
    cu = np.concatenate([[0], np.cumsum(lens)])
    qb = W.to_bf16_bits(r.standard_normal((1, 3, Hq, N, d)))
    kb = W.to_bf16_bits(r.standard_normal((1, cu[-1], Hkv, d)))
    # a huge key at the very end of sequence 0 must not leak into sequence 1 through the pool window
    kb[0, cu[1] - 1, 0] = W.to_bf16_bits(8.0 * O.bf16_bits_to_f64(qb[0, 0, 0, 0]))
    vb = r.integers(0, 65536, size=kb.shape, dtype=np.uint16)
    out = O.compress(qb, kb, vb, Hkv, [5, 5, 100], cu)
    for b, L in enumerate(lens):
        solo = O.compress(qb[:, b:b + 1], kb[:, cu[b]:cu[b + 1]], vb[:, cu[b]:cu[b + 1]], Hkv,
                          [5, 5, 100][b], None)
        n = min([5, 5, 100][b], L)
        assert (out["count"][0, b] == n).all() and (solo["count"] == n).all()
        assert np.array_equal(out["idx"][0, b, :, :n], solo["idx"][0, 0, :, :n])
        assert np.array_equal(out["k_out"][0, b, :, :n], solo["k_out"][0, 0, :, :n])
        assert np.array_equal(out["v_out"][0, b, :, :n], solo["v_out"][0, 0, :, :n])
        assert np.allclose(out["P"][0, :, cu[b]:cu[b + 1]], solo["P"][0], rtol=1e-14)
        for kv in range(Hkv):
            keep = out["idx"][0, b, kv, :n]
            assert np.array_equal(out["k_out"][0, b, kv, :n], kb[0, cu[b]:cu[b + 1], kv][keep])
            assert np.array_equal(out["v_out"][0, b, kv, :n], vb[0, cu[b]:cu[b + 1], kv][keep])
            assert keep.min() >= 0 and keep.max() < L
    assert out["S"][0, 0, cu[1] - 1] > 3.0
    assert out["P"][0, 0, cu[1]] < out["S"][0, 0, cu[1] - 1]
    assert (out["idx"][0, 1, :, 3:] == -1).all()                 # budget 5 > L = 3: three rows kept


def test_planted_needles_survive_eviction_small_workload():
    # synthetic stand-in for the needle-retrieval result of Sec. 5.2: keys aligned with a pseudo
    # query before rotation stay in M_retain at a ~12 % budget
    w = W.workload("C1")
    for seed in (0, 1):
        p = W.host_problem(w, seed)
        q = np.stack([O.rope_apply(p["q"][0, 0].transpose(1, 0, 2), p["q_pos"][0], w.theta).transpose(1, 0, 2)])[None]
        k = O.rope_apply(p["k"][0], p["k_pos"], w.theta)[None]
        out = O.compress(q, k, p["v"], w.n_kv_heads, w.budget, None, w.pool_width)
        for kv in range(w.n_kv_heads):
            pos, _, _ = W.needle_plan(w, seed, 0, 0, kv, w.seq_len)
            assert set(pos.tolist()) <= set(out["idx"][0, 0, kv].tolist())
            assert abs(out["S"][0, kv].sum() - w.group * w.n_pseudo) < 1e-9
        assert (out["count"] == w.budget).all()


def test_recall_definition():
    assert O.recall([1, 2, 3, 4], [2, 4, 9]) == 0.5
    assert O.recall([5], [5]) == 1.0 and O.recall([5, 6], [7]) == 0.0


def test_compress_selects_on_the_pooled_scores():
    # one query, keys on a line: key 5 dominates, keys 0 and 10 come next, the rest are equal and small.  On the raw
    # scores the three best are {0, 5, 10}; pooled with a window of 3 the neighbours of key 5 inherit its score and
    # the three best are {4, 5, 6} (Sec. 1 / Sec. 5.1: selection runs on the pooled accumulated scores)
    L, d = 12, 2
    k = np.zeros((1, L, 1, d))
    k[0, 5, 0, 0], k[0, 0, 0, 0], k[0, 10, 0, 0] = 8.0, 4.0, 4.0
    q = np.zeros((1, 1, 1, 1, d))
    q[0, 0, 0, 0, 0] = 1.0
    qb, kb = W.to_bf16_bits(q), W.to_bf16_bits(k)
    vb = np.arange(L * d, dtype=np.uint16).reshape(1, L, 1, d)
    raw = O.compress(qb, kb, vb, 1, 3, width=1)
    assert raw["idx"][0, 0, 0].tolist() == [0, 5, 10]
    pooled = O.compress(qb, kb, vb, 1, 3, width=3)
    assert pooled["idx"][0, 0, 0].tolist() == [4, 5, 6]
    assert pooled["P"][0, 0, 4] == pooled["S"][0, 0, 5] == pooled["P"][0, 0, 6]
    assert pooled["v_out"][0, 0, 0].tolist() == [[8, 9], [10, 11], [12, 13]]      # rows 4, 5, 6 of V, bit for bit
    assert pooled["count"][0, 0, 0] == 3


# ------------------------------------------------------------------ extended sequence (Sec. 4.1): pseudo keys in the normaliser
def test_extended_attention_golden_two_pseudo(golden):
    g = golden("attention_extended_two_pseudo.txt")
    q = np.array([g["q"], g["q"]])
    k = np.array([g["k1"], g["k2"], g["k3"]])
    kp = np.array([g["kp0"], g["kp1"]])
    a = O.attention_extended(q, k, kp)
    assert np.allclose(a[0], g["alpha0"], rtol=0, atol=1e-15)
    assert np.allclose(a[1], g["alpha1"], rtol=0, atol=1e-15)
    S = O.score_head(q[None], k, None, kp)
    assert np.allclose(S, g["S"], rtol=0, atol=1e-15)


def test_extended_attention_identical_keys_is_harmonic():
    # every key, prompt or pseudo, equal: query i spreads evenly over its L + i + 1 visible keys,
    # so S(j) = g * sum_i 1/(L + i + 1); a mask that hid the wrong side would give 1/(L + N - i)
    L, N, g, d = 9, 5, 3, 8
    key = rng(70).standard_normal(d)
    q = rng(71).standard_normal((g, N, d))
    S = O.score_head(q, np.tile(key, (L, 1)), None, np.tile(key, (N, 1)))
    want = g * sum(1.0 / (L + i + 1) for i in range(N))
    assert np.allclose(S, want, rtol=1e-13)
    a = O.attention_extended(q[0], np.tile(key, (L, 1)), np.tile(key, (N, 1)))
    assert np.allclose(a[0, :L + 1], 1.0 / (L + 1)) and np.all(a[0, L + 1:] == 0)


def test_extended_attention_matches_torch_masked_softmax_and_conserves_mass():
    L, N, d = 37, 11, 16
    r = rng(72)
    q, k, kp = r.standard_normal((N, d)), r.standard_normal((L, d)), r.standard_normal((N, d))
    a = O.attention_extended(q, k, kp)
    logits = torch.from_numpy(np.concatenate([k, kp]) @ q.T).T / math.sqrt(d)         # [N, L+N]
    visible = torch.cat([torch.ones(N, L, dtype=torch.bool), torch.tril(torch.ones(N, N, dtype=torch.bool))], dim=1)
    want = torch.softmax(logits.masked_fill(~visible, float("-inf")), dim=1).numpy()
    assert np.allclose(a, want, rtol=1e-12, atol=1e-16)
    assert np.allclose(a.sum(axis=1), 1.0, rtol=1e-13)
    # S over the prompt keys + the mass that went to the pseudo keys = N
    S = O.score_head(q[None], k, None, kp)
    assert np.isclose(S.sum() + want[:, L:].sum(), N, rtol=1e-12)


def test_extended_attention_brute_force_and_causality():
    L, N, d, scale = 6, 4, 5, 0.3
    r = rng(73)
    q, k, kp = r.standard_normal((N, d)), r.standard_normal((L, d)), r.standard_normal((N, d))
    a = O.attention_extended(q, k, kp, scale)
    for i in range(N):
        w = [math.exp(scale * sum(q[i, c] * k[j, c] for c in range(d))) for j in range(L)]
        w += [math.exp(scale * sum(q[i, c] * kp[t, c] for c in range(d))) for t in range(i + 1)]
        tot = sum(w)
        for j, x in enumerate(w):
            assert math.isclose(a[i, j], x / tot, rel_tol=1e-12)
        assert np.all(a[i, L + i + 1:] == 0)
    # a later pseudo key cannot change an earlier query's weights
    kp2 = kp.copy()
    kp2[N - 1] += 5.0
    a2 = O.attention_extended(q, k, kp2, scale)
    assert np.array_equal(a2[:N - 1], a[:N - 1]) and not np.allclose(a2[N - 1], a[N - 1])


def test_extended_score_reduces_to_prompt_only_when_pseudo_keys_are_far():
    # pseudo keys opposite to every query: their weight vanishes and S equals the prompt-only score
    L, N, g, d = 50, 8, 2, 16
    r = rng(74)
    q = np.abs(r.standard_normal((g, N, d))) + 0.5
    k = r.standard_normal((L, d))
    kp = -200.0 * np.ones((N, d))
    assert np.allclose(O.score_head(q, k, None, kp), O.score_head(q, k), rtol=1e-12)
    # and never exceeds it: the extra keys only take mass away
    kp = r.standard_normal((N, d))
    assert np.all(O.score_head(q, k, None, kp) < O.score_head(q, k))


def test_extended_score_batch_layout():
    layers, B, Hq, Hkv, N, d = 2, 2, 4, 2, 3, 8
    lens = [5, 9]
    r = rng(75)
    qb = W.to_bf16_bits(r.standard_normal((layers, B, Hq, N, d)))
    kb = W.to_bf16_bits(r.standard_normal((layers, sum(lens), Hkv, d)))
    kpb = W.to_bf16_bits(r.standard_normal((layers, B, Hkv, N, d)))
    cu = np.array([0, 5, 14])
    S = O.score(qb, kb, Hkv, cu, None, kpb)
    l, b, kv = 1, 1, 1
    want = O.score_head(O.bf16_bits_to_f64(qb[l, b, 2:4]), O.bf16_bits_to_f64(kb[l, 5:14, kv]), None,
                        O.bf16_bits_to_f64(kpb[l, b, kv]))
    assert np.array_equal(S[l, kv, 5:14], want)


# ------------------------------------------------------------------ decode step over a cache (Sec. 4.2, last paragraph)
def test_decode_attention_closed_forms():
    r = rng(80)
    d = 8
    q = r.standard_normal((3, d))
    v = r.standard_normal((5, d))
    # one key: the output is its value, whatever the logit
    assert np.allclose(O.decode_attention(q, r.standard_normal((1, d)), v[:1]), np.tile(v[0], (3, 1)), rtol=1e-14)
    # identical keys: uniform weights, the output is the mean value
    key = r.standard_normal(d)
    assert np.allclose(O.decode_attention(q, np.tile(key, (5, 1)), v), np.tile(v.mean(axis=0), (3, 1)), rtol=1e-13)
    # two keys: logistic weight on the first (App. C.1 with d_k = 8)
    k2 = r.standard_normal((2, d))
    w = 1.0 / (1.0 + np.exp(-(q @ (k2[0] - k2[1])) / math.sqrt(d)))
    want = w[:, None] * v[0] + (1 - w)[:, None] * v[1]
    assert np.allclose(O.decode_attention(q, k2, v[:2]), want, rtol=1e-13)


def test_decode_attention_matches_torch_sdpa():
    r = rng(81)
    q, k, v = r.standard_normal((4, 16)), r.standard_normal((50, 16)), r.standard_normal((50, 16))
    want = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(k)[None],
                                                            torch.from_numpy(v)[None])[0].numpy()
    assert np.allclose(O.decode_attention(q, k, v), want, rtol=1e-12, atol=1e-15)
    # every output channel is a convex combination of that channel's values
    o = O.decode_attention(q, k, v)
    assert np.all(o <= v.max(axis=0) + 1e-12) and np.all(o >= v.min(axis=0) - 1e-12)


def test_decode_over_compact_cache_is_within_the_dropped_mass_bound():
    # dropping keys that hold attention mass m moves the output by at most 2 m max|v|:
    # o_full = sum_kept a_j v_j + sum_drop a_j v_j and o_compact = sum_kept a_j v_j / (1 - m)
    r = rng(82)
    L, d, Kb = 400, 16, 60
    q = r.standard_normal((1, d)) * 3.0
    k, v = r.standard_normal((L, d)), r.standard_normal((L, d))
    alpha = O.attention(q, k)[0]
    keep = O.topk(alpha, Kb)
    m = 1.0 - alpha[keep].sum()
    diff = np.abs(O.decode_attention(q, k[keep], v[keep]) - O.decode_attention(q, k, v)).max()
    assert 0 < m < 1 and diff <= 2 * m * np.abs(v).max()
    # and keeping the keys with the LEAST mass is far worse than keeping those with the most
    worst = np.argsort(alpha, kind="stable")[:Kb]
    diff_worst = np.abs(O.decode_attention(q, k[worst], v[worst]) - O.decode_attention(q, k, v)).max()
    assert diff_worst > 3 * diff


# ------------------------------------------------------------------ pseudo tokens (Sec. 4.1 positions, Sec. 5.1 Fm_Ln content)
def test_pseudo_tokens_first_m_last_n_and_positions():
    # the paper's own example shapes: first 4 + last 28, first 2 + last 30 (Sec. 5.1)
    src, pos = O.pseudo_tokens(1000, 4, 28)
    assert src.tolist() == [0, 1, 2, 3] + list(range(972, 1000))
    assert pos.tolist() == list(range(1000, 1032))                  # Positions(T_pseudo) = [L_p, ..., L_p+N-1]
    src, pos = O.pseudo_tokens(50, 2, 30)
    assert src.tolist() == [0, 1] + list(range(20, 50)) and pos[0] == 50 and pos[-1] == 81
    # short prompts repeat their ends, an empty one has no source
    assert O.pseudo_tokens(3, 4, 5)[0].tolist() == [0, 1, 2, 2, 0, 0, 0, 1, 2]
    assert O.pseudo_tokens(0, 1, 2)[0].tolist() == [-1, -1, -1] and O.pseudo_tokens(0, 1, 2)[1].tolist() == [0, 1, 2]


# ------------------------------------------------------------------ queries of the pseudo tokens (Sec. 4.1)
def _bits(x):
    return W.to_bf16_bits(np.asarray(x, dtype=np.float64))


def test_pseudo_queries_golden_two_heads(golden):
    g = golden("pseudo_queries_two_heads.txt")
    x = _bits([g["x0"], g["x1"], g["x2"]])
    w = _bits([g["w0"], g["w1"], g["w2"], g["w3"]])
    tok = [int(v) for v in g["token_idx"]]
    pre = O.bf16_bits_to_f64(O.pseudo_queries(x, tok, w, 2))
    assert pre[0].ravel().tolist() == g["q_pre_head0"] and pre[1].ravel().tolist() == g["q_pre_head1"]
    q = O.bf16_bits_to_f64(O.pseudo_queries(x, tok, w, 2, positions=[int(v) for v in g["positions"]], theta=10000.0))
    assert q[0].ravel().tolist() == g["q_head0"] and q[1].ravel().tolist() == g["q_head1"]


def test_pseudo_queries_golden_rounding_order(golden):
    g = golden("pseudo_queries_rounding_order.txt")
    x, w = _bits([g["x0"]]), _bits([g["w0"], g["w1"]])
    tok = [int(v) for v in g["token_idx"]]
    assert O.bf16_bits_to_f64(O.pseudo_queries(x, tok, w, 1))[0, 0].tolist() == g["q_pre"]
    q = O.bf16_bits_to_f64(O.pseudo_queries(x, tok, w, 1, positions=[int(v) for v in g["positions"]]))
    assert q[0, 0].tolist() == g["q"]


def test_pseudo_queries_permutation_weight_is_a_gather():
    # w = rows of a permutation matrix: feature f copies hidden channel perm[f], bit for bit; using w
    # transposed would apply the inverse permutation instead
    r = rng(90)
    tokens, hidden, Hq, rows = 11, 24, 3, 7
    x = W.to_bf16_bits(r.standard_normal((tokens, hidden)))
    perm = r.permutation(hidden)
    assert not np.array_equal(np.argsort(perm), perm)
    w = np.zeros((hidden, hidden))
    w[np.arange(hidden), perm] = 1.0
    tok = r.integers(0, tokens, rows)
    got = O.pseudo_queries(x, tok, _bits(w), Hq)
    want = x[tok][:, perm].reshape(rows, Hq, hidden // Hq).transpose(1, 0, 2)
    assert np.array_equal(got, want)


def test_pseudo_queries_brute_force_exact_sums():
    # every product of two bf16 numbers and every partial sum here is exact in rational arithmetic;
    # the result must be the bf16 nearest to the exact sum
    from fractions import Fraction
    r = rng(91)
    tokens, hidden, Hq, d, rows = 5, 9, 2, 4, 6
    x = W.to_bf16_bits(r.standard_normal((tokens, hidden)))
    w = W.to_bf16_bits(r.standard_normal((Hq * d, hidden)))
    tok = [4, 0, 0, -1, 2, 3]
    got = O.bf16_bits_to_f64(O.pseudo_queries(x, tok, w, Hq))
    xf, wf = W.from_bf16_bits(x).astype(np.float64), W.from_bf16_bits(w).astype(np.float64)
    for row in range(rows):
        for h in range(Hq):
            for c in range(d):
                exact = Fraction(0)
                if tok[row] >= 0:
                    for t in range(hidden):
                        exact += Fraction(float(xf[tok[row], t])) * Fraction(float(wf[h * d + c, t]))
                if exact == 0:
                    assert got[h, row, c] == 0.0
                    continue
                e = math.frexp(float(abs(exact)))[1]          # |exact| in [2^(e-1), 2^e)
                ulp = Fraction(2) ** (e - 8)                  # spacing of bf16 there (8 significant bits)
                k = abs(exact) / ulp
                lo = k.numerator // k.denominator
                rem = k - lo
                n = lo + 1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1) else lo
                want = float(n * ulp) * (1 if exact > 0 else -1)
                assert got[h, row, c] == want, (row, h, c)


def test_pseudo_queries_round_once_from_the_exact_sum():
    # 1 + 2^-8 is halfway between two bf16 numbers; the 2^-30 on top decides it upwards.  Rounding the
    # sum to float32 first would lose the 2^-30 and then fall to the even neighbour 1.0.
    x = _bits([[1.0, 2.0 ** -8, 2.0 ** -30]])
    w = _bits([[1.0, 1.0, 1.0], [1.0, 1.0, 0.0]])
    got = O.bf16_bits_to_f64(O.pseudo_queries(x, [0], w, 1))
    assert got[0, 0].tolist() == [1.0 + 2.0 ** -7, 1.0]


def test_pseudo_queries_positions_and_layout():
    r = rng(92)
    tokens, hidden, Hq, d, rows = 13, 16, 4, 8, 5
    x = W.to_bf16_bits(r.standard_normal((tokens, hidden)))
    w = W.to_bf16_bits(r.standard_normal((Hq * d, hidden)) / 4.0)
    tok = r.integers(0, tokens, rows)
    pre = O.pseudo_queries(x, tok, w, Hq)
    assert pre.shape == (Hq, rows, d) and pre.dtype == np.uint16
    # position 0 is no rotation; rows that copy the same token differ only by their positions
    assert np.array_equal(O.pseudo_queries(x, tok, w, Hq, positions=np.zeros(rows, dtype=np.int64)), pre)
    same = O.pseudo_queries(x, [3, 3], w, Hq, positions=[100, 101])
    assert not np.array_equal(same[:, 0], same[:, 1])
    assert np.array_equal(O.pseudo_queries(x, [3, 3], w, Hq)[:, 0], O.pseudo_queries(x, [3, 3], w, Hq)[:, 1])
    # the rotation is the one rope_apply does on the rounded projection, per head, and keeps each pair's norm
    pos = np.array([7, 1000, 32768, 5, 131071])
    q = O.bf16_bits_to_f64(O.pseudo_queries(x, tok, w, Hq, positions=pos))
    p = O.bf16_bits_to_f64(pre)
    n_q = np.hypot(q[..., : d // 2], q[..., d // 2:])
    n_p = np.hypot(p[..., : d // 2], p[..., d // 2:])
    assert np.allclose(n_q, n_p, rtol=2.0 ** -7, atol=1e-3)
    # torch's float64 matmul, rounded by torch, agrees on the projection
    xt = torch.from_numpy(W.from_bf16_bits(x).astype(np.float64))
    wt = torch.from_numpy(W.from_bf16_bits(w).astype(np.float64))
    want = (xt[torch.from_numpy(tok)] @ wt.T).to(torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    agree = (want.reshape(rows, Hq, d).transpose(1, 0, 2) == pre).mean()
    assert agree > 0.99          # float32 in between may flip a halfway case, nothing else
