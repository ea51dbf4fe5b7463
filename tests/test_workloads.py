"""The seeded input generator: determinism, shapes, needle and heavy-hitter structure."""
import numpy as np

import workloads as W


def test_slices_are_deterministic_and_independent():
    w = W.workload("C1")
    a = W.k_pre(w, 3, 0, 0, 5, 1024)
    b = W.k_pre(w, 3, 0, 0, 5, 1024)
    assert a.dtype == np.uint16 and a.shape == (1024, 128) and np.array_equal(a, b)
    assert not np.array_equal(a, W.k_pre(w, 4, 0, 0, 5, 1024))
    assert not np.array_equal(a, W.k_pre(w, 3, 0, 0, 6, 1024))
    p = W.host_problem(w, 3)
    assert np.array_equal(p["k"][0, :, 5], a)
    assert p["q"].shape == (1, 1, 32, 64, 128) and p["q_pos"].tolist() == [list(range(1024, 1088))]
    assert p["k_pos"].tolist() == list(range(1024))


def test_values_are_standard_normal_bf16():
    w = W.workload("C2")
    x = W.from_bf16_bits(W.v_rows(w, 0, 1, 0, 2, 8192)).astype(np.float64)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert np.array_equal(W.to_bf16_bits(W.from_bf16_bits(W.v_rows(w, 0, 1, 0, 2, 64))),
                          W.v_rows(w, 0, 1, 0, 2, 64))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1 + 2 ** -8, 1 + 3 * 2 ** -8, 1 + 2 ** -8 + 2 ** -20], dtype=np.float32)
    assert W.to_bf16_bits(x).tolist() == [0x3F80, 0x3F80, 0x3F82, 0x3F81]


def test_needles_are_stratified_and_copy_a_group_query():
    w = W.workload("C2")
    L = w.seq_len
    q = W.q_pre(w, 7, 2, 0)
    k = W.k_pre(w, 7, 2, 0, 3, L, q)
    pos, qh, qr = W.needle_plan(w, 7, 2, 0, 3, L)
    assert len(pos) == 16 and len(set(pos.tolist())) == 16
    assert ((pos // (L // 16)) == np.arange(16)).all()                  # one per stratum
    assert ((qh // w.group) == 3).all() and (qr < w.n_pseudo).all()
    want = 3.0 * W.from_bf16_bits(q[qh, qr]).astype(np.float64)
    got = W.from_bf16_bits(k[pos]).astype(np.float64)
    assert np.allclose(got, want, rtol=2.0 ** -8)


def test_ragged_lengths_and_heavy_tail():
    w = W.workload("C3")
    lens = W.seq_lens(w, 11)
    assert len(lens) == 8 and all(4096 <= v <= 16384 for v in lens) and lens == W.seq_lens(w, 11)
    cu = W.cu_seqlens(w, 11)
    assert cu[0] == 0 and (np.diff(cu) == lens).all()
    L = lens[0]
    k = W.from_bf16_bits(W.k_pre(w, 11, 0, 0, 0, L)).astype(np.float64)
    hm = W.heavy_mask(w, 11, 0, 0, 0, L)
    assert 0.08 < hm.mean() < 0.12
    n = np.linalg.norm(k, axis=1)
    assert abs(n[hm].mean() / n[~hm].mean() - 4.0) < 0.1
    assert W.workload("C4", 256).n_pseudo == 256 and W.workload("C5").group == 8
