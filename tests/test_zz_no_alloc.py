"""The entry point that allocates nothing (dapq_score_static): same scores as dapq_score, bit for bit, on two calls in
a row that share the library's built-in scratch array, the second with a smaller input; sizes beyond the array are
refused on the host."""
import numpy as np
import pytest
import torch

import paper_2603_11564_amd as D
import workloads as W
from dapq_harness import Problem, assert_scores_close
from oracle import dapq_oracle as O

pytestmark = pytest.mark.gpu


def make_problem(seed, layers, L, n_pseudo, Hq=8, Hkv=2):
    rng = np.random.default_rng(seed)
    q = O.f64_to_bf16_bits(rng.standard_normal((layers, 1, Hq, n_pseudo, 128)))
    k = O.f64_to_bf16_bits(rng.standard_normal((layers, L, Hkv, 128)))
    v = O.f64_to_bf16_bits(rng.standard_normal((layers, L, Hkv, 128)))
    return Problem(q, k, v, Hkv, None, "thd", 128 ** -0.5)


def new_scores(prob):
    return torch.full((prob.layers, prob.Hkv, prob.tokens), float("nan"), dtype=torch.float32, device=prob.device)


def test_static_scratch_matches_caller_workspace_twice_in_a_row():
    big = make_problem(11, layers=3, L=5000, n_pseudo=64)      # several chunks per head, a ragged tail
    small = make_problem(12, layers=1, L=333, n_pseudo=16)     # fewer layers, rows and keys: leaves stale scratch behind
    assert D.workspace_bytes(big.shape) <= D.score_static_capacity()
    ref_big, ref_small = big.score(), small.score()            # also loads the kernels before memory is measured
    S_big, S_small, S_again = new_scores(big), new_scores(small), new_scores(big)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    D.dapq_score_static(big.shape, big.q, big.k, S_big)
    D.dapq_score_static(small.shape, small.q, small.k, S_small)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before         # the calls took no device memory
    assert torch.equal(S_big, ref_big)
    assert torch.equal(S_small, ref_small)
    # and the scores are the oracle's (the bar of the other score tests)
    ref = O.score(small.q_bits, small.k_bits, small.Hkv, None, 128 ** -0.5)
    assert_scores_close(S_small.cpu().numpy(), ref, "static small")
    # a third call after the small one: the big problem again, over whatever the small one left behind
    D.dapq_score_static(big.shape, big.q, big.k, S_again)
    torch.cuda.synchronize()
    assert torch.equal(S_again, ref_big)


def test_static_scratch_serves_a_ragged_batch():
    """A ragged batch keeps a prefix of chunk counts and the ticket counter of its work list in the scratch array; both
    are rewritten by every call, so calls in a row (another batch in between) give the scores of dapq_score."""
    rng = np.random.default_rng(13)
    lens = [700, 0, 45, 1300]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q = O.f64_to_bf16_bits(rng.standard_normal((2, len(lens), 8, 32, 128)))
    k = O.f64_to_bf16_bits(rng.standard_normal((2, int(cu[-1]), 2, 128)))
    ragged = Problem(q, k, k, 2, cu, "thd", 128 ** -0.5)
    dense = make_problem(14, layers=1, L=900, n_pseudo=16)
    assert D.workspace_bytes(ragged.shape) <= D.score_static_capacity()
    ref_ragged, ref_dense = ragged.score(), dense.score()
    S1, S2, S3 = new_scores(ragged), new_scores(dense), new_scores(ragged)
    D.dapq_score_static(ragged.shape, ragged.q, ragged.k, S1)
    D.dapq_score_static(dense.shape, dense.q, dense.k, S2)
    D.dapq_score_static(ragged.shape, ragged.q, ragged.k, S3)
    torch.cuda.synchronize()
    assert torch.equal(S1, ref_ragged) and torch.equal(S2, ref_dense) and torch.equal(S3, ref_ragged)
    assert_scores_close(S1.cpu().numpy(), O.score(ragged.q_bits, ragged.k_bits, 2, cu, 128 ** -0.5), "static ragged")


def test_static_scratch_one_kernel_shape():
    """A shape whose two passes run in one kernel (no workspace is touched at all) between two that use the scratch
    array: the scores of the separate passes with a caller workspace, bit for bit."""
    one = make_problem(15, layers=2, L=400, n_pseudo=32)       # four chunks of a sequence = the waves of a workgroup
    other = make_problem(16, layers=1, L=2000, n_pseudo=16)
    assert D.score_single_launch(one.shape) and not D.score_single_launch(other.shape)
    ref_one, ref_other = one.score_split(), other.score()
    S1, S2, S3 = new_scores(other), new_scores(one), new_scores(other)
    D.dapq_score_static(other.shape, other.q, other.k, S1)
    D.dapq_score_static(one.shape, one.q, one.k, S2)
    D.dapq_score_static(other.shape, other.q, other.k, S3)
    torch.cuda.synchronize()
    assert torch.equal(S1, ref_other) and torch.equal(S2, ref_one) and torch.equal(S3, ref_other)
    assert_scores_close(S2.cpu().numpy(), O.score(one.q_bits, one.k_bits, one.Hkv, None, 128 ** -0.5), "static one-kernel")


def test_static_scratch_refuses_what_does_not_fit():
    w = W.workload("C3")                                        # ragged batch: 134 MB of workspace
    cu = torch.zeros(w.batch + 1, dtype=torch.int32, device="cuda")
    shape = D.make_shape(n_layers=w.n_layers, batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                         n_pseudo=w.n_pseudo, total_tokens=80000, cu_seqlens=cu,
                         k_strides=(80000 * 8 * 128, 0, 128, 8 * 128), q_strides=(8 * 32 * 128 * 128, 32 * 128 * 128, 128 * 128, 128),
                         scale=w.scale)
    assert D.workspace_bytes(shape) > D.score_static_capacity()
    fake = torch.empty(16, dtype=torch.uint8, device="cuda")    # never dereferenced: the call must fail on the host
    with pytest.raises(D.DapqError) as e:
        D.dapq_score_static(shape, fake, fake, fake)
    assert e.value.code == -3 and "built-in scratch" in str(e.value)
