"""Shared helpers of the GPU parity tests: device tensors from host bit patterns, one call per
C-ABI entry point, and the comparison rules (score tolerance, retained-set rule)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2603_11564_amd as D
from oracle import dapq_oracle as O

SCORE_RTOL = 1e-3      # relative error allowed on fp32 scores against the float64 oracle
MARGIN_RTOL = 1e-4     # retained sets must be identical when the boundary is clearer than this


def dev_bf16(bits: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class Problem:
    """Device-side view of one problem.  k/v are [layers, tokens, Hkv, d] ("thd") or
    [layers, Hkv, tokens, d] ("hnd"); q is [layers, batch, Hq, N, d]."""

    def __init__(self, q_bits, k_bits, v_bits, n_kv_heads, cu_seqlens=None, layout="thd", scale=None,
                 device="cuda"):
        self.q_bits, self.k_bits, self.v_bits = q_bits, k_bits, v_bits      # host, thd
        self.layers, self.batch, self.Hq, self.N, self.d = q_bits.shape
        self.tokens = k_bits.shape[1]
        self.Hkv = n_kv_heads
        self.layout = layout
        self.cu_host = None if cu_seqlens is None else np.asarray(cu_seqlens, dtype=np.int32)
        self.cu = None if cu_seqlens is None else torch.from_numpy(self.cu_host).to(device)
        self.q = dev_bf16(q_bits, device)
        if layout == "thd":
            self.k, self.v = dev_bf16(k_bits, device), dev_bf16(v_bits, device)
            ks = (self.tokens * self.Hkv * self.d, 0, self.d, self.Hkv * self.d)
        else:
            self.k = dev_bf16(k_bits.transpose(0, 2, 1, 3), device)
            self.v = dev_bf16(v_bits.transpose(0, 2, 1, 3), device)
            ks = (self.tokens * self.Hkv * self.d, 0, self.tokens * self.d, self.d)
        qs = (self.batch * self.Hq * self.N * self.d, self.Hq * self.N * self.d, self.N * self.d, self.d)
        self.shape = D.make_shape(n_layers=self.layers, batch=self.batch, n_q_heads=self.Hq, n_kv_heads=self.Hkv,
                                  n_pseudo=self.N, total_tokens=self.tokens, cu_seqlens=self.cu,
                                  k_strides=ks, v_strides=ks, q_strides=qs,
                                  scale=self.d ** -0.5 if scale is None else scale)
        self.device = device
        self.ws = torch.empty(max(D.workspace_bytes(self.shape), 256), dtype=torch.uint8, device=device)

    def seq_bounds(self):
        if self.cu_host is None:
            L = self.tokens // self.batch
            return [(b * L, (b + 1) * L) for b in range(self.batch)]
        return [(int(self.cu_host[b]), int(self.cu_host[b + 1])) for b in range(self.batch)]

    # ---- one call per entry point -----------------------------------------------------------
    def score(self):
        S = torch.full((self.layers, self.Hkv, self.tokens), float("nan"), dtype=torch.float32, device=self.device)
        D.dapq_score(self.shape, self.q, self.k, S, self.ws)
        return S

    def score_split(self):
        """The same scores through the two separate entry points (pass 1 + merge, then pass 2)."""
        lse = self.stats()
        S = torch.full((self.layers, self.Hkv, self.tokens), float("nan"), dtype=torch.float32, device=self.device)
        D.dapq_score_accumulate(self.shape, self.q, self.k, lse, S, self.ws)
        return S

    def stats(self):
        lse = torch.full((self.layers, self.batch, self.Hq, self.N), float("nan"), dtype=torch.float32,
                         device=self.device)
        D.dapq_score_stats(self.shape, self.q, self.k, lse, self.ws)
        return lse

    def score_extended(self, kp_bits):
        """S with every row normalised over the extended sequence: pass 1, the causal block of the pseudo
        tokens' own keys (kp_bits: [layers, batch, Hkv, N, d]), pass 2."""
        kp = dev_bf16(kp_bits, self.device)
        lse = self.stats()
        strides = (self.batch * self.Hkv * self.N * self.d, self.Hkv * self.N * self.d, self.N * self.d, self.d)
        D.dapq_score_stats_extend(self.shape, self.q, kp, strides, lse)
        S = torch.full((self.layers, self.Hkv, self.tokens), float("nan"), dtype=torch.float32, device=self.device)
        D.dapq_score_accumulate(self.shape, self.q, self.k, lse, S, self.ws)
        return S

    def pool(self, S, width=7):
        P = torch.full_like(S, float("nan"))
        D.dapq_pool(self.shape, S, P, width)
        return P

    def topk_workspace(self, budget, pieces=True):
        """The optional workspace of the selection calls (long heads go in pieces through it), filled with a
        pattern: the calls must not rely on its contents.  None if the shape needs none or `pieces` is False."""
        n = D.topk_workspace_bytes(self.shape, budget) if pieces else 0
        return torch.full((n,), 0xA5, dtype=torch.uint8, device=self.device) if n else None

    def topk(self, P, budget, per_seq=None, pieces=True):
        idx = torch.full((self.layers, self.batch, self.Hkv, budget), -7, dtype=torch.int32, device=self.device)
        count = torch.full((self.layers, self.batch, self.Hkv), -7, dtype=torch.int32, device=self.device)
        ps = None if per_seq is None else torch.tensor(per_seq, dtype=torch.int32, device=self.device)
        D.dapq_topk(self.shape, P, budget, ps, idx, count, self.topk_workspace(budget, pieces))
        return idx, count

    def pool_topk(self, S, width, budget, per_seq=None, want_pooled=True, pieces=False):
        idx = torch.full((self.layers, self.batch, self.Hkv, budget), -7, dtype=torch.int32, device=self.device)
        count = torch.full((self.layers, self.batch, self.Hkv), -7, dtype=torch.int32, device=self.device)
        ps = None if per_seq is None else torch.tensor(per_seq, dtype=torch.int32, device=self.device)
        P = torch.full_like(S, float("nan")) if want_pooled else None
        D.dapq_pool_topk(self.shape, S, width, budget, ps, idx, count, P, workspace=self.topk_workspace(budget, pieces))
        return idx, count, P

    def gather(self, idx, count, budget):
        ko = torch.zeros((self.layers, self.batch, self.Hkv, budget, self.d), dtype=torch.bfloat16,
                         device=self.device)
        vo = torch.zeros_like(ko)
        D.dapq_gather(self.shape, self.k, self.v, idx, count, budget, ko, vo)
        return ko, vo


def rope_gpu(bits: np.ndarray, pos: np.ndarray, theta: float, pairing=0, device="cuda") -> np.ndarray:
    """dapq_rope_apply on a contiguous [rows, heads, d] bf16 array."""
    rows, heads, d = bits.shape
    x = dev_bf16(bits, device)
    y = torch.empty_like(x)
    p = torch.from_numpy(np.asarray(pos, dtype=np.int32)).to(device)
    D.dapq_rope_apply(x, y, p, rows, heads, d, heads * d, d, theta, pairing)
    return host_bits(y)


def rope_problem_oracle(p, theta):
    """Post-RoPE bit patterns of a workloads.host_problem() dict, computed by the oracle."""
    q = np.empty_like(p["q"])
    for l in range(p["q"].shape[0]):
        for b in range(p["q"].shape[1]):
            q[l, b] = O.rope_apply(p["q"][l, b].transpose(1, 0, 2), p["q_pos"][b], theta).transpose(1, 0, 2)
    k = np.stack([O.rope_apply(p["k"][l], p["k_pos"], theta) for l in range(p["k"].shape[0])])
    return q, k


def assert_scores_close(got, want, what="scores"):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert np.isfinite(got).all(), f"{what}: non-finite values from the GPU"
    err = np.abs(got - want) / np.maximum(np.abs(want), 1e-30)
    worst = float(err.max()) if err.size else 0.0
    assert worst <= SCORE_RTOL, f"{what}: max relative error {worst:.3e} > {SCORE_RTOL}"
    return worst


def check_retained(P_oracle, idx_gpu, Kb):
    """Retained-set rule.  P_oracle: float64 pooled scores of one head; idx_gpu: the GPU's ascending
    positions.  If the boundary score is separated from its neighbouring distinct values by more than
    MARGIN_RTOL (relative), the set must equal the oracle's; otherwise every kept key must score at
    least v(1-tol), every key scoring above v(1+tol) must be kept, and the size must be right.
    Returns "exact" or "margin"."""
    L = P_oracle.shape[0]
    n = min(Kb, L)
    idx_gpu = np.asarray(idx_gpu[:n], dtype=np.int64)
    assert (np.diff(idx_gpu) > 0).all(), "positions not strictly ascending"
    assert idx_gpu.size == 0 or (idx_gpu[0] >= 0 and idx_gpu[-1] < L), "position outside the sequence"
    want = O.topk(P_oracle, Kb)
    v, gap = O.topk_margin(P_oracle, Kb)
    if gap > MARGIN_RTOL:
        assert np.array_equal(idx_gpu, want), "retained set differs although the boundary margin is clear"
        return "exact"
    kept = np.zeros(L, dtype=bool)
    kept[idx_gpu] = True
    assert (P_oracle[idx_gpu] >= v * (1 - MARGIN_RTOL)).all(), "kept a key below the boundary band"
    assert kept[P_oracle > v * (1 + MARGIN_RTOL)].all(), "dropped a key above the boundary band"
    return "margin"
