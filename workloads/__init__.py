"""Seeded synthetic workloads for the DapQ eviction step.

This module only *draws inputs*: pre-RoPE pseudo queries, pre-RoPE prompt keys (with planted
needle keys or a heavy-hitter tail), values, sequence lengths and position ids.  It contains none
of the method's arithmetic (no rotary embedding, no softmax, no pooling, no selection), so both the
CPU oracle's tests and the GPU path's tests / benchmark can take their inputs from it without
sharing any code of the method.  The tensors stand in for the activations of the models the paper
evaluates (Sec. 5.1), which need trained weights that are not available here: shapes follow those
models, values are N(0,1).

Every slice (layer, sequence, head) has its own counter-based Philox stream keyed by
(seed, kind, layer, sequence, head), so any slice can be regenerated alone, in any order, on any
machine, and a full-size tensor never has to exist on the host.

bf16 values are returned as uint16 bit patterns.  A float64 draw becomes bf16 by rounding to
float32 and then to bf16, both round-to-nearest-even; the bits this module returns *are* the
workload, whatever path they took.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import numpy as np

_KIND_Q, _KIND_K, _KIND_V, _KIND_NEEDLE, _KIND_HEAVY, _KIND_LEN, _KIND_FILL, _KIND_X, _KIND_WQ = range(9)


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_pseudo: int                 # N
    budget: int                   # Kb per KV head
    seq_len: int                  # L_p when the batch is not ragged
    ragged: Optional[Tuple[int, int]] = None   # (lo, hi): L_p of each sequence uniform in [lo, hi]
    pool_width: int = 7
    theta: float = 500000.0
    needles: int = 0              # planted needle keys per (layer, sequence, KV head)
    needle_gain: float = 3.0
    heavy_frac: float = 0.0       # fraction of keys scaled by heavy_gain (pre-RoPE)
    heavy_gain: float = 4.0
    layout: str = "hnd"           # "hnd": K[layer][Hkv][L][d] (batch 1); "thd": K[layer][token][Hkv][d]

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


# The five configurations the benchmark and the parity tests use (names C1..C5).
def workload(name: str, n_pseudo: Optional[int] = None) -> Workload:
    if name == "C1":    # single layer, small: the case the oracle finishes in well under a second
        w = Workload("C1", 1, 1, 32, 8, 128, 64, 128, 1024, needles=4)
    elif name == "C2":  # Llama-3-8B shape, 32k prompt, 3 % budget: the configuration the metric is quoted on
        w = Workload("C2", 32, 1, 32, 8, 128, 64, 983, 32768, needles=16)
    elif name == "C3":  # ragged batch of 8, packed token-major layout, heavy-hitter tail
        w = Workload("C3", 32, 8, 32, 8, 128, 128, 512, 0, ragged=(4096, 16384),
                     heavy_frac=0.10, layout="thd")
    elif name == "C4":  # pseudo-query length sweep, 64k prompt
        w = Workload("C4", 32, 1, 32, 8, 128, 64 if n_pseudo is None else n_pseudo, 2048, 65536,
                     needles=32)
    elif name == "C5":  # 70B-class shape, 128k prompt, all 80 layers resident
        w = Workload("C5", 80, 1, 64, 8, 128, 64, 3932, 131072, needles=64)
    else:
        raise KeyError(name)
    if n_pseudo is not None and name != "C4":
        w = replace(w, n_pseudo=n_pseudo)
    return w


def _rng(seed: int, kind: int, layer: int = 0, seq: int = 0, head: int = 0) -> np.random.Generator:
    key0 = int(seed) & 0xFFFFFFFFFFFFFFFF
    key1 = ((kind & 0xFF) << 56) | ((layer & 0xFFFF) << 40) | ((seq & 0xFFFFF) << 20) | (head & 0xFFFFF)
    return np.random.Generator(np.random.Philox(key=[key0, key1]))


def to_bf16_bits(x) -> np.ndarray:
    """float -> float32 (RNE) -> bf16 (RNE) bit patterns."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(bits) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def seq_lens(w: Workload, seed: int) -> List[int]:
    """Prompt length of every sequence of the batch."""
    if w.ragged is None:
        return [w.seq_len] * w.batch
    lo, hi = w.ragged
    return [int(v) for v in _rng(seed, _KIND_LEN).integers(lo, hi + 1, size=w.batch)]


def cu_seqlens(w: Workload, seed: int) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(seq_lens(w, seed))]).astype(np.int32)


def q_positions(L: int, n_pseudo: int) -> np.ndarray:
    """Position ids of the pseudo queries of a prompt of length L: L .. L+N-1 (Sec. 4.1)."""
    return np.arange(L, L + n_pseudo, dtype=np.int32)


def k_positions(L: int) -> np.ndarray:
    return np.arange(L, dtype=np.int32)


def q_pre(w: Workload, seed: int, layer: int, seq: int) -> np.ndarray:
    """Pre-RoPE pseudo queries of one (layer, sequence): bf16 bits [Hq, N, d], N(0,1)."""
    out = np.empty((w.n_q_heads, w.n_pseudo, w.head_dim), dtype=np.uint16)
    for h in range(w.n_q_heads):
        out[h] = to_bf16_bits(_rng(seed, _KIND_Q, layer, seq, h).standard_normal(
            (w.n_pseudo, w.head_dim), dtype=np.float32))
    return out


def projection_rows(seed: int, layer: int, tokens: int, hidden: int) -> np.ndarray:
    """Input rows of one layer's query projection (the normalised hidden states of the prompt tokens):
    bf16 bits [tokens, hidden], N(0,1) -- unit RMS, as a normalisation layer leaves them."""
    return to_bf16_bits(_rng(seed, _KIND_X, layer).standard_normal((tokens, hidden), dtype=np.float32))


def query_weight(seed: int, layer: int, features: int, hidden: int) -> np.ndarray:
    """Query weight of one layer, one row per output feature: bf16 bits [features, hidden], N(0, 1/hidden),
    so that the projected queries are N(0,1) like q_pre()."""
    w = _rng(seed, _KIND_WQ, layer).standard_normal((features, hidden), dtype=np.float32)
    return to_bf16_bits(w / np.float32(np.sqrt(hidden)))


def needle_plan(w: Workload, seed: int, layer: int, seq: int, kv_head: int, L: int):
    """Where the needle keys of one (layer, sequence, KV head) sit and which pseudo query each copies.

    Returns (pos [n], q_head [n], q_row [n]).  One needle per equal stratum of [0, L), at a seeded
    offset inside the stratum; the copied query is uniform over the KV head's group and over [0, N).
    """
    n = min(w.needles, L)
    if n == 0:
        z = np.zeros(0, dtype=np.int64)
        return z, z, z
    r = _rng(seed, _KIND_NEEDLE, layer, seq, kv_head)
    edges = (np.arange(n + 1, dtype=np.int64) * L) // n
    pos = edges[:-1] + (r.random(n) * (edges[1:] - edges[:-1])).astype(np.int64)
    q_head = kv_head * w.group + r.integers(0, w.group, size=n)
    q_row = r.integers(0, w.n_pseudo, size=n)
    return pos, q_head, q_row


def needle_rows(w: Workload, q_pre_bits: np.ndarray, q_head, q_row) -> np.ndarray:
    """bf16 bits of the needle keys: needle_gain x the chosen pre-RoPE pseudo query, rounded to bf16."""
    q = from_bf16_bits(q_pre_bits[q_head, q_row]).astype(np.float64)
    return to_bf16_bits(w.needle_gain * q)


def heavy_mask(w: Workload, seed: int, layer: int, seq: int, kv_head: int, L: int) -> np.ndarray:
    if w.heavy_frac <= 0.0:
        return np.zeros(L, dtype=bool)
    return _rng(seed, _KIND_HEAVY, layer, seq, kv_head).random(L) < w.heavy_frac


def k_pre(w: Workload, seed: int, layer: int, seq: int, kv_head: int, L: int,
          q_pre_bits: Optional[np.ndarray] = None) -> np.ndarray:
    """Pre-RoPE prompt keys of one (layer, sequence, KV head): bf16 bits [L, d].

    N(0,1); a heavy-hitter subset is scaled by heavy_gain; needle rows are overwritten last."""
    x = _rng(seed, _KIND_K, layer, seq, kv_head).standard_normal((L, w.head_dim), dtype=np.float32)
    hm = heavy_mask(w, seed, layer, seq, kv_head, L)
    if hm.any():
        x[hm] *= np.float32(w.heavy_gain)
    bits = to_bf16_bits(x)
    if w.needles:
        if q_pre_bits is None:
            q_pre_bits = q_pre(w, seed, layer, seq)
        pos, qh, qr = needle_plan(w, seed, layer, seq, kv_head, L)
        bits[pos] = needle_rows(w, q_pre_bits, qh, qr)
    return bits


def v_rows(w: Workload, seed: int, layer: int, seq: int, kv_head: int, L: int) -> np.ndarray:
    """Prompt values of one (layer, sequence, KV head): bf16 bits [L, d], N(0,1)."""
    return to_bf16_bits(_rng(seed, _KIND_V, layer, seq, kv_head).standard_normal(
        (L, w.head_dim), dtype=np.float32))


def host_problem(w: Workload, seed: int, layers=None):
    """Whole pre-RoPE problem on the host (small workloads / selected layers only).

    Returns dict(q [layers, batch, Hq, N, d], k, v [layers, tokens, Hkv, d], cu_seqlens [batch+1],
    q_pos [batch, N], k_pos [tokens]) with bf16 tensors as uint16 bits."""
    layers = list(range(w.n_layers)) if layers is None else list(layers)
    lens = seq_lens(w, seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    tokens = int(cu[-1])
    q = np.empty((len(layers), w.batch, w.n_q_heads, w.n_pseudo, w.head_dim), dtype=np.uint16)
    k = np.empty((len(layers), tokens, w.n_kv_heads, w.head_dim), dtype=np.uint16)
    v = np.empty_like(k)
    for li, layer in enumerate(layers):
        for b, L in enumerate(lens):
            q[li, b] = q_pre(w, seed, layer, b)
            for kv in range(w.n_kv_heads):
                k[li, cu[b]:cu[b + 1], kv] = k_pre(w, seed, layer, b, kv, L, q[li, b])
                v[li, cu[b]:cu[b + 1], kv] = v_rows(w, seed, layer, b, kv, L)
    q_pos = np.stack([q_positions(L, w.n_pseudo) for L in lens])
    k_pos = np.concatenate([k_positions(L) for L in lens]).astype(np.int32)
    return dict(q=q, k=k, v=v, cu_seqlens=cu, q_pos=q_pos, k_pos=k_pos, layers=layers)


def device_fill(w: Workload, seed: int, device, layers=None):
    """Full-size pre-RoPE problem built directly in device memory with torch (plumbing only).

    Pseudo queries and needle rows are the exact host values of q_pre()/needle_rows(); the bulk of
    K and V is drawn by torch's device generator with the same N(0,1) / heavy-hitter recipe (its
    bits differ from k_pre()'s, so callers that compare against the oracle overwrite the slices
    they check with host-generated ones).  Returns torch tensors: q bf16 [layers, batch, Hq, N, d],
    k, v bf16 in w.layout, cu_seqlens int32 [batch+1], q_pos int32 [batch, N], k_pos int32 [tokens].
    """
    import torch

    layers = list(range(w.n_layers)) if layers is None else list(layers)
    lens = seq_lens(w, seed)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    tokens = int(cu[-1])
    nl = len(layers)
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) * 7919 + _KIND_FILL)
    if w.layout == "hnd":
        shape = (nl, w.n_kv_heads, tokens, w.head_dim)
    else:
        shape = (nl, tokens, w.n_kv_heads, w.head_dim)
    k = torch.empty(shape, dtype=torch.bfloat16, device=device)
    v = torch.empty(shape, dtype=torch.bfloat16, device=device)
    for li in range(nl):                                   # one layer at a time bounds the fp32 temporaries
        k[li].copy_(torch.randn(shape[1:], generator=gen, device=device, dtype=torch.float32))
        v[li].copy_(torch.randn(shape[1:], generator=gen, device=device, dtype=torch.float32))
        if w.heavy_frac > 0.0:
            tok_shape = (w.n_kv_heads, tokens, 1) if w.layout == "hnd" else (tokens, w.n_kv_heads, 1)
            hm = torch.rand(tok_shape, generator=gen, device=device) < w.heavy_frac
            k[li].mul_(torch.where(hm, w.heavy_gain, 1.0).to(torch.bfloat16))
    q_host = np.empty((nl, w.batch, w.n_q_heads, w.n_pseudo, w.head_dim), dtype=np.uint16)
    for li, layer in enumerate(layers):
        for b in range(w.batch):
            q_host[li, b] = q_pre(w, seed, layer, b)
    q = torch.from_numpy(q_host.view(np.int16)).to(device).view(torch.bfloat16)
    if w.needles:
        for li, layer in enumerate(layers):
            for b, L in enumerate(lens):
                for kv in range(w.n_kv_heads):
                    pos, qh, qr = needle_plan(w, seed, layer, b, kv, L)
                    rows = needle_rows(w, q_host[li, b], qh, qr)
                    rows_t = torch.from_numpy(rows.view(np.int16)).to(device).view(torch.bfloat16)
                    pos_t = torch.from_numpy(pos + int(cu[b])).to(device)
                    if w.layout == "hnd":
                        k[li, kv].index_copy_(0, pos_t, rows_t)
                    else:
                        k[li, :, kv].index_copy_(0, pos_t, rows_t)
    q_pos = torch.from_numpy(np.stack([q_positions(L, w.n_pseudo) for L in lens])).to(device)
    k_pos = torch.from_numpy(np.concatenate([k_positions(L) for L in lens]).astype(np.int32)).to(device)
    return dict(q=q, k=k, v=v, cu_seqlens=torch.from_numpy(cu).to(device), q_pos=q_pos, k_pos=k_pos,
                layers=layers, lens=lens)
