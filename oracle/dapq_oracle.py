"""Float64 CPU oracle for DapQ's eviction step (score -> pool -> top-K -> gather).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, written-out definition of
what the eviction path computes.  It is imported by the tests, by the smoke check
and by the benchmark's CPU-baseline leg, and by nothing else: the GPU library never
calls it, shares no code with it, and does not import it.  Nothing here is blocked,
fused or reordered; every function follows one passage of the paper and can be
checked against it by eye.  numpy.matmul / numpy.exp / list sorting are the only
library primitives used.

Symbols (the paper overloads N and K; this file uses):
    L      prompt length L_p (number of prompt keys of one sequence)      Sec. 4.1
    N      number of pseudo queries (observation-window size)             Sec. 4.1
    Kb     retention budget per KV head (the paper's "cache of size K")   Sec. 4.2
    g      query heads sharing one KV head (grouped-query attention)
    d      head dimension d_k                                  App. C.1, theorem

Readings taken where the paper is silent (each is listed in the design notes of
this repository): the softmax runs over the L prompt keys only (Sec. 4.2 indexes
j in [0, L_p-1]) unless the pseudo tokens' own keys are passed in, in which case the
extended sequence of Sec. 4.1 is attended causally; scores of the g query heads of a group are summed and selection
is per KV head; pooling is a stride-1 max over a centred window clipped at the
sequence ends, applied after the group sum; TopK ties go to the lowest index and
the retained set is reported in ascending position; RoPE pairs channel c with
c + d/2 and uses no frequency rescaling; a pseudo token's row of a layer's query
projection input is the row of the prompt token it copies (exact where rows do not
depend on position, i.e. at the embedding; the paper's point that content is
secondary covers the rest), and the projection is rounded to bf16 before the rotation.

Parity status: every function below is pinned by tests/test_oracle_pins.py against
closed forms, invariants, brute force or hand-worked fixtures (tests/golden/).
The paper's end-task numbers (LongBench, NIAH, ...) need trained weights and data
sets that are not available: "parity unpinned" for those, and they are not a goal.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits_to_f64", "f64_to_bf16_bits", "rope_rotate", "rope_apply", "attention", "score_head",
    "score", "pool", "topk", "gather", "compress", "recall", "topk_margin", "attention_extended",
    "decode_attention", "pseudo_tokens", "pseudo_queries",
]


# --------------------------------------------------------------------------------------
# bfloat16 <-> float64 (storage format of Q, K, V; not part of the method itself)
# --------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits) -> np.ndarray:
    """Decode bfloat16 bit patterns (uint16) exactly: bf16 is the top half of an IEEE float32."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x) -> np.ndarray:
    """Round float64 to the nearest bfloat16, ties to the even mantissa, and return the bits.

    Done directly on the float64 value (no intermediate float32 rounding, which could
    double-round): a finite bf16 has 8 significant bits, so x is scaled to put those
    8 bits in the integer part, rounded half-to-even with numpy.rint, and scaled back.
    The result is exactly representable in float32, whose top 16 bits are the answer.
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.zeros(x.shape, dtype=np.float64)
    finite = np.isfinite(x) & (x != 0.0)
    m, e = np.frexp(x[finite])                       # x = m * 2**e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)                          # below 2**-126: fixed (subnormal) spacing
    q = np.rint(np.ldexp(x[finite], 8 - e))          # 8 significant bits -> integer part
    out[finite] = np.ldexp(q, e - 8)
    out[~np.isfinite(x)] = x[~np.isfinite(x)]
    f32 = out.astype(np.float32)                     # exact for every in-range value
    f32 = np.where(np.signbit(x) & (f32 == 0), np.float32(-0.0), f32).astype(np.float32)
    return (f32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------------------
# Sec. 4.1: positions of the pseudo tokens, applied through rotary position embedding
# --------------------------------------------------------------------------------------
def rope_rotate(x, pos, theta: float = 500000.0, pairing: str = "half") -> np.ndarray:
    """Rotate each (row, head) vector of float64 x [rows, heads, d] to the position pos[row].

    Sec. 4.1 assigns the pseudo tokens the positions L_p .. L_p+N-1; the models the paper runs
    encode a position p by rotating channel pair c through the angle p * theta**(-2c/d).
    pairing "half" pairs channel c with c + d/2, "interleaved" pairs 2c with 2c+1.
    Everything is float64; nothing is rounded here.
    """
    x = np.asarray(x, dtype=np.float64)
    rows, heads, d = x.shape
    pos = np.asarray(pos, dtype=np.float64).reshape(rows, 1, 1)
    c = np.arange(d // 2, dtype=np.float64)
    omega = theta ** (-2.0 * c / d)                  # [d/2]
    ang = pos * omega                                # [rows, 1, d/2]
    cos, sin = np.cos(ang), np.sin(ang)
    if pairing == "half":
        a, b = x[..., : d // 2], x[..., d // 2:]
    elif pairing == "interleaved":
        a, b = x[..., 0::2], x[..., 1::2]
    else:
        raise ValueError(pairing)
    ra = a * cos - b * sin
    rb = b * cos + a * sin
    y = np.empty_like(x)
    if pairing == "half":
        y[..., : d // 2], y[..., d // 2:] = ra, rb
    else:
        y[..., 0::2], y[..., 1::2] = ra, rb
    return y


def rope_apply(x_bits, pos, theta: float = 500000.0, pairing: str = "half") -> np.ndarray:
    """bf16 in, bf16 out: decode exactly, rope_rotate in float64, round to bf16 once.
    x_bits: bf16 bits [rows, heads, d]; pos: integer [rows]."""
    return f64_to_bf16_bits(rope_rotate(bf16_bits_to_f64(x_bits), pos, theta, pairing))


# --------------------------------------------------------------------------------------
# App. C.1 (theorem statement and Step 1): Attention(q, K) = softmax(q K^T / sqrt(d_k))
# --------------------------------------------------------------------------------------
def attention(q, k, scale=None) -> np.ndarray:
    """Attention weights of each query row over the keys: alpha = softmax(q k^T * scale).

    q: float64 [rows, d]; k: float64 [L, d]; returns float64 [rows, L], every row >= 0
    and summing to 1 (App. C.1, Step 1).  scale defaults to 1/sqrt(d_k).  The row
    maximum is subtracted before exponentiating, which leaves the softmax unchanged.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[-1])
    s = (q @ k.T) * scale                            # pre-softmax scores s_j
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def attention_extended(q, k, k_pseudo, scale=None) -> np.ndarray:
    """Attention weights of the pseudo queries over the extended sequence of Sec. 4.1: the L prompt
    keys followed by the N keys of the pseudo tokens themselves, prefilled causally, so that query i
    (position L_p+i) sees every prompt key and the pseudo keys at positions L_p..L_p+i.

    q: float64 [N, d]; k: float64 [L, d]; k_pseudo: float64 [N, d]; returns float64 [N, L+N] with
    zeros where the causal mask hides a key; every row sums to 1."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    kp = np.asarray(k_pseudo, dtype=np.float64)
    N, L = q.shape[0], k.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(q.shape[-1])
    s = (q @ np.concatenate([k, kp], axis=0).T) * scale
    for i in range(N):
        s[i, L + i + 1:] = -np.inf                   # pseudo tokens after query i do not exist yet
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


# --------------------------------------------------------------------------------------
# Sec. 4.2, importance score: S(j) = sum over the pseudo queries of Attention(q_i, k_j)
# --------------------------------------------------------------------------------------
def score_head(q, k, scale=None, k_pseudo=None) -> np.ndarray:
    """S(j) for one KV head.  q: float64 [g, N, d] (the g query heads of the group, N pseudo
    queries each, already rotated to L_p+i); k: float64 [L, d] (prompt keys, rotated).
    Sum over the N pseudo queries (Sec. 4.2) and over the g heads of the group.
    k_pseudo (float64 [N, d], the KV head's keys of the pseudo tokens): if given, every row is
    normalised over the extended sequence (attention_extended); S is still reported for the
    prompt keys only, j in [0, L_p-1]."""
    q = np.asarray(q, dtype=np.float64)
    g, N, d = q.shape
    if k_pseudo is None:
        alpha = attention(q.reshape(g * N, d), k, scale)
        return alpha.sum(axis=0)
    L = np.asarray(k).shape[0]
    S = np.zeros(L, dtype=np.float64)
    for h in range(g):
        S += attention_extended(q[h], k, k_pseudo, scale)[:, :L].sum(axis=0)
    return S


def _seq_bounds(total_tokens, batch, cu_seqlens):
    if cu_seqlens is None:
        L = total_tokens // batch
        return [(b * L, (b + 1) * L) for b in range(batch)]
    cu = [int(v) for v in cu_seqlens]
    return [(cu[b], cu[b + 1]) for b in range(batch)]


def score(q_bits, k_bits, n_kv_heads, cu_seqlens=None, scale=None, kp_bits=None) -> np.ndarray:
    """Scores for a (possibly ragged) batch.  q_bits: bf16 bits [layers, batch, Hq, N, d];
    k_bits: bf16 bits [layers, tokens, Hkv, d] with the sequences packed along tokens;
    cu_seqlens: [batch+1] token offsets (None: equal lengths); kp_bits: optional bf16 bits
    [layers, batch, Hkv, N, d], the pseudo tokens' own keys (see score_head).  Returns float64
    [layers, Hkv, tokens].  Query head h belongs to KV head h // g."""
    q_bits = np.asarray(q_bits)
    k_bits = np.asarray(k_bits)
    layers, batch, Hq, N, d = q_bits.shape
    tokens = k_bits.shape[1]
    g = Hq // n_kv_heads
    out = np.zeros((layers, n_kv_heads, tokens), dtype=np.float64)
    for l in range(layers):
        for b, (s, e) in enumerate(_seq_bounds(tokens, batch, cu_seqlens)):
            if e == s:
                continue
            for kv in range(n_kv_heads):
                q = bf16_bits_to_f64(q_bits[l, b, kv * g:(kv + 1) * g])
                k = bf16_bits_to_f64(k_bits[l, s:e, kv])
                kp = None if kp_bits is None else bf16_bits_to_f64(np.asarray(kp_bits)[l, b, kv])
                out[l, kv, s:e] = score_head(q, k, scale, kp)
    return out


# --------------------------------------------------------------------------------------
# Sec. 1 / Sec. 5.1: selection works on *pooled* accumulated attention scores
# --------------------------------------------------------------------------------------
def pool(S, width: int = 7) -> np.ndarray:
    """P(j) = max{ S(t) : |t - j| <= (width-1)/2, 0 <= t < L } for one sequence (1-D S)."""
    S = np.asarray(S, dtype=np.float64)
    L = S.shape[0]
    r = (width - 1) // 2
    P = np.empty_like(S)
    for j in range(L):
        P[j] = S[max(0, j - r):min(L, j + r + 1)].max()
    return P


# --------------------------------------------------------------------------------------
# Sec. 4.2: M_retain = TopK_j S(j)
# --------------------------------------------------------------------------------------
def topk(P, Kb: int) -> np.ndarray:
    """The min(Kb, L) positions with the highest scores, ties to the lowest position,
    returned in ascending position (int64)."""
    P = np.asarray(P)
    order = sorted(range(P.shape[0]), key=lambda j: (-P[j], j))
    return np.array(sorted(order[:max(0, min(int(Kb), P.shape[0]))]), dtype=np.int64)


def topk_margin(P, Kb: int):
    """Boundary value v (the lowest retained score) and its relative distance to the nearest
    *distinct* score value above and below it; (v, inf) when no other value exists.  Used by the
    parity tests to decide whether a retained set must match bit for bit."""
    P = np.asarray(P, dtype=np.float64)
    if Kb >= P.shape[0] or Kb <= 0:
        return None, np.inf
    vals = np.sort(P)[::-1]
    v = vals[Kb - 1]
    lower = vals[vals < v]
    upper = vals[vals > v]
    gaps = []
    if lower.size:
        gaps.append((v - lower[0]) / v)
    if upper.size:
        gaps.append((upper[-1] - v) / v)
    return v, (min(gaps) if gaps else np.inf)


# --------------------------------------------------------------------------------------
# Sec. 4.2: the cache keeps only the pairs in M_retain; the pseudo segment is dropped
# --------------------------------------------------------------------------------------
def gather(kv_bits, idx) -> np.ndarray:
    """Rows idx of a [L, d] bit-pattern array, copied bit for bit."""
    return np.asarray(kv_bits)[np.asarray(idx, dtype=np.int64)].copy()


def compress(q_bits, k_bits, v_bits, n_kv_heads, Kb, cu_seqlens=None, width=7, scale=None):
    """The whole eviction step.  Shapes as in score(); v_bits like k_bits.  Kb is one budget or a
    per-sequence list.  Returns a dict with
      S, P    float64 [layers, Hkv, tokens]   accumulated / pooled scores
      idx     int64   [layers, batch, Hkv, Kmax]  retained positions inside the sequence, ascending,
                                              slots past count hold -1
      count   int64   [layers, batch, Hkv]
      k_out, v_out  uint16 [layers, batch, Hkv, Kmax, d], rows past count are zero."""
    q_bits = np.asarray(q_bits)
    k_bits = np.asarray(k_bits)
    v_bits = np.asarray(v_bits)
    layers, batch = q_bits.shape[:2]
    tokens, d = k_bits.shape[1], k_bits.shape[3]
    budgets = [int(Kb)] * batch if np.ndim(Kb) == 0 else [int(v) for v in Kb]
    Kmax = max(budgets) if budgets else 0
    S = score(q_bits, k_bits, n_kv_heads, cu_seqlens, scale)
    P = np.zeros_like(S)
    idx = np.full((layers, batch, n_kv_heads, Kmax), -1, dtype=np.int64)
    count = np.zeros((layers, batch, n_kv_heads), dtype=np.int64)
    k_out = np.zeros((layers, batch, n_kv_heads, Kmax, d), dtype=np.uint16)
    v_out = np.zeros_like(k_out)
    for l in range(layers):
        for b, (s, e) in enumerate(_seq_bounds(tokens, batch, cu_seqlens)):
            for kv in range(n_kv_heads):
                P[l, kv, s:e] = pool(S[l, kv, s:e], width)
                keep = topk(P[l, kv, s:e], budgets[b])
                n = keep.shape[0]
                count[l, b, kv] = n
                idx[l, b, kv, :n] = keep
                k_out[l, b, kv, :n] = gather(k_bits[l, s:e, kv], keep)
                v_out[l, b, kv, :n] = gather(v_bits[l, s:e, kv], keep)
    return dict(S=S, P=P, idx=idx, count=count, k_out=k_out, v_out=v_out)


# --------------------------------------------------------------------------------------
# Sec. 4.1 / Sec. 5.1: the pseudo tokens (which prompt tokens they copy, their positions) and their queries
# --------------------------------------------------------------------------------------
def pseudo_tokens(L: int, first_m: int, last_n: int):
    """Sec. 4.1 / Sec. 5.1: the N = m + n pseudo tokens take their content from the first m and the
    last n tokens of the prompt (the paper's Fm_Ln construction) and the positions L_p .. L_p+N-1 of the
    first N decode steps.  Returns (source token of each pseudo token, position of each pseudo token).
    A prompt shorter than m or n repeats its first / last token; an empty prompt has no source (-1)."""
    src = []
    for t in range(first_m):
        src.append(min(t, L - 1))
    for t in range(last_n):
        src.append(max(L - last_n + t, 0) if L > 0 else -1)
    pos = [L + i for i in range(first_m + last_n)]
    return np.asarray(src, dtype=np.int64), np.asarray(pos, dtype=np.int64)


def pseudo_queries(x_bits, token_idx, w_bits, n_q_heads, positions=None, theta: float = 500000.0,
                   pairing: str = "half") -> np.ndarray:
    """Sec. 4.1: the queries the model computes for the pseudo tokens of one layer.  Pseudo token r takes
    its content from prompt token token_idx[r] (its row of the layer's query-projection input is that
    token's row: content is secondary, the position is what is assigned), is projected by the layer's
    query weight, split into heads and rotated to its position:
        q[h, r, :] = RoPE_{positions[r]}( bf16( x[token_idx[r], :] . w[h*d:(h+1)*d, :]^T ) ).
    x_bits: bf16 bits [tokens, hidden]; token_idx: [rows], -1 = no source (an empty prompt), the query is
    zero; w_bits: bf16 bits [Hq*d, hidden], one row per output feature; positions: [rows] or None (no
    rotation).  The product is exact in float64 up to its summation; it is rounded to bf16 once, which is
    the precision the model hands its queries on in, then rotated by rope_apply.
    Returns bf16 bits [Hq, rows, d]."""
    x = bf16_bits_to_f64(x_bits)
    w = bf16_bits_to_f64(w_bits)
    token_idx = np.asarray(token_idx, dtype=np.int64)
    rows, hidden = token_idx.shape[0], w.shape[1]
    assert w.shape[0] % n_q_heads == 0
    d = w.shape[0] // n_q_heads
    xg = np.zeros((rows, hidden), dtype=np.float64)
    for r in range(rows):
        if token_idx[r] >= 0:
            xg[r] = x[token_idx[r]]
    q_bits = f64_to_bf16_bits(xg @ w.T).reshape(rows, n_q_heads, d)
    if positions is not None:
        q_bits = rope_apply(q_bits, positions, theta, pairing)
    return np.ascontiguousarray(q_bits.transpose(1, 0, 2))


# --------------------------------------------------------------------------------------
# Sec. 4.2, last paragraph: decoding from position L_p over the compressed cache only
# --------------------------------------------------------------------------------------
def decode_attention(q, k_cache, v_cache, scale=None) -> np.ndarray:
    """One decode step over a cache (Sec. 4.2, last paragraph: decoding starts at position L_p and uses
    only the compressed cache): o = Attention(q, K) V with Attention = softmax(q K^T / sqrt(d_k))
    (App. C.1).  q: float64 [rows, d] (already rotated to the decode position); k_cache, v_cache:
    float64 [n, d]; returns float64 [rows, d]."""
    alpha = attention(q, k_cache, scale)
    return alpha @ np.asarray(v_cache, dtype=np.float64)


# --------------------------------------------------------------------------------------
# Sec. 3.3: recall of a predicted retained set against a gold one
# --------------------------------------------------------------------------------------
def recall(M_gold, M_pred) -> float:
    """|M_gold ∩ M_pred| / |M_gold| (Sec. 3.3, recall equation)."""
    gold = set(int(v) for v in M_gold)
    pred = set(int(v) for v in M_pred)
    return len(gold & pred) / len(gold)
