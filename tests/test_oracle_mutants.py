"""Do the pins bite?  Every entry below plants one plausible mistake in a copy of the oracle's source (a dropped
term, a wrong sign or index, a transposed operand, a rounding done in the wrong place) and runs the pin tests
against that copy, on the CPU, in a process of its own.  Each mutant must make at least one pin fail.  Nothing here touches the GPU path; the
mutated copies live in a temporary directory."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# name -> (text in oracle/dapq_oracle.py, what the mistake puts there)
MUTANTS = {
    # bf16 codec
    "bf16 rounds half up": ("q = np.rint(np.ldexp(x[finite], 8 - e))", "q = np.floor(np.ldexp(x[finite], 8 - e) + 0.5)"),
    "bf16 truncates": ("q = np.rint(np.ldexp(x[finite], 8 - e))", "q = np.trunc(np.ldexp(x[finite], 8 - e))"),
    "bf16 ignores the subnormal spacing": ("    e = np.maximum(e, -125) ", "    e = np.maximum(e, -1250) "),
    "bf16 loses the sign of zero": ("np.where(np.signbit(x) & (f32 == 0), np.float32(-0.0), f32)", "np.where(np.signbit(x) & (f32 == 7), np.float32(-0.0), f32)"),
    # rotary embedding
    "rope turns the other way": ("    ra = a * cos - b * sin\n    rb = b * cos + a * sin", "    ra = a * cos + b * sin\n    rb = b * cos - a * sin"),
    "rope frequency exponent halved": ("omega = theta ** (-2.0 * c / d)", "omega = theta ** (-1.0 * c / d)"),
    "rope frequency index starts at 1": ("c = np.arange(d // 2, dtype=np.float64)", "c = np.arange(1, d // 2 + 1, dtype=np.float64)"),
    "rope pairs neighbours where it should pair halves": ("        a, b = x[..., : d // 2], x[..., d // 2:]", "        a, b = x[..., 0::2], x[..., 1::2]"),
    # attention and scores
    "attention without the scale": ("    s = (q @ k.T) * scale   ", "    s = (q @ k.T) * 1.0     "),
    "attention scaled by 1/d": ("        scale = 1.0 / np.sqrt(q.shape[-1])\n    s = (q @ k.T) * scale ", "        scale = 1.0 / q.shape[-1]\n    s = (q @ k.T) * scale "),
    "softmax over the queries": ("    e = np.exp(s)\n    return e / e.sum(axis=1, keepdims=True)\n\n\ndef attention_extended", "    e = np.exp(s)\n    return e / e.sum(axis=0, keepdims=True)\n\n\ndef attention_extended"),
    "causal mask hides the query's own key": ("s[i, L + i + 1:] = -np.inf", "s[i, L + i:] = -np.inf"),
    "no causal mask among the pseudo tokens": ("s[i, L + i + 1:] = -np.inf ", "s[i, L + N + 1:] = -np.inf "),
    "pseudo keys in reverse order": ("np.concatenate([k, kp], axis=0)", "np.concatenate([k, kp[::-1]], axis=0)"),
    "extended scores reported for the wrong columns": ("attention_extended(q[h], k, k_pseudo, scale)[:, :L].sum(axis=0)", "attention_extended(q[h], k, k_pseudo, scale)[:, N:].sum(axis=0)"),
    "mean instead of sum over the pseudo queries": ("        return alpha.sum(axis=0)", "        return alpha.mean(axis=0)"),
    "query heads dealt round-robin to KV heads": ("q_bits[l, b, kv * g:(kv + 1) * g]", "q_bits[l, b, kv::n_kv_heads]"),
    "one query head of the group dropped": ("    g = Hq // n_kv_heads\n    out = np.zeros((layers, n_kv_heads, tokens)", "    g = max(1, Hq // n_kv_heads - 1)\n    out = np.zeros((layers, n_kv_heads, tokens)"),
    "pseudo keys of KV head 0 for every head": ("np.asarray(kp_bits)[l, b, kv]", "np.asarray(kp_bits)[l, b, 0]"),
    "pseudo keys of sequence 0 for every sequence": ("np.asarray(kp_bits)[l, b, kv]", "np.asarray(kp_bits)[l, 0, kv]"),
    # pooling, selection, pruning
    "pooling window too wide": ("    r = (width - 1) // 2", "    r = width // 2 + 1"),
    "pooling looks left only": ("S[max(0, j - r):min(L, j + r + 1)].max()", "S[max(0, j - r):j + 1].max()"),
    "mean pooling": ("S[max(0, j - r):min(L, j + r + 1)].max()", "S[max(0, j - r):min(L, j + r + 1)].mean()"),
    "ties to the highest position": ("key=lambda j: (-P[j], j)", "key=lambda j: (-P[j], -j)"),
    "keeps the smallest scores": ("key=lambda j: (-P[j], j)", "key=lambda j: (P[j], j)"),
    "retained set in score order": ("return np.array(sorted(order[:max(0, min(int(Kb), P.shape[0]))]), dtype=np.int64)", "return np.array(order[:max(0, min(int(Kb), P.shape[0]))], dtype=np.int64)"),
    "selection on the raw scores": ("keep = topk(P[l, kv, s:e], budgets[b])", "keep = topk(S[l, kv, s:e], budgets[b])"),
    "budget of sequence 0 for every sequence": ("keep = topk(P[l, kv, s:e], budgets[b])", "keep = topk(P[l, kv, s:e], budgets[0])"),
    "values gathered from the keys": ("v_out[l, b, kv, :n] = gather(v_bits[l, s:e, kv], keep)", "v_out[l, b, kv, :n] = gather(k_bits[l, s:e, kv], keep)"),
    "gather in descending position": ("np.asarray(kv_bits)[np.asarray(idx, dtype=np.int64)].copy()", "np.asarray(kv_bits)[np.sort(np.asarray(idx, dtype=np.int64))[::-1]].copy()"),
    "margin from the farthest value below": ("gaps.append((v - lower[0]) / v)", "gaps.append((v - lower[-1]) / v)"),
    "margin from the farthest value above": ("gaps.append((upper[-1] - v) / v)", "gaps.append((upper[0] - v) / v)"),
    "margin at the first dropped score": ("    v = vals[Kb - 1]", "    v = vals[Kb]"),
    # recall, pseudo tokens, their queries, decode
    "recall over the predicted set": ("return len(gold & pred) / len(gold)", "return len(gold & pred) / len(pred)"),
    "recall as intersection over union": ("return len(gold & pred) / len(gold)", "return len(gold & pred) / len(gold | pred)"),
    "last-n tokens off by one": ("src.append(max(L - last_n + t, 0) if L > 0 else -1)", "src.append(max(L - last_n + t - 1, 0) if L > 0 else -1)"),
    "first-m tokens not clipped to a short prompt": ("src.append(min(t, L - 1))", "src.append(t)"),
    "positions start one late": ("pos = [L + i for i in range(first_m + last_n)]", "pos = [L + i + 1 for i in range(first_m + last_n)]"),
    "query weight transposed": ("q_bits = f64_to_bf16_bits(xg @ w.T)", "q_bits = f64_to_bf16_bits(xg @ (w if w.shape[0] == w.shape[1] else w.T))"),
    "projection rounded through float32": ("q_bits = f64_to_bf16_bits(xg @ w.T)", "q_bits = f64_to_bf16_bits((xg @ w.T).astype(np.float32).astype(np.float64))"),
    "missing source reads the last token": ("        if token_idx[r] >= 0:\n            xg[r] = x[token_idx[r]]", "        xg[r] = x[token_idx[r]]"),
    "features split channel-major": (".reshape(rows, n_q_heads, d)", ".reshape(rows, d, n_q_heads).transpose(0, 2, 1)"),
    "rotation before the rounding of the projection": ("        q_bits = rope_apply(q_bits, positions, theta, pairing)", "        q_bits = f64_to_bf16_bits(rope_rotate((xg @ w.T).reshape(rows, n_q_heads, d), positions, theta, pairing))"),
    "queries rotated one position late": ("        q_bits = rope_apply(q_bits, positions, theta, pairing)", "        q_bits = rope_apply(q_bits, np.asarray(positions) + 1, theta, pairing)"),
    "decode step without the scale": ("    alpha = attention(q, k_cache, scale)\n    return alpha @", "    alpha = attention(q, k_cache, 1.0)\n    return alpha @"),
    "decode step with the query rows reversed": ("    alpha = attention(q, k_cache, scale)\n    return alpha @", "    alpha = attention(q[::-1], k_cache, scale)\n    return alpha @"),
}


def run_mutant(args):
    name, old, new, source, base = args
    d = os.path.join(base, "m%03d" % (abs(hash(name)) % 1000) + "_" + "".join(ch for ch in name if ch.isalnum())[:40])
    os.makedirs(os.path.join(d, "oracle"))
    open(os.path.join(d, "oracle", "__init__.py"), "w").close()
    with open(os.path.join(d, "oracle", "dapq_oracle.py"), "w") as f:
        f.write(source.replace(old, new, 1))
    env = dict(os.environ, PYTHONPATH=d + os.pathsep + ROOT, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1",
               MKL_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=d)
    return name, r.returncode, r.stdout[-1500:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    source = open(os.path.join(ROOT, "oracle", "dapq_oracle.py")).read()
    missing = [name for name, (old, _) in MUTANTS.items() if old not in source]
    assert not missing, f"mutants out of date with the oracle's source: {missing}"
    jobs = [(name, old, new, source, str(tmp_path)) for name, (old, new) in MUTANTS.items()]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        results = list(ex.map(run_mutant, jobs))
    survivors = [name for name, rc, _ in results if rc == 0]
    assert not survivors, f"no pin notices: {survivors}"
    # a mutant counts only if a pin failed (pytest exit status 1), not if the copy could not be imported or collected
    broken = [(name, rc, out) for name, rc, out in results if rc != 1]
    assert not broken, broken[:2]


def test_the_unmutated_copy_passes(tmp_path):
    """The harness itself: an unchanged copy in the same set-up passes every pin."""
    source = open(os.path.join(ROOT, "oracle", "dapq_oracle.py")).read()
    name, rc, out = run_mutant(("unchanged", "import numpy as np", "import numpy as np", source, str(tmp_path)))
    assert rc == 0, out
