"""Pure-Python brute force used to pin the C oracle on tiny inputs.

Written directly from the definitions (Eq. 1, 2, 3/6, 4, 5 of the paper) with
lists of Python floats and math.fsum; it shares nothing with oracle/ and is far
too slow for anything but a few hundred tokens.
"""
import math


def tokens_of(seq_len, S, pages):
    """Logical token positions covered by the given logical pages, page by page."""
    out = []
    for p in pages:
        out.extend(range(p * S, min((p + 1) * S, seq_len)))
    return out


def key_rows(k_cache, page_table_row, S, hkv, toks):
    """k_cache: nested [phys][Hkv][S][D] floats -> list of D-vectors for logical tokens."""
    return [[float(x) for x in k_cache[page_table_row[t // S]][hkv][t % S]] for t in toks]


def page_mean_std(rows):
    n, D = len(rows), len(rows[0])
    mean = [math.fsum(r[d] for r in rows) / n for d in range(D)]
    per_dim_std = [math.sqrt(math.fsum((r[d] - mean[d]) ** 2 for r in rows) / n) for d in range(D)]
    return mean, math.sqrt(math.fsum(s * s for s in per_dim_std))


def page_score(q_group, mean, std, lam):
    vals = []
    for q in q_group:
        dot = math.fsum(a * b for a, b in zip(q, mean))
        vals.append(dot + lam * math.sqrt(math.fsum(a * a for a in q)) * std)
    return max(vals)


def topk_set(scores, k):
    order = sorted(range(len(scores)), key=lambda p: (-scores[p], p))
    return order[:min(k, len(scores))]


def softmax_attention(q, krows, vrows, scale):
    logits = [scale * math.fsum(a * b for a, b in zip(q, kr)) for kr in krows]
    m = max(logits)
    w = [math.exp(l - m) for l in logits]
    z = math.fsum(w)
    D = len(vrows[0])
    out = [math.fsum(w[t] * vrows[t][d] for t in range(len(vrows))) / z for d in range(D)]
    return out, m + math.log(z)
