"""Brute-force definitions used only to pin the oracle (pure Python loops, math/cmath).

Nothing here is imported by the oracle or by the product; the formulations are
chosen to differ from the oracle's (scalar loops instead of matrix products,
complex multiplication instead of the cos/sin pair form, Python's sorted() on
tuples instead of lexsort, a closed form instead of a step-by-step simulation).
"""
from __future__ import annotations

import cmath
import math


def silu(z: float) -> float:
    return z / (1.0 + math.exp(-z))


def mlp_scores(q, k, v, W1, W2, g, expand):
    """Triple-loop retaining head (Section 3.3).  Returns list [T][h_kv]."""
    T, h, d = len(q), len(q[0]), len(q[0][0])
    h_kv = len(k[0])
    d_R = len(W1[0])
    out = []
    for t in range(T):
        x = [q[t][j][i] for j in range(h) for i in range(d)]
        if expand:
            x += [k[t][j // g][i] for j in range(h) for i in range(d)]
            x += [v[t][j // g][i] for j in range(h) for i in range(d)]
        else:
            x += [k[t][m][i] for m in range(h_kv) for i in range(d)]
            x += [v[t][m][i] for m in range(h_kv) for i in range(d)]
        hid = []
        for r in range(d_R):
            acc = 0.0
            for c, xc in enumerate(x):
                acc += xc * W1[c][r]
            hid.append(silu(acc))
        out.append([sum(hid[r] * W2[r][m] for r in range(d_R)) for m in range(h_kv)])
    return out


def rank_key(score: float, pos: int):
    """Sort key of the total order (score descending, position ascending; NaN last; zeros tie)."""
    if score != score:
        return (1, 0.0, pos)
    return (0, -score + 0.0, pos)


def closed_form_kept(scores, n_seen: int, b: int, n_s: int, n_pin: int = 0):
    """Kept original positions after n_seen tokens, for a constant stabilizer length:
    the most recent n_s tokens plus the best (b - n_s) of the earlier ones, taken over
    ALL earlier tokens (Appendix "Causal Importance Score Simulates a Cache Problem":
    a unit once evicted never returns, so the running top-b equals the global one).
    With a pinned prefix the first n_pin tokens of the stream are kept as well and the
    competition is among the tokens between them and the stabilizers."""
    ns = min(n_s, n_seen)
    npin = min(n_pin, n_seen - ns)
    n_keep = min(n_seen, b)
    cand = sorted(range(npin, n_seen - ns), key=lambda p: rank_key(float(scores[p]), p))
    return list(range(npin)) + sorted(cand[: n_keep - ns - npin]) + list(range(n_seen - ns, n_seen))


def simulate_algorithm1(scores, boundaries, b, n_s_per_chunk, n_pin: int = 0):
    """Literal list-based run of the cache loop of Algorithm 1 for one head: returns the kept
    original positions after every chunk.  The +inf mask is applied to a copy, the stored
    score stays the true one.  A pinned prefix is masked the same way at the front; where the two
    masks would overlap the stabilizers come first (the prefix only covers what they leave)."""
    cache = []  # list of (true_score, pos)
    hist = []
    start = 0
    for end, n_s in zip(boundaries, n_s_per_chunk):
        cache += [(float(scores[p]), p) for p in range(start, end)]
        L = len(cache)
        npin = min(n_pin, L - min(n_s, L))
        masked = [(math.inf if (i >= L - n_s or i < npin) else s, i) for i, (s, _) in enumerate(cache)]
        order = sorted(masked, key=lambda si: rank_key(si[0], si[1]))
        keep_slots = sorted(i for _, i in order[: min(L, b)])
        cache = [cache[i] for i in keep_slots]
        hist.append([p for _, p in cache])
        start = end
    return hist


def rope_complex(vec, pos: float, theta: float):
    d = len(vec)
    half = d // 2
    out = [0.0] * d
    for i in range(half):
        z = complex(vec[i], vec[i + half]) * cmath.exp(1j * pos * theta ** (-2.0 * i / d))
        out[i], out[i + half] = z.real, z.imag
    return out


def dense_masked_attention(q, k, v, boundaries, kept_before, g, rope, theta, scale=None):
    """Attention of every token of the stream under the eviction mask.

    q [N][h][d], k, v [N][h_kv][d] nested lists; boundaries = chunk end positions;
    kept_before[c][m] = sorted original positions retained for KV head m when chunk c starts.
    Query i of chunk c sees kept_before[c][m] and the chunk's tokens start..i.  With rope, a
    retained key takes its rank in kept_before as position, chunk token j takes
    len(kept) + (j - start), and so does the query.
    Returns out [N][h][d].
    """
    N, h, d = len(q), len(q[0]), len(q[0][0])
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = [[[0.0] * d for _ in range(h)] for _ in range(N)]
    start = 0
    for c, end in enumerate(boundaries):
        for i in range(start, end):
            for j in range(h):
                m = j // g
                kept = kept_before[c][m]
                vis = [(p, r) for r, p in enumerate(kept)] + \
                      [(p, len(kept) + (p - start)) for p in range(start, i + 1)]
                qi = q[i][j]
                if rope:
                    qi = rope_complex(qi, len(kept) + (i - start), theta)
                logits = []
                for p, posn in vis:
                    kp = k[p][m]
                    if rope:
                        kp = rope_complex(kp, posn, theta)
                    logits.append(scale * sum(a * bb for a, bb in zip(qi, kp)))
                mx = max(logits)
                w = [math.exp(x - mx) for x in logits]
                z = sum(w)
                for (p, _), wi in zip(vis, w):
                    vp = v[p][m]
                    for e in range(d):
                        out[i][j][e] += (wi / z) * vp[e]
        start = end
    return out
