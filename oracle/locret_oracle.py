"""CPU oracle for the Locret per-layer chunked-prefill step with learned KV eviction.

TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute;
it is deliberately plain and slow (numpy, float64, no blocking, no fusion).  Only
tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import it.
It shares no code with the HIP path and never imports the product package.

One chunk step, in the order of the paper's inference pseudocode (Appendix A.2,
Algorithm 1) for a single attention layer:

  1. attention of the chunk's queries over [retained cache ; chunk]     (Section 3.1, Eq. 1)
  2. retaining head R([Q,K,V]) = act([Q,K,V] W1) W2, one score per KV head (Section 3.3)
  3. concatenate chunk K, V, scores to the cache                          (Algorithm 1)
  4. force-keep the last n_s entries, keep the top scores up to budget b  (Section 3.4, Algorithm 1)
  5. gather the kept units, order preserved, into the cache               (Algorithm 1)

Readings taken where the paper leaves a choice (each is restated where used):
  * softmax scale is 1/sqrt(head_dim); query head j uses KV head floor(j/g) (0-based).
  * The retaining head has no bias and uses SiLU (the backbones' activation, Appendix A.1).
  * The retaining head sees q, k, v before any rotary embedding, so that a score,
    once computed, does not depend on the position a unit later occupies (Section 3.4).
  * K is cached un-rotated; at every step cache slot i takes position i and chunk
    token t takes position n_c + t (Section 3.4: positions are handed out anew,
    contiguously from zero, at every step); rotate-half pairing (i, i + d/2),
    inverse frequency theta^(-2i/d).
  * The +infinity written on the stabilizers is a selection-time mask: the cache
    keeps each unit's true score.
  * The kept units stay in their original order (indices ascending).
  * Total order for selection: score descending, then index ascending; -0 == +0;
    NaN ranks below every number, -inf included.
  * Scores are stored, and the selection is decided, in float32.
  * Head-wise budgets (Appendix "Orthogonality to Other Methods", head-wise budget
    allocation): KV heads evict independently, so each may have a budget of its own;
    the caches of the heads then differ in length, and a head's positions are counted
    within its own cache (slot i of head m sits at position i, chunk token t at
    n_c[m] + t).

Parity pins (tests/test_oracle_*.py): brute-force dense masked attention written
with Python loops, a library SDPA for the never-evicting case, sliding-window
special case, closed-form kept sets, the two cache-problem conditions of
Appendix "Causal Importance Score Simulates a Cache Problem", a triple-loop MLP,
the bookkeeping numbers the paper prints (tests/golden/), and for head-wise budgets
the closed form and the brute force applied head by head.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------
# rotary position embedding (Section 3.4: positions reassigned from 0 each step)
# ----------------------------------------------------------------------------

def rope_rotate(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate x[n, d] (float64) so that row r sits at position pos[r].

    Pair (i, i + d/2) is rotated by angle pos * theta^(-2i/d).
    """
    n, d = x.shape
    half = d // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[:, :half], x[:, half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=1)


# ----------------------------------------------------------------------------
# retaining head (Section 3.3)
# ----------------------------------------------------------------------------

def retaining_head(q, k, v, W1, W2, rh_kv_expand: int = 0) -> np.ndarray:
    """Scores S~[t, m] = SiLU([q_t ; k_t ; v_t] W1) W2  for T tokens.

    q [T][h][d], k, v [T][h_kv][d] (un-rotated); W1 [d_in][d_R]; W2 [d_R][h_kv].
    rh_kv_expand = 0: the input is (h + 2 h_kv) d wide, as the paper's W1 shape states.
    rh_kv_expand = 1: the K and V blocks are repeated g times in query-head order
    (query head j reads KV head floor(j/g)), giving 3 h d.
    Returns float64 [T][h_kv].
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T, h, d = q.shape
    h_kv = k.shape[1]
    g = h // h_kv
    if rh_kv_expand:
        k = np.repeat(k, g, axis=1)
        v = np.repeat(v, g, axis=1)
    x = np.concatenate([q.reshape(T, -1), k.reshape(T, -1), v.reshape(T, -1)], axis=1)
    z = x @ np.asarray(W1, dtype=np.float64)
    a = z / (1.0 + np.exp(-z))
    return a @ np.asarray(W2, dtype=np.float64)


# ----------------------------------------------------------------------------
# stabilizer mask + top-b (Section 3.4, Algorithm 1)
# ----------------------------------------------------------------------------

def select_keep(scores: np.ndarray, budget: int, n_stab: int, n_pin: int = 0) -> np.ndarray:
    """Indices (ascending) of the units kept out of the L concatenated scores of one KV head.

    The last min(n_stab, L) entries are always kept; so are the first n_pin of the others (the
    query tokens that Locret-Q puts at the start of the sequence so that every eviction sees them,
    Section "Supporting Query-Driven Tasks"); the rest of the budget goes to the best of the
    remaining ones under (score descending, index ascending).
    """
    s = np.asarray(scores, dtype=np.float32)
    L = s.shape[0]
    n_keep = min(L, budget)
    ns = min(n_stab, L)
    npin = min(n_pin, L - ns)
    if ns + npin > n_keep:
        raise ValueError("stabilizers and pinned prefix exceed the budget")
    n_cand = L - ns - npin
    cand = s[npin:npin + n_cand].astype(np.float64)
    isnan = np.isnan(cand)
    neg = np.where(isnan, 0.0, -cand) + 0.0          # -0.0 + 0.0 = +0.0: the two zeros tie
    # lexsort: last key is the primary one.  NaN after all numbers, then larger score first,
    # then lower index first.
    order = np.lexsort((np.arange(n_cand), neg, isnan.astype(np.int8)))
    top = order[: n_keep - ns - npin] + npin
    kept = np.concatenate([np.arange(npin), np.sort(top), np.arange(npin + n_cand, L)])
    return kept.astype(np.int64)


# ----------------------------------------------------------------------------
# one layer's state and the chunk step
# ----------------------------------------------------------------------------

class LocretLayerOracle:
    """State = per-KV-head K, V (un-rotated), true scores and original token positions.

    budget: one int for every KV head, or a sequence of h_kv ints (head-wise budgets)."""

    def __init__(self, h: int, h_kv: int, d: int, budget: int, W1, W2, rh_kv_expand: int = 0,
                 rope: bool = False, theta: float = 10000.0, scale: float | None = None, n_pin: int = 0):
        assert h % h_kv == 0
        self.n_pin = n_pin          # units at the start of the cache that are never evicted (Locret-Q)
        self.h, self.h_kv, self.d, self.g = h, h_kv, d, h // h_kv
        self.budgets = [int(budget)] * h_kv if np.ndim(budget) == 0 else [int(x) for x in budget]
        assert len(self.budgets) == h_kv
        self.budget = max(self.budgets)
        self.W1 = np.asarray(W1, dtype=np.float64)
        self.W2 = np.asarray(W2, dtype=np.float64)
        self.rh_kv_expand = rh_kv_expand
        self.rope, self.theta = rope, theta
        self.scale = (1.0 / np.sqrt(d)) if scale is None else scale
        self.reset()

    def reset(self):
        z = lambda *s: np.zeros(s, dtype=np.float64)
        self.K = [z(0, self.d) for _ in range(self.h_kv)]
        self.V = [z(0, self.d) for _ in range(self.h_kv)]
        self.S = [np.zeros(0, dtype=np.float32) for _ in range(self.h_kv)]
        self.P = [np.zeros(0, dtype=np.int64) for _ in range(self.h_kv)]
        self.seen = 0

    @property
    def n_c(self) -> int:
        """Cache length (with head-wise budgets: of the longest head)."""
        return max(self.K[m].shape[0] for m in range(self.h_kv))

    def n_c_of(self, m: int) -> int:
        return self.K[m].shape[0]

    # -- step 1: Eq. 1 over [cache ; chunk], causal inside the chunk ---------------------------
    def attention(self, q, k, v, rows=None) -> np.ndarray:
        """out[t][j] for the chunk's queries.  rows: optional list of query rows t to compute
        (the others are returned as NaN); rows are independent of each other."""
        q = np.asarray(q, dtype=np.float64)
        k = np.asarray(k, dtype=np.float64)
        v = np.asarray(v, dtype=np.float64)
        T = q.shape[0]
        out = np.full((T, self.h, self.d), np.nan)
        ts = np.arange(T) if rows is None else np.asarray(rows)
        for j in range(self.h):
            m = j // self.g
            n_c = self.n_c_of(m)
            keys = np.concatenate([self.K[m], k[:, m, :]], axis=0)       # [n_c + T][d]
            vals = np.concatenate([self.V[m], v[:, m, :]], axis=0)
            qj = q[ts, j, :]
            if self.rope:
                keys = rope_rotate(keys, np.arange(n_c + T), self.theta)
                qj = rope_rotate(qj, n_c + ts, self.theta)
            logits = (qj @ keys.T) * self.scale                          # [len(ts)][n_c + T]
            visible = np.arange(n_c + T)[None, :] <= (n_c + ts)[:, None]
            logits = np.where(visible, logits, -np.inf)
            logits -= logits.max(axis=1, keepdims=True)
            p = np.exp(logits)
            p /= p.sum(axis=1, keepdims=True)
            out[ts, j, :] = p @ vals
        return out

    # -- step 2 -------------------------------------------------------------------------------
    def score(self, q, k, v) -> np.ndarray:
        """float32 [h_kv][T] (the storage precision of scores)."""
        return np.ascontiguousarray(retaining_head(q, k, v, self.W1, self.W2, self.rh_kv_expand).T, dtype=np.float32)

    # -- steps 3-5 ----------------------------------------------------------------------------
    def evict_compact(self, scores, k, v, n_stab: int, evict: bool = True) -> np.ndarray:
        """Append the chunk (scores [h_kv][T] float32) and reduce to the budget.
        Returns kept indices [h_kv][n_keep] in the concatenated index space (a list of h_kv arrays
        when head-wise budgets make the rows differ in length)."""
        k = np.asarray(k, dtype=np.float64)
        v = np.asarray(v, dtype=np.float64)
        scores = np.asarray(scores, dtype=np.float32)
        T = k.shape[0]
        kept_all = []
        for m in range(self.h_kv):
            Kc = np.concatenate([self.K[m], k[:, m, :]], axis=0)
            Vc = np.concatenate([self.V[m], v[:, m, :]], axis=0)
            Sc = np.concatenate([self.S[m], scores[m]])
            Pc = np.concatenate([self.P[m], self.seen + np.arange(T, dtype=np.int64)])
            if evict:
                idx = select_keep(Sc, self.budgets[m], n_stab, self.n_pin)
            else:
                idx = np.arange(Sc.shape[0], dtype=np.int64)
            self.K[m], self.V[m], self.S[m], self.P[m] = Kc[idx], Vc[idx], Sc[idx], Pc[idx]
            kept_all.append(idx)
        self.seen += T
        if len({len(x) for x in kept_all}) > 1:
            return kept_all
        return np.stack(kept_all)

    # -- the whole step -----------------------------------------------------------------------
    def prefill_chunk(self, q, k, v, n_stab: int, evict: bool = True, scores_in=None,
                      attn_rows=None, want_attn: bool = True):
        """Returns (attn_out [T][h][d] float64, scores [h_kv][T] float32, kept_idx [h_kv][n_keep]).
        scores_in, if given, replaces the retaining head's scores in the selection."""
        out = self.attention(q, k, v, rows=attn_rows) if want_attn else None
        sc = self.score(q, k, v)
        kept = self.evict_compact(sc if scores_in is None else scores_in, k, v, n_stab, evict)
        return out, sc, kept
