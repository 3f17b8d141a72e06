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

  * Quantized cache rows (Appendix "Orthogonality to Other Methods", combination with 4-bit
    KV-cache quantization; the paper uses a third-party quantizer and gives no format).
    Reading: every K and V row is quantized when it enters the cache, per unit and per
    group of 32 consecutive head dims (a unit must stay self-contained, because units are
    evicted one by one): asymmetric 4-bit codes, code = round-half-even((x - lo) / s) clamped
    to 0..15 with lo = the group's minimum and s = (max - min) / 15 rounded to bfloat16
    (s = 1 for a constant group), decided in float32; value = lo + code * s.  K is quantized
    un-rotated.  Attention reads the cache, so it sees dequantized rows, the chunk's own
    included; the retaining head sees the raw q, k, v.

Parity pins (tests/test_oracle_*.py): brute-force dense masked attention written
with Python loops, a library SDPA for the never-evicting case, sliding-window
special case, closed-form kept sets, the two cache-problem conditions of
Appendix "Causal Importance Score Simulates a Cache Problem", a triple-loop MLP,
the bookkeeping numbers the paper prints (tests/golden/), and for head-wise budgets
the closed form and the brute force applied head by head; for the 4-bit rows hand-worked
groups with their packed bytes written out, the half-step round-trip bound, nearest-code
brute force, and the layer with quantized rows == the plain layer fed dequantized k, v
(tests/test_oracle_quant.py).
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
# 4-bit cache rows (Appendix "Orthogonality to Other Methods", quantization combination)
# ----------------------------------------------------------------------------

Q4_GROUP = 32       # consecutive head dims that share one (scale, minimum) pair


def _bf16_round(x32: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
    return r.view(np.float32)


def quantize_rows_q4(x: np.ndarray):
    """x [n][d] (values representable in bfloat16, d a multiple of 32) -> (codes uint8 [n][d] in 0..15,
    scale float32 [n][d/32] holding bfloat16 values, lo float32 [n][d/32]).
    Every step is float32, the precision in which the code is decided."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    n, d = x.shape
    assert d % Q4_GROUP == 0
    g = x.reshape(n, d // Q4_GROUP, Q4_GROUP)
    lo = g.min(axis=2)
    hi = g.max(axis=2)
    scale = _bf16_round((hi - lo) / np.float32(15.0))
    scale = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    t = (g - lo[:, :, None]) / scale[:, :, None]                  # float32 subtraction and division
    codes = np.clip(np.rint(t), 0, 15).astype(np.uint8)          # rint: ties to even
    return codes.reshape(n, d), scale, lo.astype(np.float32)


def dequantize_rows_q4(codes: np.ndarray, scale: np.ndarray, lo: np.ndarray) -> np.ndarray:
    """value = lo + code * scale, exactly (float64)."""
    n, d = codes.shape
    c = codes.reshape(n, d // Q4_GROUP, Q4_GROUP).astype(np.float64)
    return (lo.astype(np.float64)[:, :, None] + c * scale.astype(np.float64)[:, :, None]).reshape(n, d)


def pack_rows_q4(codes: np.ndarray, scale: np.ndarray, lo: np.ndarray) -> np.ndarray:
    """Storage form of the rows, uint8 [n][d/2 + 4 d/32]: first the codes, two per byte (dim 2i in the low
    nibble, dim 2i+1 in the high one), then per group the scale and the minimum as little-endian bfloat16."""
    n, d = codes.shape
    nib = codes.reshape(n, d // 2, 2)
    body = (nib[:, :, 0] | (nib[:, :, 1] << 4)).astype(np.uint8)
    par = np.stack([scale, lo], axis=2).astype(np.float32)       # [n][groups][2]
    bits = (par.view(np.uint32) >> np.uint32(16)).astype(np.uint16)   # both are bfloat16 values: the low half is zero
    assert np.array_equal((bits.astype(np.uint32) << np.uint32(16)).view(np.float32), par), "scale/min not bfloat16"
    tail = np.ascontiguousarray(bits.reshape(n, -1)).astype("<u2").view(np.uint8).reshape(n, -1)
    return np.concatenate([body, tail], axis=1)


def q4_roundtrip(x: np.ndarray):
    """(dequantized rows float64 [n][d], packed rows uint8) of x [n][d]."""
    codes, scale, lo = quantize_rows_q4(x)
    return dequantize_rows_q4(codes, scale, lo), pack_rows_q4(codes, scale, lo)


# ----------------------------------------------------------------------------
# one layer's state and the chunk step
# ----------------------------------------------------------------------------

class LocretLayerOracle:
    """State = per-KV-head K, V (un-rotated), true scores and original token positions.

    budget: one int for every KV head, or a sequence of h_kv ints (head-wise budgets).
    kv_bits: 0 = rows kept as given; 4 = rows quantized to 4 bits when they enter the cache (K, V then hold the
    dequantized values and Kq, Vq the packed rows)."""

    def __init__(self, h: int, h_kv: int, d: int, budget: int, W1, W2, rh_kv_expand: int = 0,
                 rope: bool = False, theta: float = 10000.0, scale: float | None = None, n_pin: int = 0,
                 kv_bits: int = 0):
        assert h % h_kv == 0
        assert kv_bits in (0, 4)
        self.kv_bits = kv_bits
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
        row_bytes = self.d // 2 + 4 * (self.d // Q4_GROUP)
        self.Kq = [np.zeros((0, row_bytes), dtype=np.uint8) for _ in range(self.h_kv)]
        self.Vq = [np.zeros((0, row_bytes), dtype=np.uint8) for _ in range(self.h_kv)]
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
        if self.kv_bits:
            # attention reads the cache: the chunk's own rows are seen as they are stored
            k = np.stack([q4_roundtrip(k[:, m, :])[0] for m in range(self.h_kv)], axis=1)
            v = np.stack([q4_roundtrip(v[:, m, :])[0] for m in range(self.h_kv)], axis=1)
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
            km, vm = k[:, m, :], v[:, m, :]
            if self.kv_bits:
                km, kq = q4_roundtrip(km)
                vm, vq = q4_roundtrip(vm)
                Kqc = np.concatenate([self.Kq[m], kq], axis=0)
                Vqc = np.concatenate([self.Vq[m], vq], axis=0)
            Kc = np.concatenate([self.K[m], km], axis=0)
            Vc = np.concatenate([self.V[m], vm], axis=0)
            Sc = np.concatenate([self.S[m], scores[m]])
            Pc = np.concatenate([self.P[m], self.seen + np.arange(T, dtype=np.int64)])
            if evict:
                idx = select_keep(Sc, self.budgets[m], n_stab, self.n_pin)
            else:
                idx = np.arange(Sc.shape[0], dtype=np.int64)
            self.K[m], self.V[m], self.S[m], self.P[m] = Kc[idx], Vc[idx], Sc[idx], Pc[idx]
            if self.kv_bits:
                self.Kq[m], self.Vq[m] = Kqc[idx], Vqc[idx]
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
