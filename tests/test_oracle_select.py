"""Pins for the oracle's stabilizer-masked top-b and the cache loop (Section 3.4, Algorithm 1,
Appendix "Causal Importance Score Simulates a Cache Problem")."""
import math
import os

import numpy as np
import pytest

from oracle.locret_oracle import LocretLayerOracle, select_keep
from tests import bruteforce as bf

INF, NAN = math.inf, math.nan


# ---- hand-worked cases: expected values written out by hand, not computed -----------------------
HAND = [
    # scores, budget, n_stab, expected kept indices
    ([1, 5, 3, 2, 4], 3, 0, [1, 2, 4]),                    # plain top-3, order preserved
    ([1, 5, 3, 2, 4], 3, 2, [1, 3, 4]),                    # last two forced, best of the first three
    ([1, 5, 3, 2, 4], 3, 3, [2, 3, 4]),                    # n_s = b: sliding window
    ([1, 5, 3], 8, 1, [0, 1, 2]),                          # L < b keeps everything
    ([7, 7, 7, 7, 7], 2, 0, [0, 1]),                       # all equal: lowest indices win
    ([7, 7, 7, 7, 7], 3, 1, [0, 1, 4]),
    ([2, 9, 2, 9, 2, 9, 2], 4, 0, [0, 1, 3, 5]),           # duplicates straddle the threshold
    ([0.0, -0.0, -0.0, 0.0, -1], 2, 0, [0, 1]),            # -0 ties +0: index decides
    ([-0.0, 0.0, 1.0], 2, 0, [0, 2]),
    ([-INF, INF, 0, -INF, INF], 3, 0, [1, 2, 4]),          # infinities ordered as values
    ([-INF, NAN, -INF, 1], 3, 0, [0, 2, 3]),               # NaN below -inf
    ([NAN, NAN, NAN, 1], 3, 0, [0, 1, 3]),                 # among NaNs the lower index wins
    ([NAN, 3, NAN, 1], 2, 1, [1, 3]),                      # NaN never beats a number
    ([5, 4, 3, 2, 1], 2, 2, [3, 4]),                       # stabilizers take the whole budget
    ([], 4, 2, []),
    ([3], 1, 0, [0]),
]


@pytest.mark.parametrize("scores,b,ns,want", HAND)
def test_select_hand_cases(scores, b, ns, want):
    got = select_keep(np.array(scores, dtype=np.float32), b, ns)
    assert got.tolist() == want


def test_select_rejects_stabilizers_over_budget():
    with pytest.raises(ValueError):
        select_keep(np.arange(10, dtype=np.float32), 3, 4)


def test_select_vs_sorted_bruteforce():
    rng = np.random.default_rng(11)
    for trial in range(300):
        L = int(rng.integers(1, 80))
        b = int(rng.integers(1, 90))
        ns = int(rng.integers(0, b + 1))
        # few distinct values -> many ties; sprinkle specials
        s = rng.integers(-3, 4, size=L).astype(np.float32) * 0.5
        for special in (np.nan, np.inf, -np.inf, -0.0):
            if rng.random() < 0.3:
                s[rng.integers(0, L)] = special
        got = select_keep(s, b, ns).tolist()
        nsp = min(ns, L)
        n_keep = min(L, b)
        cand = sorted(range(L - nsp), key=lambda i: bf.rank_key(float(s[i]), i))
        want = sorted(cand[: n_keep - nsp]) + list(range(L - nsp, L))
        assert got == want, (trial, s, b, ns)


# ---- cache loop: step-by-step oracle vs closed form vs literal list simulation ----------------------
def _run_scores_only(scores, B, b, n_s, last_chunk_unmasked=False):
    """Drive the oracle's cache loop with given per-token scores (one head, d = 1)."""
    N = len(scores)
    o = LocretLayerOracle(1, 1, 1, b, np.zeros((3, 1)), np.zeros((1, 1)))
    hist, kept_hist, bounds, ns_list = [], [], [], []
    for lo in range(0, N, B):
        hi = min(N, lo + B)
        T = hi - lo
        ns = 0 if (last_chunk_unmasked and hi == N) else n_s
        kv = np.arange(lo, hi, dtype=np.float64).reshape(T, 1, 1)
        kept = o.evict_compact(scores[None, lo:hi], kv, -kv, ns)
        hist.append(o.P[0].tolist())
        kept_hist.append(kept[0].tolist())
        bounds.append(hi)
        ns_list.append(ns)
        # K, V, S travel with the unit
        assert o.K[0][:, 0].tolist() == o.P[0].tolist()
        assert (o.V[0][:, 0] == -o.K[0][:, 0]).all()
        np.testing.assert_array_equal(o.S[0], scores[o.P[0]])
    return hist, kept_hist, bounds, ns_list


PARAMS = [
    # N, B, b, n_s
    (200, 16, 40, 8),
    (200, 16, 40, 0),      # no stabilizers (multi-turn setting, Appendix "multi-turn")
    (203, 16, 40, 24),     # n_s > B and a ragged last chunk (the GQA backbone's row has n_s > B)
    (150, 32, 32, 32),     # n_s = b: pure sliding window
    (97, 10, 25, 3),
    (64, 64, 100, 5),      # single chunk below the budget
    (300, 7, 21, 20),
]


@pytest.mark.parametrize("N,B,b,n_s", PARAMS)
@pytest.mark.parametrize("ties", [False, True])
def test_cache_loop_matches_closed_form_and_invariants(N, B, b, n_s, ties):
    rng = np.random.default_rng(N * 7 + B)
    scores = rng.standard_normal(N).astype(np.float32)
    if ties:
        scores = np.round(scores * 2) / 2      # heavy duplication
    hist, kept_hist, bounds, ns_list = _run_scores_only(scores, B, b, n_s)
    sim = bf.simulate_algorithm1(scores, bounds, b, ns_list)
    prev = []
    prev_end = 0
    for c, end in enumerate(bounds):
        got = hist[c]
        assert got == bf.closed_form_kept(scores, end, b, n_s)
        assert got == sim[c]
        # invariants
        assert len(got) == min(end, b)                                   # |Sel| <= b, cache stays full
        assert all(x < y for x, y in zip(got, got[1:]))                  # order preserved
        nsp = min(n_s, len(got))
        assert got[len(got) - nsp:] == list(range(end - nsp, end))       # stabilizers = most recent tokens
        assert set(got) - set(prev) <= set(range(prev_end, end))         # an evicted unit never returns
        # kept_idx is in the concatenated index space [old cache ; chunk]
        cat = prev + list(range(prev_end, end))
        assert [cat[i] for i in kept_hist[c]] == got
        prev, prev_end = got, end
    if n_s == 0:
        top = sorted(range(N), key=lambda p: bf.rank_key(float(scores[p]), p))[: min(N, b)]
        assert hist[-1] == sorted(top)


def test_last_chunk_without_mask_as_in_algorithm1():
    rng = np.random.default_rng(5)
    scores = rng.standard_normal(120).astype(np.float32)
    hist, _, bounds, ns_list = _run_scores_only(scores, 16, 30, 6, last_chunk_unmasked=True)
    assert ns_list[-1] == 0 and ns_list[0] == 6
    assert hist == bf.simulate_algorithm1(scores, bounds, 30, ns_list)


def test_heads_evict_independently():
    rng = np.random.default_rng(9)
    h_kv, N, B, b, n_s = 3, 90, 12, 20, 4
    scores = rng.standard_normal((h_kv, N)).astype(np.float32)
    o = LocretLayerOracle(3, 3, 1, b, np.zeros((9, 1)), np.zeros((1, 3)))
    for lo in range(0, N, B):
        hi = min(N, lo + B)
        kv = np.zeros((hi - lo, h_kv, 1))
        o.evict_compact(scores[:, lo:hi], kv, kv, n_s)
    for m in range(h_kv):
        assert o.P[m].tolist() == bf.closed_form_kept(scores[m], N, b, n_s)


# ---- head-wise budgets (Appendix "Orthogonality to Other Methods": heads evict independently, so each
# may have a budget of its own) ----------------------------------------------------------------------
@pytest.mark.parametrize("budgets,n_s,n_pin", [
    ([20, 7, 33], 4, 0),
    ([12, 40, 12, 25], 12, 0),       # n_s equals the smallest budget: that head is a sliding window
    ([200, 9, 30], 3, 0),            # one head never fills its budget
    ([18, 9, 30], 3, 5),             # with a pinned prefix
])
def test_head_wise_budgets_match_closed_form_per_head(budgets, n_s, n_pin):
    rng = np.random.default_rng(sum(budgets))
    h_kv, N, B = len(budgets), 110, 12
    scores = np.round(rng.standard_normal((h_kv, N)).astype(np.float32) * 2) / 2
    o = LocretLayerOracle(h_kv, h_kv, 1, budgets, np.zeros((3 * h_kv, 1)), np.zeros((1, h_kv)), n_pin=n_pin)
    prev = [[] for _ in range(h_kv)]
    for lo in range(0, N, B):
        hi = min(N, lo + B)
        kv = np.arange(lo, hi, dtype=np.float64)[:, None, None] * np.ones((1, h_kv, 1))
        kept = o.evict_compact(scores[:, lo:hi], kv, -kv, n_s)
        for m in range(h_kv):
            want = bf.closed_form_kept(scores[m], hi, budgets[m], n_s, n_pin)
            assert o.P[m].tolist() == want
            assert len(want) == min(hi, budgets[m])                     # every head within its own budget
            cat = prev[m] + list(range(lo, hi))
            assert [cat[i] for i in kept[m]] == want                    # indices in the head's own space
            assert o.K[m][:, 0].tolist() == want and (o.V[m] == -o.K[m]).all()
            np.testing.assert_array_equal(o.S[m], scores[m][want])
            prev[m] = want
    assert o.n_c == min(N, max(budgets)) and [o.n_c_of(m) for m in range(h_kv)] == [min(N, b) for b in budgets]


def test_equal_head_budgets_are_the_single_budget():
    rng = np.random.default_rng(3)
    scores = rng.standard_normal((2, 60)).astype(np.float32)
    a = LocretLayerOracle(2, 2, 1, 14, np.zeros((6, 1)), np.zeros((1, 2)))
    b = LocretLayerOracle(2, 2, 1, [14, 14], np.zeros((6, 1)), np.zeros((1, 2)))
    for lo in range(0, 60, 10):
        kv = np.zeros((10, 2, 1))
        ka = a.evict_compact(scores[:, lo:lo + 10], kv, kv, 3)
        kb = b.evict_compact(scores[:, lo:lo + 10], kv, kv, 3)
        np.testing.assert_array_equal(ka, kb)


# ---- pinned prefix (Locret-Q: the query sits at the start of the sequence and is never evicted) -------
PIN_HAND = [
    # scores, budget, n_stab, n_pin, expected kept indices (written out by hand)
    ([1, 5, 3, 2, 4], 3, 0, 1, [0, 1, 4]),                 # slot 0 forced although it scores lowest
    ([1, 5, 3, 2, 4], 3, 1, 1, [0, 1, 4]),                 # first and last forced, best of the middle
    ([1, 5, 3, 2, 4], 3, 1, 2, [0, 1, 4]),                 # prefix + stabilizer fill the budget
    ([1, 2, 9, 8, 7, 3], 4, 1, 2, [0, 1, 2, 5]),
    ([9, 9, 9], 8, 0, 2, [0, 1, 2]),                       # L < b keeps everything
    ([1, 2], 5, 2, 3, [0, 1]),                             # stabilizers cover the list: nothing left to pin
    ([4, 4, 4, 4, 4, 4], 4, 1, 1, [0, 1, 2, 5]),           # ties in the middle: lowest index
    ([NAN, 1, 2, 3], 2, 0, 1, [0, 3]),                     # a pinned unit is kept whatever its score
]


@pytest.mark.parametrize("scores,b,ns,npin,want", PIN_HAND)
def test_select_pinned_prefix_hand_cases(scores, b, ns, npin, want):
    assert select_keep(np.array(scores, dtype=np.float32), b, ns, npin).tolist() == want


def test_select_pinned_prefix_rejects_overfull_budget():
    with pytest.raises(ValueError):
        select_keep(np.arange(10, dtype=np.float32), 4, 2, 3)
    assert select_keep(np.arange(10, dtype=np.float32), 5, 2, 3).tolist() == [0, 1, 2, 8, 9]


def test_select_pinned_prefix_vs_sorted_bruteforce():
    rng = np.random.default_rng(23)
    for trial in range(300):
        L = int(rng.integers(1, 80))
        b = int(rng.integers(1, 90))
        ns = int(rng.integers(0, b + 1))
        npin = int(rng.integers(0, b - ns + 1))
        s = rng.integers(-3, 4, size=L).astype(np.float32) * 0.5
        for special in (np.nan, np.inf, -np.inf, -0.0):
            if rng.random() < 0.3:
                s[rng.integers(0, L)] = special
        got = select_keep(s, b, ns, npin).tolist()
        nsp = min(ns, L)
        npp = min(npin, L - nsp)
        n_keep = min(L, b)
        cand = sorted(range(npp, L - nsp), key=lambda i: bf.rank_key(float(s[i]), i))
        want = list(range(npp)) + sorted(cand[: n_keep - nsp - npp]) + list(range(L - nsp, L))
        assert got == want, (trial, s, b, ns, npin)
        assert select_keep(s, b, ns, 0).tolist() == select_keep(s, b, ns).tolist()


@pytest.mark.parametrize("N,B,b,n_s,n_pin", [(200, 16, 40, 8, 5), (203, 16, 40, 24, 16), (150, 7, 21, 0, 21),
                                            (120, 32, 33, 3, 30), (90, 10, 25, 5, 1)])
@pytest.mark.parametrize("ties", [False, True])
def test_cache_loop_with_pinned_prefix_matches_closed_form_and_simulation(N, B, b, n_s, n_pin, ties):
    rng = np.random.default_rng(N + 13 * n_pin)
    scores = rng.standard_normal(N).astype(np.float32)
    scores[:n_pin] = -50.0                     # the pinned tokens would be the first to go on their merits
    if ties:
        scores = np.round(scores * 2) / 2
    o = LocretLayerOracle(1, 1, 1, b, np.zeros((3, 1)), np.zeros((1, 1)), n_pin=n_pin)
    bounds, hist = [], []
    for lo in range(0, N, B):
        hi = min(N, lo + B)
        kv = np.arange(lo, hi, dtype=np.float64).reshape(hi - lo, 1, 1)
        o.evict_compact(scores[None, lo:hi], kv, -kv, n_s)
        bounds.append(hi)
        hist.append(o.P[0].tolist())
        np.testing.assert_array_equal(o.S[0], scores[o.P[0]])            # true scores stored, not a mask value
    sim = bf.simulate_algorithm1(scores, bounds, b, [n_s] * len(bounds), n_pin)
    for c, end in enumerate(bounds):
        assert hist[c] == sim[c]
        assert hist[c] == bf.closed_form_kept(scores, end, b, n_s, n_pin)
        npp = min(n_pin, end - min(n_s, end))
        assert hist[c][:npp] == list(range(npp))                          # the prefix stays at the front


# ---- numbers the paper prints --------------------------------------------------------------------
def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_bookkeeping.txt")
    rows = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, N, b, val, _ = [x.strip() for x in line.split("|")]
        rows[name] = (int(N), int(b), float(val))
    return rows


def test_printed_compression_ratios():
    g = _golden()
    # 10M-token run: drive the real cache loop at the paper's (b, B, n_s) on scores only
    N, b, want = g["ratio_10m"]
    B, n_s = 10240, 2500
    rng = np.random.default_rng(1)
    o = LocretLayerOracle(1, 1, 1, b, np.zeros((3, 1)), np.zeros((1, 1)))
    step = 64                                   # every 64th chunk of the stream is enough to fill and churn
    kv = np.zeros((B, 1, 1))
    for c in range(0, N // B, step):
        o.evict_compact(rng.standard_normal((1, B)).astype(np.float32), kv, kv, n_s)
        assert o.n_c == min(b, o.seen)
    assert round(N / o.n_c, 1) == want
    N, b, want = g["ratio_llama"]
    assert N / min(N, b) == want
    N, b, want = g["ratio_phi3"]
    assert N / min(N, b) > want
    N, _, want = g["kv_full_gib"]
    assert 32 * 32 * 96 * 2 * 2 * N / 2 ** 30 == want
