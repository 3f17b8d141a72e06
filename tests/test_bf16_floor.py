"""How much of the bf16 tolerance the arithmetic itself uses up (CPU only).

north_star's "2e-2 relative" is met per tensor by every configuration.  The element-wise form of it used by
the GPU tests, |d| <= kappa (2e-2 |ref| + 2e-2 rms(row)), needs kappa > 1 on the one workload whose keys
are planted 4x larger (config 3): there a handful of large logits carry a row, and rounding the rotated
q and k to bf16, which no bf16 matrix-core kernel can avoid, already moves their probabilities by 1-2 %.
This file measures that floor with tests/floor_model.py on the first steady-state chunk of config 3 and of
config 2 and ties the tests' kappa to the measurement.

Figures (this test, seeded, deterministic; |d| / bound at kappa = 1):
  config 2, 96 rows x 4 heads:   worst 0.54, worst row L2 error 0.52 %
  config 3, 96 rows x 4 heads:   worst 1.92, worst row L2 error 2.1 %   (q, k rounding alone: 1.97; P alone 0.25;
                                 output alone 0.14; on 48 rows x 2 heads 1.66, 0.17, 0.13)
  config 3, all 4096 rows x all 32 query heads of the first steady-state chunk (16.8 M elements; run once by hand
                                 with the same functions, 110 s on 8 cores): worst per head 2.27 ... 4.13 (heads 31,
                                 17, 5, 14: 4.13, 3.95, 3.79, 3.66); about 400 of 4096 rows per head hold an element
                                 above 1, 4-13 rows one above 2; worst row L2 error 2.9 %
KAPPA_PLANTED_X4 = 5.25 is that whole-chunk floor (4.13) with a margin of 1.27 for what a kernel adds: float32
accumulation, a running maximum that is not the exact row maximum, hardware exp2.  The worst of N elements grows
with N (the sample of 49 K elements below reaches 1.92, one head's 524 K elements 2.3-4.1), so the floor that
counts is the one over as many elements as the GPU test compares: a whole chunk.  The GPU test
(tests/test_gpu_fullsize.py) in addition compares the kernel with this model directly at kappa = 1.
"""
import functools

import numpy as np

from paper_2410_01805_amd import synth
from tests.floor_model import floor_attention, ratio_to_unit_bound
from tests.gpu_util import KAPPA_PLANTED_X4, make_oracle

WHOLE_CHUNK_FLOOR_CFG3 = 4.13      # worst of 32 heads x 4096 rows, see above


@functools.lru_cache(maxsize=2)
def _steady_state(name):
    """(workload, oracle holding the cache at the budget, index of the first steady-state chunk); shared, read-only."""
    w = synth.WORKLOADS[name]
    W1, W2 = synth.weights(w)
    o = make_oracle(w, W1, W2)
    c = 0
    while o.n_c < w.b:
        q, k, v = synth.chunk(w, c)
        o.prefill_chunk(q, k, v, w.n_s, want_attn=False)
        c += 1
    return w, o, c


def _floor(name, n_rows, heads, **kw):
    w, o, c = _steady_state(name)
    q, k, v = synth.chunk(w, c)
    rows = np.sort(np.random.default_rng(1).choice(q.shape[0], n_rows, replace=False))
    ref = o.attention(q, k, v, rows=rows)
    fl = floor_attention(o, q, k, v, rows, heads, **kw)
    worst = max(float(ratio_to_unit_bound(fl[j], ref[rows, j, :]).max()) for j in heads)
    l2 = max(float((np.linalg.norm(fl[j] - ref[rows, j, :], axis=-1) / np.linalg.norm(ref[rows, j, :], axis=-1)).max())
             for j in heads)
    tensor = max(float(np.abs(fl[j] - ref[rows, j, :]).max() / np.abs(ref[rows, j, :]).max()) for j in heads)
    return worst, l2, tensor


def test_floor_of_unplanted_workload_is_inside_the_plain_bound():
    worst, l2, tensor = _floor("cfg2_llama_32k", 96, (0, 5, 17, 31))
    print(f"config 2 floor: worst |d|/bound {worst:.3f}, worst row L2 {l2:.4f}, tensor-wide {tensor:.4f}")
    assert worst < 0.75            # kappa = 1 leaves a kernel at least a quarter of the bound
    assert tensor < 1e-2


def test_floor_of_planted_workload_sets_kappa():
    worst, l2, tensor = _floor("cfg3_llama_128k", 96, (0, 5, 17, 31))
    print(f"config 3 floor: worst |d|/bound {worst:.3f}, worst row L2 {l2:.4f}, tensor-wide {tensor:.4f}")
    # the sample's floor is already above kappa = 1 ...
    assert 1.5 < worst < 2.5
    assert 1.5e-2 < l2 < 3e-2
    # ... the tensor-wide bar of 2e-2 is not in question ...
    assert tensor < 1e-2
    # ... and kappa is the whole-chunk floor times a margin between 1.2 and 1.5, no more
    assert worst < WHOLE_CHUNK_FLOOR_CFG3
    assert 1.2 * WHOLE_CHUNK_FLOOR_CFG3 <= KAPPA_PLANTED_X4 <= 1.5 * WHOLE_CHUNK_FLOOR_CFG3


def test_floor_comes_from_rounding_q_and_k():
    w, o, c = _steady_state("cfg3_llama_128k")
    q, k, v = synth.chunk(w, c)
    rows = np.sort(np.random.default_rng(1).choice(q.shape[0], 48, replace=False))
    ref = o.attention(q, k, v, rows=rows)
    heads = (5, 17)
    only = {}
    for what in ("round_qk", "round_p", "round_out"):
        kw = dict(round_qk=False, round_p=False, round_out=False)
        kw[what] = True
        fl = floor_attention(o, q, k, v, rows, heads, **kw)
        only[what] = max(float(ratio_to_unit_bound(fl[j], ref[rows, j, :]).max()) for j in heads)
    none = floor_attention(o, q, k, v, rows, heads, round_qk=False, round_p=False, round_out=False)
    for j in heads:                # with no rounding the model IS Eq. 1: it must reproduce the oracle
        np.testing.assert_allclose(none[j], ref[rows, j, :], rtol=1e-9, atol=1e-12)
    print("config 3 floor by source:", {k_: round(v_, 3) for k_, v_ in only.items()})
    assert only["round_qk"] > 4 * only["round_p"] and only["round_qk"] > 4 * only["round_out"]
    assert only["round_p"] < 0.5 and only["round_out"] < 0.5
