"""GPU parity of the decode step (locret_decode_step: Eq. 1 with B = 1 on the retained cache)
against the oracle, which runs the same token through its general chunk step with T = 1 and no
eviction.  A teacher-forced prefill stream first brings both caches to the same state."""
import numpy as np
import pytest
import torch

from paper_2410_01805_amd import synth
from tests.gpu_util import DEV, assert_close, dev, host, kappa_for, make_layer, make_oracle
from tests.test_gpu_prefill import _run_stream

pytestmark = pytest.mark.gpu

N_DEC = 7

CASES = [
    dict(name="dec_f32_gqa", dtype="f32", h=8, h_kv=2, d=64, N=1000, B=200, b=400, n_s=32, d_R=64, rope=False),
    dict(name="dec_f32_rope_d32", dtype="f32", h=4, h_kv=2, d=32, N=800, B=160, b=300, n_s=40, d_R=64, rope=True),
    dict(name="dec_f32_mha_d16", dtype="f32", h=3, h_kv=3, d=16, N=500, B=100, b=150, n_s=0, d_R=40, rope=True),
    dict(name="dec_f32_d128", dtype="f32", h=4, h_kv=2, d=128, N=700, B=128, b=333, n_s=10, d_R=64, rope=True),
    dict(name="dec_bf16_llama_like", dtype="bf16", h=8, h_kv=2, d=128, N=1500, B=300, b=700, n_s=100, d_R=128,
         theta=500000.0),
    dict(name="dec_bf16_phi_like", dtype="bf16", h=4, h_kv=4, d=96, N=1200, B=256, b=600, n_s=64, d_R=128),
    dict(name="dec_bf16_g8_norope", dtype="bf16", h=8, h_kv=1, d=64, N=1100, B=250, b=500, n_s=50, d_R=128,
         rope=False),
    dict(name="dec_bf16_g3", dtype="bf16", h=6, h_kv=2, d=128, N=900, B=128, b=641, n_s=30, d_R=128),
    dict(name="dec_bf16_short_cache", dtype="bf16", h=8, h_kv=2, d=128, N=40, B=64, b=256, n_s=8, d_R=128),
]


def _prefill(w):
    """Teacher-forced prefill of the first N - N_DEC tokens."""
    n_pre = w.N - N_DEC
    sizes = [w.B] * (n_pre // w.B) + ([n_pre % w.B] if n_pre % w.B else [])
    layer, o, _ = _run_stream(w, teacher_forced=True, chunk_sizes=sizes)
    assert layer.cache_len == o.n_c
    return layer, o, n_pre


@pytest.mark.parametrize("kw", CASES, ids=[c["name"] for c in CASES])
def test_decode_tokens_with_scores(kw):
    w = synth.tiny(**kw)
    layer, o, n_pre = _prefill(w)
    n0 = o.n_c
    for i in range(N_DEC):
        q, k, v = synth.tokens(w, n_pre + i, n_pre + i + 1)
        out_ref, sc_ref, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, sc = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=True)
        tag = f"{w.name} token {i}"
        assert_close(host(out), out_ref, w.dtype, tag + " attention", per_row=True)
        assert_close(sc.cpu().numpy(), sc_ref[:, 0], w.dtype, tag + " score")
        assert layer.cache_len == o.n_c == n0 + i + 1
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
        s = S[m].cpu().numpy()
        np.testing.assert_array_equal(s[:n0], o.S[m][:n0])          # prefill part: teacher-forced, exact
    layer.close()


def test_decode_without_scores_then_evicting_chunk():
    # generated units carry NaN scores; a later evicting chunk drops them before any scored unit
    w = synth.tiny(name="dec_nan", dtype="bf16", h=8, h_kv=2, d=128, N=1400, B=200, b=500, n_s=40, d_R=128)
    layer, o, n_pre = _prefill(w)
    n0 = o.n_c
    for i in range(N_DEC):
        q, k, v = synth.tokens(w, n_pre + i, n_pre + i + 1)
        out_ref, _, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, sc = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=False)
        assert sc is None
        assert_close(host(out), out_ref, w.dtype, f"token {i} attention", per_row=True)
    for m in range(w.h_kv):
        o.S[m][n0:] = np.nan                                          # what the library stores for them
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        s = S[m].cpu().numpy()
        assert np.isnan(s[n0:]).all() and not np.isnan(s[:n0]).any()
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
    q, k, v = synth.tokens(w, 0, w.B - N_DEC)                         # a further chunk that still fits, teacher-forced
    out_ref, sc_ref, kept_ref = o.prefill_chunk(q, k, v, w.n_s)
    out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s,
                                        scores_in=torch.from_numpy(sc_ref).to(DEV))
    np.testing.assert_array_equal(kept.cpu().numpy()[:, :w.b], kept_ref)
    assert not np.isin(np.arange(n0, n0 + N_DEC), kept_ref[0]).any()   # the generated units went first
    assert_close(host(out), out_ref, w.dtype, "chunk after decode", per_row=True)
    layer.close()


def test_decode_capacity_and_argument_errors():
    from paper_2410_01805_amd import binding as B
    w = synth.tiny(name="dec_err", dtype="f32", h=4, h_kv=2, d=32, N=600, B=4, b=8, n_s=2, d_R=64)
    layer = B.LocretLayer(B.config_from_workload(w), DEV)
    q, k, v = (dev(x, w) for x in synth.tokens(w, 0, 1))
    with pytest.raises(B.LocretError) as e:        # scoring needs weights
        layer.decode_step(q, k, v, with_score=True)
    assert e.value.code == B.LOCRET_ESTATE
    for _ in range(12):                            # capacity = budget + chunk_max = 12 units
        layer.decode_step(q, k, v, with_score=False)
    assert layer.cache_len == 12
    with pytest.raises(B.LocretError) as e:
        layer.decode_step(q, k, v, with_score=False)
    assert e.value.code == B.LOCRET_ESTATE
    with pytest.raises(B.LocretError) as e:
        B.locret_decode_step(layer.ctx, q.data_ptr() + 4, k, v, 0, torch.empty_like(q))
    assert e.value.code == B.LOCRET_EALIGN
    layer.close()


def test_decode_on_the_full_budget_of_config3():
    # the headline layer with its cache at the budget: one generated token over 16384 units
    w = synth.WORKLOADS["cfg3_llama_128k"]
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    for c in range(5):                             # 5 chunks: cache full and compacted once
        q, k, v = synth.chunk(w, c)
        sc_ref = o.score(q, k, v)
        o.evict_compact(sc_ref, k, v, w.n_s)
        layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s, scores_in=torch.from_numpy(sc_ref).to(DEV))
    assert layer.cache_len == o.n_c == w.b
    for i in range(3):
        q, k, v = synth.tokens(w, 5 * w.B + i, 5 * w.B + i + 1)
        out_ref, _, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, _ = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=False)
        assert_close(host(out), out_ref, w.dtype, f"cfg3 decode token {i}", per_row=True, kappa=kappa_for(w))
    layer.close()
