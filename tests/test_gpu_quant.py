"""4-bit cache rows on the GPU (config.kv_bits = 4) against the oracle's (kv_bits = 4), through the C ABI.

Bit-exact: the packed rows (codes, scales, minima) of every unit in the cache, kept indices, positions, score
bits.  Within the bf16 tolerance: attention (chunk and decode), which on both sides reads the dequantized
rows, and the retaining head's scores (computed from the raw inputs)."""
import numpy as np
import pytest
import torch

from oracle.locret_oracle import LocretLayerOracle, q4_roundtrip
from paper_2410_01805_amd import binding as B
from paper_2410_01805_amd import synth
from tests.gpu_util import DEV, assert_close, dev, host, make_layer

pytestmark = pytest.mark.gpu


def _oracle(w, W1, W2):
    return LocretLayerOracle(w.h, w.h_kv, w.d, w.b, W1, W2, w.rh_kv_expand, w.rope, w.theta, kv_bits=4)


def _assert_packed_cache_equal(layer, o, w, tag=""):
    Kq, Vq, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        n = o.Kq[m].shape[0]
        np.testing.assert_array_equal(P[m].cpu().numpy()[:n], o.P[m], err_msg=tag)
        np.testing.assert_array_equal(Kq[m].cpu().numpy()[:n], o.Kq[m], err_msg=tag + " packed K rows")
        np.testing.assert_array_equal(Vq[m].cpu().numpy()[:n], o.Vq[m], err_msg=tag + " packed V rows")
        np.testing.assert_array_equal(S[m].cpu().numpy()[:n].view(np.uint32), o.S[m].view(np.uint32), err_msg=tag)


STREAMS = [
    dict(name="q4_llama_like", dtype="bf16", h=8, h_kv=2, d=128, N=2500, B=300, b=700, n_s=100, d_R=128, theta=500000.0),
    dict(name="q4_phi_like", dtype="bf16", h=4, h_kv=4, d=96, N=2000, B=256, b=600, n_s=64, d_R=128),
    dict(name="q4_d64_norope", dtype="bf16", h=4, h_kv=1, d=64, N=1500, B=250, b=500, n_s=500, d_R=256, rope=False),
    dict(name="q4_ns_gt_B", dtype="bf16", h=4, h_kv=2, d=128, N=1800, B=128, b=640, n_s=300, d_R=128),
]


@pytest.mark.parametrize("kw", STREAMS, ids=[s["name"] for s in STREAMS])
def test_teacher_forced_stream_with_4bit_rows(kw):
    w = synth.tiny(kv_bits=4, **kw)
    layer, W1, W2 = make_layer(w)
    o = _oracle(w, W1, W2)
    for c in range(w.n_chunks):
        q, k, v = synth.chunk(w, c)
        n_c, T = o.n_c, q.shape[0]
        out_ref, sc_ref, kept_ref = o.prefill_chunk(q, k, v, w.n_s)
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s, scores_in=torch.from_numpy(sc_ref).to(DEV))
        tag = f"{w.name} chunk {c}"
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :min(n_c + T, w.b)], kept_ref, err_msg=tag)
        assert_close(sc.cpu().numpy(), sc_ref, w.dtype, tag + " scores")
        assert_close(host(out), out_ref, w.dtype, tag + " attention", per_row=True)
        _assert_packed_cache_equal(layer, o, w, tag)
    # the tail pass of Algorithm 1 (no eviction) and two generated tokens on top
    q, k, v = synth.tokens(w, w.N, w.N + 50)
    out_ref, sc_ref, _ = o.prefill_chunk(q, k, v, 0, evict=False)
    out, sc, _ = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), 0, evict=False)
    assert_close(host(out), out_ref, w.dtype, w.name + " tail attention", per_row=True)
    for i in range(2):
        q, k, v = synth.tokens(w, w.N + 50 + i, w.N + 51 + i)
        out_ref, sc_ref, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, sc = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=(i == 0))
        assert_close(host(out), out_ref, w.dtype, f"{w.name} decode {i} attention", per_row=True)
        if i == 0:
            assert_close(sc.cpu().numpy(), sc_ref[:, 0], w.dtype, f"{w.name} decode {i} score")
    Kq, Vq, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(Kq[m].cpu().numpy(), o.Kq[m])
        np.testing.assert_array_equal(Vq[m].cpu().numpy(), o.Vq[m])
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
    layer.close()


def test_evict_compact_entry_point_moves_packed_rows_bit_exactly():
    w = synth.tiny(name="q4_evict", kv_bits=4, dtype="bf16", h=8, h_kv=4, d=128, N=6000, B=1000, b=2200, n_s=300, d_R=128)
    layer, W1, W2 = make_layer(w)
    o = _oracle(w, W1, W2)
    for c in range(w.n_chunks):
        q, k, v = synth.chunk(w, c)
        T = k.shape[0]
        s_in = synth.standard_normal(w.seed, 77, c * w.h_kv * w.B, w.h_kv * T).reshape(w.h_kv, T).astype(np.float32)
        n_c = o.n_c
        kept_ref = o.evict_compact(s_in, k, v, w.n_s)
        kept = layer.evict_compact(torch.from_numpy(s_in).to(DEV), dev(k, w), dev(v, w), w.n_s)
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :min(n_c + T, w.b)], kept_ref)
    _assert_packed_cache_equal(layer, o, w)
    layer.close()


def test_edge_values_quantize_like_the_oracle():
    # constant groups, groups with one outlier, tiny and huge magnitudes, exact ties: rows chosen by hand, fed as k and v
    w = synth.tiny(name="q4_edges", kv_bits=4, dtype="bf16", h=2, h_kv=2, d=64, N=64, B=64, b=64, n_s=0, d_R=128, rope=False)
    layer, W1, W2 = make_layer(w)
    o = _oracle(w, W1, W2)
    q, k, v = synth.chunk(w, 0)
    k = k.copy(); v = v.copy()
    k[0] = 3.5                                                        # constant rows
    k[1] = 0.0
    k[2, :, :32] = np.arange(32) % 16                                 # step exactly 1
    k[2, :, 32:] = (np.arange(32) % 16) + np.where(np.arange(32) % 5 == 0, 0.5, 0.0)      # exact ties
    k[3] = 0.0; k[3, :, 7] = 1.0; k[3, :, 40] = -1.0                  # single outliers
    k[4] = synth.storage_round(k[4].astype(np.float64) * 1e-30, "bf16")           # tiny
    k[5] = synth.storage_round(k[5].astype(np.float64) * 1e30, "bf16")            # huge
    k[6, :, ::2] = 1.0; k[6, :, 1::2] = -1.0
    v[:7] = k[:7][::-1]
    s_in = np.zeros((w.h_kv, 64), np.float32)
    o.evict_compact(s_in, k, v, 0)
    layer.evict_compact(torch.from_numpy(s_in).to(DEV), dev(k, w), dev(v, w), 0)
    _assert_packed_cache_equal(layer, o, w)
    layer.close()


def test_argument_errors_of_the_4bit_mode():
    w = synth.tiny(name="q4_err", kv_bits=4, dtype="bf16", h=4, h_kv=2, d=128, N=256, B=64, b=128, n_s=8, d_R=128)
    layer, W1, W2 = make_layer(w)
    with pytest.raises(B.LocretError) as e:
        layer.set_head_budgets([64, 128])
    assert e.value.code == B.LOCRET_ESHAPE
    view = B.locret_cache_view(layer.ctx)
    assert view["K"] is None and view["V"] is not None
    vq = B.locret_cache_view_q4(layer.ctx)
    assert vq["row_bytes"] == 64 + 16 and vq["row_stride_bytes"] == 80 and vq["row_stride"] == w.b + w.B
    layer.close()
    # float32 tensors, an unsupported head_dim, a bad bit count
    for kw, code in ((dict(dtype="f32"), 0), (dict(d=32), 0)):
        cfg = B.config_from_workload(synth.tiny(name="q4_bad", kv_bits=4, h=4, h_kv=2, N=64, B=16, b=32, n_s=0, d_R=64,
                                                **{**dict(dtype="bf16", d=128), **kw}))
        assert B.locret_workspace_bytes(cfg) == code
    cfg = B.config_from_workload(synth.tiny(name="q4_bad", kv_bits=3, dtype="bf16", h=4, h_kv=2, d=128, N=64, B=16, b=32,
                                            n_s=0, d_R=64))
    assert B.locret_workspace_bytes(cfg) == 0
    # plain contexts have no packed view
    w0 = synth.tiny(name="q4_plain", dtype="bf16", h=4, h_kv=2, d=128, N=64, B=16, b=32, n_s=0, d_R=128)
    layer0, _, _ = make_layer(w0)
    with pytest.raises(B.LocretError) as e:
        B.locret_cache_view_q4(layer0.ctx)
    assert e.value.code == B.LOCRET_ESTATE
    layer0.close()


def test_4bit_rows_shrink_the_workspace():
    w = synth.WORKLOADS["cfg3_llama_128k"]
    import dataclasses
    plain = B.locret_workspace_bytes(B.config_from_workload(w))
    quant = B.locret_workspace_bytes(B.config_from_workload(dataclasses.replace(w, kv_bits=4)))
    rows = w.h_kv * (w.b + w.B)
    # two copies of K, V and the rotated shadow (1536 B per unit) against two packed copies of K, V (320 B) + one
    # bf16 staging pair (512 B)
    assert plain - quant >= rows * (1536 - 832) * 0.95


def test_config3_shape_with_4bit_rows_reaches_steady_state():
    """Config 3's layer and launch shapes (chunks of 4096, budget 16384) with 4-bit rows, 6 chunks: two steady-state
    steps.  Kept indices bit-exact on every chunk (teacher-forced), the library's scores on every chunk, attention on
    sampled rows, and at the end every packed row of the cache bit for bit."""
    import dataclasses
    from concurrent.futures import ThreadPoolExecutor
    from tests.gpu_util import kappa_for
    w = dataclasses.replace(synth.WORKLOADS["cfg3_llama_128k"], kv_bits=4, N=6 * 4096)
    layer, W1, W2 = make_layer(w)
    o = _oracle(w, W1, W2)
    with ThreadPoolExecutor(max_workers=6) as ex:
        chunks = list(ex.map(lambda c: synth.chunk(w, c), range(w.n_chunks)))
    rng = np.random.default_rng(3)
    for c, (q, k, v) in enumerate(chunks):
        n_c, T = o.n_c, q.shape[0]
        rows = np.sort(rng.choice(T, size=12, replace=False)) if c in (0, 4, 5) else None
        out_ref = o.attention(q, k, v, rows=rows) if rows is not None else None
        sc_ref = o.score(q, k, v)
        kept_ref = o.evict_compact(sc_ref, k, v, w.n_s)
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s, scores_in=torch.from_numpy(sc_ref).to(DEV))
        tag = f"cfg3 shape, 4-bit rows, chunk {c}"
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :min(n_c + T, w.b)], kept_ref, err_msg=tag)
        assert_close(sc.cpu().numpy(), sc_ref, w.dtype, tag + " scores")
        if rows is not None:
            assert_close(host(out[rows]), out_ref[rows], w.dtype, tag + " attention", per_row=True, kappa=kappa_for(w))
    assert layer.cache_len == o.n_c == w.b
    _assert_packed_cache_equal(layer, o, w, "cfg3 shape final cache")
    layer.close()
