"""GPU parity with head-wise budgets (appendix "Orthogonality to Other Methods", head-wise budget
allocation: KV heads evict independently, so each may have a budget of its own): the heads' caches
differ in length, every kernel of the step takes the lengths per head.  Same bars as the single-budget
tests: kept indices and cache contents bit-exact on equal scores, attention and scores within the
tolerance."""
import zlib

import numpy as np
import pytest
import torch

from oracle.locret_oracle import LocretLayerOracle
from paper_2410_01805_amd import binding as B
from paper_2410_01805_amd import synth
from tests.gpu_util import DEV, assert_close, dev, host, make_layer
from tests.test_gpu_select_compact import _scores

pytestmark = pytest.mark.gpu


def _oracle(w, W1, W2, budgets, n_pin=0):
    budgets = w.b if budgets is None else budgets         # None: the config's single budget
    return LocretLayerOracle(w.h, w.h_kv, w.d, budgets, W1, W2, w.rh_kv_expand, w.rope, w.theta, n_pin=n_pin)


def _assert_caches_equal(layer, o, w, check_scores=True):
    K, V, S, P = layer.cache_tensors()
    lens = layer.cache_lens
    assert lens == [o.n_c_of(m) for m in range(w.h_kv)]
    assert layer.cache_len == max(lens)
    for m in range(w.h_kv):
        n = lens[m]
        np.testing.assert_array_equal(P[m, :n].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m, :n]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m, :n]), o.V[m].astype(np.float32))
        if check_scores:
            np.testing.assert_array_equal(S[m, :n].cpu().numpy().view(np.uint32), o.S[m].view(np.uint32))


def _assert_kept_equal(kept, kept_ref, tag):
    got = kept.cpu().numpy()
    for m, ref in enumerate(kept_ref):
        np.testing.assert_array_equal(got[m, :len(ref)], ref, err_msg=f"{tag} head {m}")
        assert (got[m, len(ref):] == -1).all(), f"{tag} head {m}: entries past the head's kept list were written"


EVICT_CASES = [
    # name, workload overrides (b = the largest budget), budgets, n_pin, score kind
    ("f32_two_heads", dict(dtype="f32", h=4, h_kv=2, d=64, N=4000, B=500, b=1000, n_s=64, rope=False),
     [1000, 300], 0, "normal"),
    ("bf16_rope_pyramid", dict(dtype="bf16", h=8, h_kv=8, d=128, N=9000, B=1000, b=3000, n_s=300),
     [3000, 2600, 2200, 1800, 1400, 1000, 600, 300], 0, "ties"),
    ("bf16_d96_specials", dict(dtype="bf16", h=4, h_kv=4, d=96, N=6000, B=700, b=2048, n_s=100),
     [100, 2048, 777, 1500], 0, "specials"),          # head 0 holds stabilizers only
    ("one_head_never_full", dict(dtype="bf16", h=2, h_kv=2, d=64, N=3000, B=256, b=4000, n_s=700),
     [4000, 900], 0, "ties"),                          # n_s > B; head 0 never evicts, yet changes copy with head 1
    ("pinned_prefix", dict(dtype="bf16", h=8, h_kv=4, d=128, N=6000, B=1000, b=3000, n_s=200),
     [3000, 1000, 2000, 1300], 777, "specials"),
    ("odd_chunks", dict(dtype="f32", h=3, h_kv=3, d=32, N=3000, B=700, b=900, n_s=33, rope=True),
     [900, 34, 411], 0, "specials"),
    # the longest head sizes the launch: keys staged in LDS, or re-read from global memory, beside a short head
    ("keys_in_lds", dict(dtype="f32", h=2, h_kv=2, d=16, N=34000, B=2000, b=26000, n_s=100, rope=False),
     [26000, 500], 0, "ties"),
    ("keys_in_global", dict(dtype="f32", h=2, h_kv=2, d=16, N=50000, B=2000, b=40000, n_s=7, rope=False),
     [700, 40000], 0, "specials"),
]


@pytest.mark.parametrize("name,kw,budgets,n_pin,kind", EVICT_CASES, ids=[c[0] for c in EVICT_CASES])
def test_evict_compact_with_head_budgets_bit_exact(name, kw, budgets, n_pin, kind):
    w = synth.tiny(name=name, **kw)
    layer, W1, W2 = make_layer(w)
    layer.set_head_budgets(budgets)
    o = _oracle(w, W1, W2, budgets, n_pin)
    if n_pin:
        layer.set_pinned_prefix(n_pin)
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    sizes = [1, w.B, 7, 65, w.B - 1] + [w.B] * w.n_chunks if name == "odd_chunks" else [w.B] * w.n_chunks
    lo = 0
    for step, T in enumerate(sizes):
        hi = min(w.N, lo + T)
        T = hi - lo
        if T <= 0:
            break
        _, k, v = synth.tokens(w, lo, hi)
        sc = _scores(rng, w.h_kv, T, kind)
        kept_ref = o.evict_compact(sc, k, v, w.n_s)
        kept = layer.evict_compact(torch.from_numpy(sc).to(DEV), dev(k, w), dev(v, w), w.n_s)
        _assert_kept_equal(kept, kept_ref, f"{name} step {step}")
        assert layer.cache_lens == [o.n_c_of(m) for m in range(w.h_kv)]
        lo = hi
    _assert_caches_equal(layer, o, w)
    layer.close()


def _run_stream(w, budgets, n_pin=0, last_chunk_unmasked=True):
    """Teacher-forced chunk steps (the oracle's float32 scores decide the selection on both sides)."""
    layer, W1, W2 = make_layer(w)
    layer.set_head_budgets(budgets)
    o = _oracle(w, W1, W2, budgets, n_pin)
    if n_pin:
        layer.set_pinned_prefix(n_pin)
    lo = 0
    for step in range(w.n_chunks):
        hi = min(w.N, lo + w.B)
        q, k, v = synth.tokens(w, lo, hi)
        n_stab = 0 if (last_chunk_unmasked and hi == w.N) else w.n_s
        out_ref, sc_ref, kept_ref = o.prefill_chunk(q, k, v, n_stab)
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), n_stab,
                                            scores_in=torch.from_numpy(sc_ref).to(DEV))
        tag = f"{w.name} chunk {step}"
        assert_close(sc.cpu().numpy(), sc_ref, w.dtype, tag + " scores")
        assert_close(host(out), out_ref, w.dtype, tag + " attention", per_row=True)
        _assert_kept_equal(kept, kept_ref, tag)
        lo = hi
    return layer, o


STREAMS = [
    (dict(name="hb_f32_gqa", dtype="f32", h=8, h_kv=2, d=64, N=1500, B=200, b=400, n_s=32, d_R=64, rope=False),
     [400, 150]),
    (dict(name="hb_f32_rope_mha", dtype="f32", h=3, h_kv=3, d=16, N=700, B=100, b=150, n_s=10, d_R=40, rope=True),
     [150, 10, 77]),
    (dict(name="hb_bf16_llama_like", dtype="bf16", h=8, h_kv=2, d=128, N=2500, B=300, b=700, n_s=100, d_R=128,
          theta=500000.0), [700, 250]),
    (dict(name="hb_bf16_llama_g4_8heads", dtype="bf16", h=32, h_kv=8, d=128, N=1800, B=256, b=640, n_s=64, d_R=128),
     [640, 576, 512, 448, 384, 320, 200, 64]),
    (dict(name="hb_bf16_phi_like", dtype="bf16", h=4, h_kv=4, d=96, N=2000, B=256, b=600, n_s=64, d_R=128),
     [600, 64, 333, 500]),
    (dict(name="hb_bf16_d64_norope", dtype="bf16", h=4, h_kv=2, d=64, N=1500, B=250, b=500, n_s=120, d_R=256,
          rope=False), [120, 500]),
]


@pytest.mark.parametrize("kw,budgets", STREAMS, ids=[c[0]["name"] for c in STREAMS])
def test_chunk_step_stream_with_head_budgets(kw, budgets):
    w = synth.tiny(**kw)
    layer, o = _run_stream(w, budgets)
    _assert_caches_equal(layer, o, w)
    layer.close()


def test_chunk_step_with_head_budgets_and_pinned_prefix():
    w = synth.tiny(**STREAMS[2][0])
    layer, o = _run_stream(w, [700, 300], n_pin=48)
    _assert_caches_equal(layer, o, w)
    assert all(o.P[m][:48].tolist() == list(range(48)) for m in range(w.h_kv))
    layer.close()


def test_register_staged_attention_kernel_with_head_budgets(monkeypatch):
    monkeypatch.setenv("LOCRET_ATTN_VARIANT", "regstaged")
    w = synth.tiny(**STREAMS[2][0])
    layer, o = _run_stream(w, STREAMS[2][1])
    layer.close()


@pytest.mark.parametrize("env", [("LOCRET_FUSE_SELECT", "0"), ("LOCRET_OVERLAP", "1"), ("LOCRET_FORCE_SIMPLE", "1")])
def test_other_launch_orders_with_head_budgets(env, monkeypatch):
    # the selection as a launch of its own, selection and compaction on a second stream, the plain kernels
    monkeypatch.setenv(*env)
    w = synth.tiny(**STREAMS[2][0])
    layer, o = _run_stream(w, STREAMS[2][1])
    torch.cuda.synchronize()
    _assert_caches_equal(layer, o, w)
    layer.close()


# The matrix-core attention kernels deal their workgroups differently when the heads differ in length: every XCD
# takes every eighth token tile of every head, longest head first, instead of one head per XCD (8 token tiles here:
# whole rounds of the 8 XCDs; the other streams of this file have tile counts that leave the last round short).  LOCRET_PP_SPREAD (read when the context is created) = 0 keeps one head per XCD, 1 forces the other order.
SPREAD = dict(name="hb_spread", dtype="bf16", h=16, h_kv=4, d=128, N=3584, B=512, b=1100, n_s=64, d_R=128)


@pytest.mark.parametrize("spread,budgets", [(None, [300, 1100, 64, 700]), ("0", [300, 1100, 64, 700]), ("1", None)])
def test_workgroup_orders_of_the_head_dim_128_kernel(spread, budgets, monkeypatch):
    if spread is not None:
        monkeypatch.setenv("LOCRET_PP_SPREAD", spread)
    w = synth.tiny(**SPREAD)
    layer, o = _run_stream(w, budgets)
    _assert_caches_equal(layer, o, w)
    layer.close()


def test_workgroup_order_of_the_other_head_dims_with_head_budgets():
    # head_dim 96 (register-staged kernel, 256 tokens per workgroup): 8 token tiles
    w = synth.tiny(name="hb_spread_d96", dtype="bf16", h=4, h_kv=4, d=96, N=3 * 2048, B=2048, b=2500, n_s=64, d_R=128)
    layer, o = _run_stream(w, [2500, 300, 1200, 64])
    _assert_caches_equal(layer, o, w)
    layer.close()


def test_key_split_with_head_budgets(monkeypatch):
    monkeypatch.setenv("LOCRET_PP_SPLIT", "4")         # 8 token tiles x 4 key ranges, dealt over the XCDs longest head first
    w = synth.tiny(**SPREAD)
    layer, o = _run_stream(w, [300, 1100, 64, 700])
    _assert_caches_equal(layer, o, w)
    layer.close()


def test_full_size_launch_with_head_budgets():
    """The Llama-3-8B layer shape of the benchmark configuration (32 query / 8 KV heads x 128, chunks of 4096,
    2048 stabilizers) with a pyramid of budgets of the same total as 8 x 16384: kept indices bit-exact on every
    chunk (seeded scores drive the selection on both sides), attention on sampled rows of sampled chunks."""
    from tests.test_gpu_fullsize import _POOL, _sample_rows
    import dataclasses
    budgets = [28672, 25161, 21650, 18139, 14628, 11117, 7606, 4099]
    w = dataclasses.replace(synth.WORKLOADS["cfg3_llama_128k"], name="cfg3_shape_pyramid", b=max(budgets),
                            N=11 * 4096, planted_frac=0.0)
    layer, W1, W2 = make_layer(w)
    layer.set_head_budgets(budgets)
    o = _oracle(w, W1, W2, budgets)
    rng = np.random.default_rng(w.seed)
    chunks = list(_POOL.map(lambda c: synth.chunk(w, c), range(w.n_chunks)))
    for c, (q, k, v) in enumerate(chunks):
        T = q.shape[0]
        s_in = synth.standard_normal(w.seed, 98, c * w.h_kv * T, w.h_kv * T).reshape(w.h_kv, T).astype(np.float32)
        rows = _sample_rows(T, rng) if c in (0, 1, 7, 10) else None
        out_ref = o.attention(q, k, v, rows=rows) if rows is not None else None
        kept_ref = o.evict_compact(s_in, k, v, w.n_s)
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s,
                                            scores_in=torch.from_numpy(s_in).to(DEV))
        _assert_kept_equal(kept, kept_ref, f"chunk {c}")
        if rows is not None:
            assert_close(host(out[rows]), out_ref[rows], w.dtype, f"chunk {c} attention", per_row=True)
            assert_close(sc.cpu().numpy(), o.score(q, k, v), w.dtype, f"chunk {c} scores")
    assert layer.cache_lens == budgets
    _assert_caches_equal(layer, o, w)
    layer.close()


def test_equal_head_budgets_give_the_single_budget_results_bit_for_bit():
    w = synth.tiny(**STREAMS[2][0])
    outs = []
    for budgets in (None, [w.b] * w.h_kv):
        layer, W1, W2 = make_layer(w)
        layer.set_head_budgets(budgets)
        res = []
        for c in range(w.n_chunks):
            q, k, v = synth.chunk(w, c)
            out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s)
            res.append((out.cpu(), sc.cpu(), kept.cpu()))
        outs.append(res)
        layer.close()
    for (a_out, a_sc, a_kept), (b_out, b_sc, b_kept) in zip(*outs):
        assert torch.equal(a_out.view(torch.int16), b_out.view(torch.int16))
        assert torch.equal(a_sc.view(torch.int32), b_sc.view(torch.int32))
        assert torch.equal(a_kept, b_kept)


@pytest.mark.parametrize("kw,budgets", [STREAMS[0], STREAMS[2], STREAMS[4]],
                         ids=[STREAMS[i][0]["name"] for i in (0, 2, 4)])
def test_decode_steps_with_head_budgets(kw, budgets):
    # the decode step appends behind every head's own cache and attends over that head's units only
    w = synth.tiny(**kw)
    n_dec = 5
    w_pre = synth.tiny(**dict(kw, N=w.N - n_dec))
    layer, o = _run_stream(w_pre, budgets, last_chunk_unmasked=False)
    lens0 = layer.cache_lens
    assert len(set(lens0)) > 1
    for i in range(n_dec):
        q, k, v = synth.tokens(w, w_pre.N + i, w_pre.N + i + 1)
        out_ref, sc_ref, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, sc = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=True)
        assert_close(host(out), out_ref, w.dtype, f"{w.name} token {i} attention", per_row=True)
        assert_close(sc.cpu().numpy(), sc_ref[:, 0], w.dtype, f"{w.name} token {i} score")
        assert layer.cache_lens == [n + i + 1 for n in lens0]
    _assert_caches_equal(layer, o, w, check_scores=False)
    # a later evicting chunk brings every head back to its own budget
    T = w.B - n_dec                                       # what the capacity b + B still takes
    q, k, v = synth.tokens(w, 0, T)
    sc = np.zeros((w.h_kv, T), np.float32)
    o.evict_compact(sc, k, v, w.n_s)
    layer.evict_compact(torch.from_numpy(sc).to(DEV), dev(k, w), dev(v, w), w.n_s)
    assert layer.cache_lens == [o.n_c_of(m) for m in range(w.h_kv)] == budgets
    layer.close()


def test_head_budget_argument_errors():
    w = synth.tiny(dtype="f32", h=4, h_kv=2, d=32, N=400, B=100, b=200, n_s=20, d_R=32, rope=False)
    layer, _, _ = make_layer(w)
    for bad in ([0, 100], [100, 201], [-5, 10]):
        with pytest.raises(B.LocretError) as e:
            layer.set_head_budgets(bad)
        assert e.value.code == B.LOCRET_EINVAL
    with pytest.raises(B.LocretError):
        layer.set_head_budgets([100])                     # one value per KV head
    layer.set_head_budgets([200, 50])
    q, k, v = (dev(x, w) for x in synth.chunk(w, 0))
    with pytest.raises(B.LocretError) as e:               # stabilizers must fit the smallest budget
        layer.prefill_chunk(q, k, v, 51)
    assert e.value.code == B.LOCRET_EINVAL
    layer.set_pinned_prefix(40)
    with pytest.raises(B.LocretError) as e:               # ... together with the pinned prefix
        layer.prefill_chunk(q, k, v, 20)
    assert e.value.code == B.LOCRET_EINVAL
    assert layer.cache_lens == [0, 0]
    layer.set_pinned_prefix(0)
    layer.prefill_chunk(q, k, v, 20)
    assert layer.cache_lens == [100, 50]
    with pytest.raises(B.LocretError) as e:               # only on an empty cache
        layer.set_head_budgets([100, 100])
    assert e.value.code == B.LOCRET_ESTATE
    layer.reset()
    assert layer.cache_lens == [0, 0]
    layer.set_head_budgets(None)                          # back to the config's single budget
    layer.prefill_chunk(q, k, v, 20)
    layer.prefill_chunk(q, k, v, 20)
    layer.prefill_chunk(q, k, v, 20)
    assert layer.cache_lens == [200, 200] and layer.cache_len == 200
    layer.close()
    big = synth.tiny(dtype="f32", h=65, h_kv=65, d=16, N=64, B=16, b=32, n_s=2, d_R=32, rope=False)
    layer, _, _ = make_layer(big)
    with pytest.raises(B.LocretError) as e:
        layer.set_head_budgets([32] * 65)
    assert e.value.code == B.LOCRET_ESHAPE
    layer.close()
