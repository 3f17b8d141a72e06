"""GPU parity: stabilizer-masked top-b + compaction (Section 3.4, Algorithm 1) through
locret_evict_compact on caller-supplied scores.  Integer/byte work: everything is bit-exact."""
import zlib

import numpy as np
import pytest
import torch

from paper_2410_01805_amd import synth
from tests.gpu_util import DEV, dev, host, make_layer, make_oracle

pytestmark = pytest.mark.gpu


def _scores(rng, h_kv, T, kind):
    s = rng.standard_normal((h_kv, T)).astype(np.float32)
    if kind == "ties":
        s = (np.round(s * 2) / 2).astype(np.float32)
    elif kind == "constant":
        s[:] = 0.25
    elif kind == "specials":
        s = (np.round(s * 4) / 4).astype(np.float32)
        flat = s.reshape(-1)
        n = flat.size
        for val in (np.nan, np.inf, -np.inf, -0.0, 0.0):
            flat[rng.integers(0, n, size=max(1, n // 37))] = val
    elif kind == "tiny_spread":          # differences only in the low mantissa bits: last radix pass decides
        s = (1.0 + rng.integers(0, 200, size=(h_kv, T)) * 2.0 ** -23).astype(np.float32)
    elif kind == "negative":
        s = -np.abs(s) - 1.0
    return s


CASES = [
    # name, workload overrides, chunk sizes (None = all B), score kind
    ("f32_small", dict(dtype="f32", h=4, h_kv=2, d=64, N=4000, B=500, b=1000, n_s=64, rope=False), None, "normal"),
    ("f32_ties", dict(dtype="f32", h=4, h_kv=2, d=64, N=4000, B=500, b=1000, n_s=64, rope=False), None, "ties"),
    ("bf16_rope_ragged", dict(dtype="bf16", h=8, h_kv=8, d=128, N=9000, B=1000, b=3000, n_s=300), None, "normal"),
    ("bf16_specials", dict(dtype="bf16", h=4, h_kv=4, d=96, N=6000, B=700, b=2048, n_s=100), None, "specials"),
    ("ns_gt_B", dict(dtype="bf16", h=2, h_kv=2, d=64, N=6000, B=256, b=2000, n_s=700), None, "ties"),
    ("ns_zero", dict(dtype="f32", h=2, h_kv=2, d=32, N=3000, B=300, b=1024, n_s=0, rope=False), None, "normal"),
    ("ns_eq_b", dict(dtype="f32", h=2, h_kv=1, d=16, N=2000, B=200, b=512, n_s=512), None, "normal"),
    ("constant", dict(dtype="bf16", h=2, h_kv=2, d=64, N=5000, B=1000, b=1500, n_s=10), None, "constant"),
    ("tiny_spread", dict(dtype="f32", h=2, h_kv=2, d=16, N=5000, B=1000, b=1500, n_s=10, rope=False), None, "tiny_spread"),
    ("negative", dict(dtype="f32", h=2, h_kv=2, d=16, N=5000, B=1000, b=1500, n_s=10, rope=False), None, "negative"),
    ("odd_chunks", dict(dtype="bf16", h=4, h_kv=2, d=128, N=5000, B=1100, b=2000, n_s=33), [1, 1100, 7, 64, 65, 1023, 1, 1100, 1100, 538], "specials"),
    ("paper_phi3_row", dict(dtype="bf16", h=2, h_kv=2, d=96, N=20000, B=3072, b=6000, n_s=2500), None, "normal"),
    ("paper_llama_row", dict(dtype="bf16", h=2, h_kv=1, d=128, N=24000, B=1024, b=16384, n_s=2500), None, "normal"),
    # more candidates than the register-resident select holds: keys staged in LDS ...
    ("keys_in_lds", dict(dtype="f32", h=1, h_kv=1, d=16, N=34000, B=2000, b=26000, n_s=100, rope=False), None, "ties"),
    # ... and more than LDS holds: keys re-read from global memory in every pass
    ("keys_in_global", dict(dtype="f32", h=1, h_kv=1, d=16, N=50000, B=2000, b=40000, n_s=7, rope=False), None, "specials"),
]


@pytest.mark.parametrize("name,kw,sizes,kind", CASES, ids=[c[0] for c in CASES])
def test_evict_compact_bit_exact(name, kw, sizes, kind):
    w = synth.tiny(name=name, **kw)
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    lo = 0
    sizes = sizes or [w.B] * w.n_chunks
    for step, T in enumerate(sizes):
        hi = min(w.N, lo + T)
        T = hi - lo
        if T <= 0:
            break
        _, k, v = synth.tokens(w, lo, hi)
        sc = _scores(rng, w.h_kv, T, kind)
        n_c = o.n_c
        kept_ref = o.evict_compact(sc, k, v, w.n_s)
        kept = layer.evict_compact(torch.from_numpy(sc).to(DEV), dev(k, w), dev(v, w), w.n_s)
        n_keep = min(n_c + T, w.b)
        assert layer.cache_len == n_keep == o.n_c
        got = kept.cpu().numpy()
        np.testing.assert_array_equal(got[:, :n_keep], kept_ref, err_msg=f"{name} step {step}")
        assert (got[:, n_keep:] == -1).all()
        lo = hi
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
        np.testing.assert_array_equal(S[m].cpu().numpy().view(np.uint32), o.S[m].view(np.uint32))
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
    layer.close()


def test_select_is_deterministic_and_reset_works():
    w = synth.tiny(dtype="bf16", h=2, h_kv=2, d=64, N=4096, B=1024, b=1536, n_s=16)
    layer, _, _ = make_layer(w)
    rng = np.random.default_rng(3)
    sc = [torch.from_numpy(_scores(rng, 2, 1024, "ties")).to(DEV) for _ in range(4)]
    kv = [tuple(dev(x, w) for x in synth.chunk(w, c)[1:]) for c in range(4)]
    runs = []
    for rep in range(2):
        layer.reset()
        assert layer.cache_len == 0
        runs.append([layer.evict_compact(sc[c], kv[c][0], kv[c][1], w.n_s).cpu().numpy() for c in range(4)])
    for a, b in zip(*runs):
        np.testing.assert_array_equal(a, b)
    layer.close()


# ---- pinned prefix (Locret-Q): the first n_pin units survive every eviction ------------------------
PIN_CASES = [
    # name, workload overrides, n_pin, score kind
    ("pin_f32", dict(dtype="f32", h=4, h_kv=2, d=64, N=4000, B=500, b=1000, n_s=64, rope=False), 100, "normal"),
    ("pin_bf16_rope", dict(dtype="bf16", h=8, h_kv=4, d=128, N=9000, B=1000, b=3000, n_s=300), 777, "specials"),
    ("pin_one", dict(dtype="bf16", h=2, h_kv=2, d=64, N=5000, B=1000, b=1500, n_s=10), 1, "ties"),
    ("pin_fills_budget", dict(dtype="f32", h=2, h_kv=2, d=16, N=3000, B=300, b=512, n_s=12, rope=False), 500, "normal"),
    ("pin_gt_first_chunk", dict(dtype="bf16", h=2, h_kv=1, d=96, N=6000, B=256, b=2000, n_s=700), 900, "ties"),
    ("pin_keys_in_lds", dict(dtype="f32", h=1, h_kv=1, d=16, N=34000, B=2000, b=26000, n_s=100, rope=False), 333, "ties"),
    ("pin_keys_in_global", dict(dtype="f32", h=1, h_kv=1, d=16, N=50000, B=2000, b=40000, n_s=7, rope=False), 64, "specials"),
]


@pytest.mark.parametrize("name,kw,n_pin,kind", PIN_CASES, ids=[c[0] for c in PIN_CASES])
def test_evict_compact_with_pinned_prefix_bit_exact(name, kw, n_pin, kind):
    w = synth.tiny(name=name, **kw)
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    o.n_pin = n_pin
    layer.set_pinned_prefix(n_pin)
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    for c in range(w.n_chunks):
        lo, hi = w.chunk_range(c)
        _, k, v = synth.tokens(w, lo, hi)
        sc = _scores(rng, w.h_kv, hi - lo, kind)
        if c == 0:
            sc[:, :min(n_pin, hi - lo)] = -1e30        # on their merits the pinned units would go first
        n_c = o.n_c
        kept_ref = o.evict_compact(sc, k, v, w.n_s)
        kept = layer.evict_compact(torch.from_numpy(sc).to(DEV), dev(k, w), dev(v, w), w.n_s)
        n_keep = min(n_c + (hi - lo), w.b)
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :n_keep], kept_ref, err_msg=f"{name} chunk {c}")
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
        np.testing.assert_array_equal(S[m].cpu().numpy().view(np.uint32), o.S[m].view(np.uint32))
        npp = min(n_pin, w.b - w.n_s)
        assert P[m].cpu().numpy()[:npp].tolist() == list(range(npp))      # the stream's first tokens, in place
    layer.close()


def test_pinned_prefix_argument_errors_and_reset():
    from paper_2410_01805_amd import binding as B
    w = synth.tiny(name="pin_err", dtype="f32", h=2, h_kv=2, d=16, N=600, B=100, b=250, n_s=20, d_R=64, rope=False)
    layer, _, _ = make_layer(w)
    for bad in (-1, 251):
        with pytest.raises(B.LocretError) as e:
            layer.set_pinned_prefix(bad)
        assert e.value.code == B.LOCRET_EINVAL
    layer.set_pinned_prefix(240)
    _, k, v = synth.tokens(w, 0, 100)
    sc = torch.zeros(2, 100, device=DEV)
    with pytest.raises(B.LocretError) as e:            # 240 pinned + 20 stabilizers > 250
        layer.evict_compact(sc, dev(k, w), dev(v, w), 20)
    assert e.value.code == B.LOCRET_EINVAL
    assert layer.cache_len == 0
    layer.evict_compact(sc, dev(k, w), dev(v, w), 10)
    layer.reset()                                      # the setting survives a reset
    with pytest.raises(B.LocretError):
        layer.evict_compact(sc, dev(k, w), dev(v, w), 20)
    layer.set_pinned_prefix(0)
    layer.evict_compact(sc, dev(k, w), dev(v, w), 20)
    layer.close()
