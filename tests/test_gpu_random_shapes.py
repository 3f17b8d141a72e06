"""GPU parity on seeded random layer shapes and call patterns: head counts, group sizes, head dims,
ragged chunk sizes, stabilizer lengths, pinned prefixes and a few decode steps, all against the
oracle.  The hand-picked cases of the other files cover the named corners; this one sweeps the
combinations (every case prints its parameters, so a failure names its shape)."""
import numpy as np
import pytest
import torch

from paper_2410_01805_amd import synth
from tests.gpu_util import DEV, assert_close, dev, host, make_layer, make_oracle

pytestmark = pytest.mark.gpu


def _draw(rng, dtype):
    d = int(rng.choice([16, 32, 64, 96, 128] if dtype == "f32" else [64, 96, 128]))
    g = int(rng.choice([1, 2, 3, 4, 8]))
    h_kv = int(rng.choice([1, 2, 3, 4]))
    B = int(rng.integers(40, 400))
    b = int(rng.integers(B // 2 + 8, 3 * B))
    n_s = int(rng.integers(0, min(b, 2 * B) + 1)) if rng.random() < 0.8 else 0
    n_pin = int(rng.integers(0, b - n_s + 1)) if rng.random() < 0.4 else 0
    if dtype == "bf16":
        d_R = int(rng.choice([128, 256]))             # the MFMA retaining head takes multiples of 128 ...
        if rng.random() < 0.3:
            d_R = int(rng.choice([40, 96]))           # ... other widths go through the plain kernel
    else:
        d_R = int(rng.choice([24, 64, 100]))
    rope = bool(rng.random() < 0.7)
    n_chunks = int(rng.integers(3, 7))
    sizes = [int(rng.integers(1, B + 1)) if rng.random() < 0.5 else B for _ in range(n_chunks)]
    return dict(dtype=dtype, h=g * h_kv, h_kv=h_kv, d=d, N=sum(sizes) + 8, B=B, b=b, n_s=n_s, d_R=d_R, rope=rope,
                theta=float(rng.choice([10000.0, 500000.0]))), sizes, n_pin


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("trial", range(16))
def test_random_layer_shapes(dtype, trial):
    rng = np.random.default_rng(1000 * (dtype == "bf16") + trial)
    kw, sizes, n_pin = _draw(rng, dtype)
    print(f"shape {kw} chunks {sizes} n_pin {n_pin}", flush=True)
    w = synth.tiny(name=f"rnd_{dtype}_{trial}", **kw)
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    if n_pin:
        o.n_pin = n_pin
        layer.set_pinned_prefix(n_pin)
    lo = 0
    for step, T in enumerate(sizes):
        q, k, v = synth.tokens(w, lo, lo + T)
        n_c = o.n_c
        out_ref, sc_ref, kept_ref = o.prefill_chunk(q, k, v, w.n_s)
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s,
                                            scores_in=torch.from_numpy(sc_ref).to(DEV))
        tag = f"{w.name} chunk {step}"
        n_keep = min(n_c + T, w.b)
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :n_keep], kept_ref, err_msg=tag)
        assert_close(sc.cpu().numpy(), sc_ref, w.dtype, tag + " scores")
        assert_close(host(out), out_ref, w.dtype, tag + " attention", per_row=True)
        lo += T
    for i in range(min(3, w.b + w.B - o.n_c)):            # a few generated tokens on top
        q, k, v = synth.tokens(w, lo + i, lo + i + 1)
        out_ref, _, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, _ = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=False)
        assert_close(host(out), out_ref, w.dtype, f"{w.name} decode {i}", per_row=True)
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
    layer.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("trial", range(10))
def test_random_layer_shapes_with_head_budgets_and_launch_switches(dtype, trial, monkeypatch):
    """The same sweep with a budget per KV head (caches of different lengths) and, for the matrix-core kernels,
    randomly forced key splits, contraction splits and workgroup orders."""
    from oracle.locret_oracle import LocretLayerOracle
    rng = np.random.default_rng(5000 + 1000 * (dtype == "bf16") + trial)
    kw, sizes, n_pin = _draw(rng, dtype)
    lo_b = max(1, kw["n_s"] + n_pin)
    budgets = [int(rng.integers(lo_b, kw["b"] + 1)) for _ in range(kw["h_kv"])]
    budgets[int(rng.integers(0, kw["h_kv"]))] = kw["b"]          # one head at the config's budget
    env = {}
    for name, choices in (("LOCRET_PP_SPLIT", [None, "2", "3", "5"]), ("LOCRET_SCORE_SPLIT", [None, "0", "2", "3"]),
                          ("LOCRET_PP_SPREAD", [None, "0", "1"]), ("LOCRET_FUSE_SELECT", [None, "0"])):
        c = choices[int(rng.integers(0, len(choices)))]
        if c is not None:
            env[name] = c
            monkeypatch.setenv(name, c)
    print(f"shape {kw} chunks {sizes} n_pin {n_pin} budgets {budgets} env {env}", flush=True)
    w = synth.tiny(name=f"rndhb_{dtype}_{trial}", **kw)
    layer, W1, W2 = make_layer(w)
    layer.set_head_budgets(budgets)
    if n_pin:
        layer.set_pinned_prefix(n_pin)
    o = LocretLayerOracle(w.h, w.h_kv, w.d, budgets, W1, W2, w.rh_kv_expand, w.rope, w.theta, n_pin=n_pin)
    lo = 0
    for step, T in enumerate(sizes):
        q, k, v = synth.tokens(w, lo, lo + T)
        out_ref, sc_ref, kept_ref = o.prefill_chunk(q, k, v, w.n_s)
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s,
                                            scores_in=torch.from_numpy(sc_ref).to(DEV))
        tag = f"{w.name} chunk {step}"
        got = kept.cpu().numpy()
        for m, ref in enumerate(kept_ref):
            np.testing.assert_array_equal(got[m, :len(ref)], ref, err_msg=f"{tag} head {m}")
        assert_close(sc.cpu().numpy(), sc_ref, w.dtype, tag + " scores")
        assert_close(host(out), out_ref, w.dtype, tag + " attention", per_row=True)
        assert layer.cache_lens == [o.n_c_of(m) for m in range(w.h_kv)]
        lo += T
    for i in range(min(2, w.b + w.B - o.n_c)):
        q, k, v = synth.tokens(w, lo + i, lo + i + 1)
        out_ref, _, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, _ = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=False)
        assert_close(host(out), out_ref, w.dtype, f"{w.name} decode {i}", per_row=True)
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        n = o.n_c_of(m)
        np.testing.assert_array_equal(P[m, :n].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m, :n]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m, :n]), o.V[m].astype(np.float32))
    layer.close()
