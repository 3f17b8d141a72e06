"""GPU parity: the whole chunk step (locret_prefill_chunk) and the retaining head (locret_score)
against the oracle on the same seeded inputs.

Teacher-forced runs feed the oracle's float32 scores to the selection, so kept indices must be
bit-exact and the caches identical for the whole stream; attention and the library's own scores
are compared under the tolerance.  Free-running runs let the library select on its own scores;
any unit the two sides disagree on must lie within the score tolerance of the threshold."""
import numpy as np
import pytest
import torch

from paper_2410_01805_amd import synth
from tests.gpu_util import DEV, assert_close, dev, host, make_layer, make_oracle, near_threshold_ok

pytestmark = pytest.mark.gpu


def _run_stream(w, teacher_forced=True, chunk_sizes=None, last_chunk_unmasked=False, attn_rows=None, n_pin=0):
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    if n_pin:
        o.n_pin = n_pin
        layer.set_pinned_prefix(n_pin)
    lo = 0
    sizes = chunk_sizes or [w.B] * w.n_chunks
    diverged = False
    for step, T in enumerate(sizes):
        hi = min(w.N, lo + T)
        if hi <= lo:
            break
        q, k, v = synth.tokens(w, lo, hi)
        n_stab = 0 if (last_chunk_unmasked and hi == w.N) else w.n_s
        n_c = o.n_c
        scat_before = [np.concatenate([o.S[m], np.zeros(hi - lo, np.float32)]) for m in range(w.h_kv)]
        out_ref, sc_ref, kept_ref = o.prefill_chunk(q, k, v, n_stab, attn_rows=attn_rows)
        sin = torch.from_numpy(sc_ref).to(DEV) if teacher_forced else None
        out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), n_stab, scores_in=sin)
        tag = f"{w.name} chunk {step}"
        sc = sc.cpu().numpy()
        assert_close(sc, sc_ref, w.dtype, tag + " scores")
        if not diverged:
            g, r = host(out), out_ref
            if attn_rows is not None:
                g, r = g[attn_rows], r[attn_rows]
            assert_close(g, r, w.dtype, tag + " attention", per_row=True)
        n_keep = min(n_c + (hi - lo), w.b)
        got = kept.cpu().numpy()[:, :n_keep]
        if teacher_forced:
            np.testing.assert_array_equal(got, kept_ref, err_msg=tag)
        else:
            for m in range(w.h_kv):
                scat = scat_before[m]
                scat[n_c:] = sc_ref[m]
                if not np.array_equal(got[m], kept_ref[m]):
                    diverged = True
                    tol = 1e-5 if w.dtype == "f32" else 2e-2
                    assert near_threshold_ok(scat, got[m], kept_ref[m], tol, n_stab, n_pin), tag
            if diverged:
                break
        lo = hi
    return layer, o, diverged


SMALL = [
    dict(name="f32_gqa", dtype="f32", h=8, h_kv=2, d=64, N=1500, B=200, b=400, n_s=32, d_R=64, rope=False),
    dict(name="f32_gqa_expand", dtype="f32", h=8, h_kv=2, d=64, N=900, B=200, b=400, n_s=32, d_R=128, rope=False,
         rh_kv_expand=1),
    dict(name="f32_rope", dtype="f32", h=4, h_kv=2, d=32, N=1200, B=160, b=300, n_s=40, d_R=64, rope=True),
    dict(name="f32_mha_d16", dtype="f32", h=3, h_kv=3, d=16, N=700, B=100, b=150, n_s=0, d_R=40, rope=True),
    dict(name="bf16_llama_like", dtype="bf16", h=8, h_kv=2, d=128, N=2500, B=300, b=700, n_s=100, d_R=128,
         theta=500000.0),
    dict(name="bf16_phi_like", dtype="bf16", h=4, h_kv=4, d=96, N=2000, B=256, b=600, n_s=64, d_R=128),
    dict(name="bf16_d64_norope", dtype="bf16", h=4, h_kv=1, d=64, N=1500, B=250, b=500, n_s=500, d_R=256,
         rope=False),
    dict(name="bf16_ns_gt_B", dtype="bf16", h=4, h_kv=2, d=128, N=1800, B=128, b=640, n_s=300, d_R=128),
]


@pytest.mark.parametrize("kw", SMALL, ids=[c["name"] for c in SMALL])
def test_teacher_forced_stream(kw):
    w = synth.tiny(**kw)
    layer, o, _ = _run_stream(w, teacher_forced=True)
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(S[m].cpu().numpy(), o.S[m])
    layer.close()


@pytest.mark.parametrize("kw", [SMALL[0], SMALL[4]], ids=["f32_gqa", "bf16_llama_like"])
def test_teacher_forced_stream_with_eviction_beside_attention(kw, monkeypatch):
    # LOCRET_OVERLAP=1 is read when the context is created: selection and compaction then run on the
    # library's own stream beside attention; results must not change
    monkeypatch.setenv("LOCRET_OVERLAP", "1")
    w = synth.tiny(**kw)
    layer, o, _ = _run_stream(w, teacher_forced=True)
    K, V, S, P = layer.cache_tensors()
    torch.cuda.synchronize()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
        np.testing.assert_array_equal(host(V[m]), o.V[m].astype(np.float32))
        np.testing.assert_array_equal(S[m].cpu().numpy(), o.S[m])
    layer.close()


def test_teacher_forced_stream_with_pinned_query_prefix():
    # Locret-Q: the first 48 tokens (the query, placed at the start) survive every eviction and keep
    # positions 0..47, so every later chunk attends to them
    w = synth.tiny(name="pinned", dtype="bf16", h=8, h_kv=2, d=128, N=2400, B=300, b=700, n_s=100, d_R=128)
    layer, o, _ = _run_stream(w, teacher_forced=True, n_pin=48)
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
        assert P[m].cpu().numpy()[:48].tolist() == list(range(48))
        np.testing.assert_array_equal(host(K[m]), o.K[m].astype(np.float32))
    layer.close()


@pytest.mark.parametrize("kw", [SMALL[4], SMALL[5], SMALL[7]], ids=["bf16_llama_like", "bf16_phi_like", "bf16_ns_gt_B"])
def test_register_staged_attention_kernel_on_head_dims_128_and_96(kw, monkeypatch):
    # head dims 128 and 96 run on the direct-to-LDS kernel by default; LOCRET_ATTN_VARIANT=regstaged (read when the
    # context is created) sends them to the register-staged kernel that serves head_dim 64 and caches too long for
    # 32-bit offsets; it must meet the same bar
    monkeypatch.setenv("LOCRET_ATTN_VARIANT", "regstaged")
    w = synth.tiny(**kw)
    layer, o, _ = _run_stream(w, teacher_forced=True)
    layer.close()


@pytest.mark.parametrize("n_split", ["2", "3", "8"])
def test_key_split_of_the_head_dim_128_kernel_forced(n_split, monkeypatch):
    # LOCRET_PP_SPLIT=k (read when the context is created) cuts every (head group, token tile) item into k key ranges whose partial
    # results a second kernel merges, whatever the sizes: the first chunks, with fewer key tiles than ranges,
    # leave ranges empty, and in the range that holds the diagonal some wavefronts see no key
    monkeypatch.setenv("LOCRET_PP_SPLIT", n_split)
    for kw in (SMALL[4], SMALL[7]):
        w = synth.tiny(**kw)
        layer, o, _ = _run_stream(w, teacher_forced=True)
        layer.close()


def test_key_split_chosen_for_short_chunks_behind_a_long_cache():
    # 4 items per launch at 128-token chunks: the launcher splits the keys 8 ways once the cache is long enough
    # (every range at least 8 key tiles), and not before; the tail pass of Algorithm 1 (evict = 0) as well
    w = synth.tiny(name="short_chunks", dtype="bf16", h=8, h_kv=2, d=128, N=6 * 1024 + 5 * 128 + 100, B=1024, b=4600,
                   n_s=100, d_R=128)
    sizes = [1024] * 6 + [128] * 5 + [100]
    layer, o, _ = _run_stream(w, teacher_forced=True, chunk_sizes=sizes, last_chunk_unmasked=True)
    K, V, S, P = layer.cache_tensors()
    for m in range(w.h_kv):
        np.testing.assert_array_equal(P[m].cpu().numpy(), o.P[m])
    layer.close()


@pytest.mark.parametrize("n_z", ["0", "2", "5", "8"])
def test_contraction_split_of_the_retaining_head(n_z, monkeypatch):
    # short chunks give the retaining head too few tiles for the CUs; the launcher then slices the
    # contraction and a second kernel sums the slices, applies SiLU and W2 (chosen by itself in most streams of
    # this file).  LOCRET_SCORE_SPLIT (read when the context is created) forces the number of slices, 0 = never.
    monkeypatch.setenv("LOCRET_SCORE_SPLIT", n_z)
    for kw in (SMALL[4], SMALL[5], SMALL[6]):
        w = synth.tiny(**kw)
        layer, o, _ = _run_stream(w, teacher_forced=True)
        layer.close()


@pytest.mark.parametrize("nt,n_z", [("128", "0"), ("128", "3"), ("64", "0"), ("64", "3")])
def test_token_tile_of_the_retaining_head_forced(nt, n_z, monkeypatch):
    # the retaining head takes 64-token tiles for chunks that would leave half of the CUs without a 128-token tile
    # and 128-token tiles otherwise; LOCRET_SCORE_NT (read when the context is created) forces either, here on
    # streams with ragged chunk lengths, with and without the contraction split
    monkeypatch.setenv("LOCRET_SCORE_NT", nt)
    monkeypatch.setenv("LOCRET_SCORE_SPLIT", n_z)
    for kw in (SMALL[4], SMALL[5], SMALL[6]):
        w = synth.tiny(**kw)
        layer, o, _ = _run_stream(w, teacher_forced=True)
        layer.close()


def test_calls_on_a_stream_of_the_callers():
    # every launch of a call goes to the stream the caller passes (the binding passes torch's current stream): a
    # whole teacher-forced stream and the comparisons with the oracle inside a non-default stream
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for kw in (SMALL[0], SMALL[4], SMALL[5]):
            w = synth.tiny(**kw)
            layer, o, _ = _run_stream(w, teacher_forced=True)
            layer.close()
    stream.synchronize()


def test_selection_as_its_own_launch(monkeypatch):
    # by default the head_dim-128 attention launch carries the selection in its first workgroups;
    # LOCRET_FUSE_SELECT=0 (read when the context is created) launches it separately: same kept indices either way
    monkeypatch.setenv("LOCRET_FUSE_SELECT", "0")
    for kw in (SMALL[4], SMALL[7]):
        w = synth.tiny(**kw)
        layer, o, _ = _run_stream(w, teacher_forced=True)
        layer.close()


def test_plain_kernels_on_bf16_storage(monkeypatch):
    # LOCRET_FORCE_SIMPLE=1 (read when the context is created): the fp32 VALU attention and retaining
    # head also serve bf16 tensors
    monkeypatch.setenv("LOCRET_FORCE_SIMPLE", "1")
    w = synth.tiny(**SMALL[4])
    layer, o, _ = _run_stream(w, teacher_forced=True)
    layer.close()


def test_ragged_chunks_and_algorithm1_last_chunk():
    w = synth.tiny(name="ragged", dtype="bf16", h=8, h_kv=2, d=128, N=1500, B=400, b=500, n_s=60, d_R=128)
    layer, o, _ = _run_stream(w, chunk_sizes=[1, 400, 33, 64, 65, 127, 400, 10, 400], last_chunk_unmasked=True)
    assert layer.cache_len == o.n_c == 500
    layer.close()


def test_config1_full_stream_teacher_forced():
    w = synth.WORKLOADS["cfg1_f32_gqa_4k"]
    layer, o, _ = _run_stream(w, teacher_forced=True)
    assert layer.cache_len == w.b
    layer.close()


def test_config1_full_stream_free_running():
    w = synth.WORKLOADS["cfg1_f32_gqa_4k"]
    layer, o, diverged = _run_stream(w, teacher_forced=False)
    layer.close()


def test_free_running_bf16():
    w = synth.tiny(name="free_bf16", dtype="bf16", h=8, h_kv=2, d=128, N=3000, B=512, b=1024, n_s=64, d_R=256)
    layer, o, _ = _run_stream(w, teacher_forced=False)
    layer.close()


def test_score_entry_point_matches_and_leaves_cache_alone():
    for kw in (SMALL[0], SMALL[4]):
        w = synth.tiny(**kw)
        layer, W1, W2 = make_layer(w)
        o = make_oracle(w, W1, W2)
        q, k, v = synth.tokens(w, 0, w.B - 3)
        sc = layer.score(dev(q, w), dev(k, w), dev(v, w)).cpu().numpy()
        assert_close(sc, o.score(q, k, v), w.dtype, w.name + " locret_score")
        assert layer.cache_len == 0
        layer.close()


def test_tail_pass_without_eviction_then_capacity_error():
    from paper_2410_01805_amd import binding as B
    w = synth.tiny(name="tail", dtype="f32", h=4, h_kv=2, d=32, N=600, B=100, b=250, n_s=20, d_R=64, rope=True)
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    for c in range(5):
        q, k, v = synth.chunk(w, c)
        layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s)
        o.prefill_chunk(q, k, v, w.n_s)
    # the n_loc pass of Algorithm 1: attend and append, no eviction
    q, k, v = synth.tokens(w, 500, 560)
    out, sc, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), 0, evict=False)
    out_ref, sc_ref, _ = o.prefill_chunk(q, k, v, 0, evict=False)
    assert kept is None and layer.cache_len == o.n_c == 310
    assert_close(host(out), out_ref, "f32", "tail attention", per_row=True)
    K, V, S, P = layer.cache_tensors()
    np.testing.assert_array_equal(P[0].cpu().numpy(), o.P[0])
    # 310 + 100 > budget + chunk_max = 350
    q, k, v = synth.tokens(w, 0, 100)
    with pytest.raises(B.LocretError) as e:
        layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), 0, evict=False)
    assert e.value.code == B.LOCRET_ESTATE
    layer.close()


def test_state_and_argument_errors_on_device():
    from paper_2410_01805_amd import binding as B
    w = synth.tiny(name="err", dtype="f32", h=4, h_kv=2, d=32, N=600, B=100, b=250, n_s=20, d_R=64)
    layer = B.LocretLayer(B.config_from_workload(w), DEV)
    q, k, v = (dev(x, w) for x in synth.tokens(w, 0, 100))
    with pytest.raises(B.LocretError) as e:       # weights not set
        layer.prefill_chunk(q, k, v, 0)
    assert e.value.code == B.LOCRET_ESTATE
    W1, W2 = synth.weights(w)
    layer.set_weights(dev(W1, w), dev(W2, w))
    with pytest.raises(B.LocretError) as e:       # stabilizers beyond the budget
        layer.prefill_chunk(q, k, v, 251)
    assert e.value.code == B.LOCRET_EINVAL
    q2, k2, v2 = (dev(x, w) for x in synth.tokens(w, 0, 101))
    with pytest.raises(B.LocretError) as e:       # T beyond chunk_max
        layer.prefill_chunk(q2, k2, v2, 0)
    assert e.value.code == B.LOCRET_ESHAPE
    with pytest.raises(B.LocretError) as e:       # misaligned pointer
        B.locret_score(layer.ctx, q.data_ptr() + 4, k, v, 50, torch.empty(2, 50, device=DEV))
    assert e.value.code == B.LOCRET_EALIGN
    assert layer.cache_len == 0                   # nothing was changed by the failed calls
    layer.close()


def test_profile_modes():
    from paper_2410_01805_amd import binding as B
    w = synth.tiny(name="prof", dtype="bf16", h=8, h_kv=2, d=128, N=1200, B=300, b=700, n_s=50, d_R=128)
    layer, _, _ = make_layer(w)
    chunks = [tuple(dev(x, w) for x in synth.chunk(w, c)) for c in range(4)]
    for mode in (0, 1, 2):
        layer.reset()
        B.locret_profile_mode(layer.ctx, mode)
        B.locret_profile_enable(layer.ctx, 3)            # the 4th call is not recorded
        for q, k, v in chunks:
            layer.prefill_chunk(q, k, v, w.n_s)
        with pytest.raises(B.LocretError) as e:          # recorded calls are still unread
            B.locret_profile_mode(layer.ctx, (mode + 1) % 3)
        assert e.value.code == B.LOCRET_ESTATE
        ms, n = B.locret_profile_read(layer.ctx)
        assert n == 3 and 0.0 < ms[1] < 50.0             # attention was timed
        if mode == 0:
            assert all(x > 0.0 for x in ms)              # every stage (compaction ran from the third chunk on)
        elif mode == 1:
            assert ms[0] == ms[2] == ms[3] == ms[4] == 0.0
        else:
            # through the kernels' own dispatches: the selection rides in the attention launch here, so its entry is 0
            assert ms[0] > 0.0 and ms[2] > 0.0 and ms[4] > 0.0 and ms[3] == 0.0
        B.locret_profile_enable(layer.ctx, 0)
    with pytest.raises(B.LocretError):
        B.locret_profile_mode(layer.ctx, 3)
    layer.close()


@pytest.mark.parametrize("n_s", [24, 23], ids=["fits_the_fused_selection", "one_candidate_too_many"])
def test_selection_inside_attention_at_its_size_limit(n_s):
    # the head_dim-128 attention launch carries the selection while a wavefront's share of the candidates fits
    # 48 rounds of 64 (24576 per head); one candidate more and the step launches the separate kernel (here its
    # keys-in-LDS form).  Same kept indices either way; the oracle only scores and evicts (teacher-forced).
    w = synth.tiny(name=f"sel_limit_{n_s}", dtype="bf16", h=4, h_kv=1, d=128, N=6 * 4600, B=4600, b=20000, n_s=n_s,
                   d_R=128)
    layer, W1, W2 = make_layer(w)
    o = make_oracle(w, W1, W2)
    for c in range(6):
        q, k, v = synth.chunk(w, c)
        sc_ref = o.score(q, k, v)
        n_c = o.n_c
        kept_ref = o.evict_compact(sc_ref, k, v, w.n_s)
        _, _, kept = layer.prefill_chunk(dev(q, w), dev(k, w), dev(v, w), w.n_s, scores_in=torch.from_numpy(sc_ref).to(DEV))
        n_keep = min(n_c + w.B, w.b)
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :n_keep], kept_ref, err_msg=f"chunk {c}")
    assert o.n_c == layer.cache_len == w.b
    K, V, S, P = layer.cache_tensors()
    np.testing.assert_array_equal(P[0].cpu().numpy(), o.P[0])
    layer.close()
