"""locret_score_static (the entry point that allocates nothing: its kernels' scratch is a fixed array inside
the library's device code) against locret_score, through the C ABI.

Both run the same kernels in the same order, so the scores must be bit-identical; two calls in a row, the
second on a smaller input, check that nothing left in the shared array by the first call leaks into the
second.  Sizes beyond the array are rejected on the host."""
import numpy as np
import pytest
import torch

from paper_2410_01805_amd import binding as B
from paper_2410_01805_amd import synth
from tests.gpu_util import DEV, dev, make_layer

pytestmark = pytest.mark.gpu


def _scores_both_ways(layer, w, q, k, v):
    T = q.shape[0]
    dq, dk, dv = dev(q, w), dev(k, w), dev(v, w)
    ref = torch.full((w.h_kv, T), float("nan"), dtype=torch.float32, device=DEV)
    got = torch.full((w.h_kv, T), float("nan"), dtype=torch.float32, device=DEV)
    stream = torch.cuda.current_stream().cuda_stream or None
    rc = B.lib.locret_score(layer.ctx, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), T, ref.data_ptr(), stream)
    assert rc == B.LOCRET_OK
    rc = B.lib.locret_score_static(layer.ctx, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), T, got.data_ptr(), stream)
    assert rc == B.LOCRET_OK
    torch.cuda.synchronize()
    return got.cpu().numpy(), ref.cpu().numpy()


CASES = [
    # (workload kwargs, T of the first call, T of the second, smaller, call)
    (dict(dtype="bf16", h=32, h_kv=8, d=128, B=4096, b=4096, d_R=1024), 4096, 1000),   # full tiles, then a split contraction
    (dict(dtype="bf16", h=32, h_kv=32, d=96, B=3072, b=3072, d_R=1024), 3000, 130),    # ragged tiles, 32 score columns
    (dict(dtype="f32", h=8, h_kv=2, d=64, B=512, b=1024, d_R=256), 512, 77),           # float32 kernels
]


@pytest.mark.parametrize("kw,T1,T2", CASES)
def test_static_scratch_scores_equal_workspace_scores_two_calls(kw, T1, T2):
    w = synth.tiny(name="static", N=kw["B"], n_s=0, theta=10000.0, **kw)
    layer, W1, W2 = make_layer(w)
    q, k, v = synth.tokens(w, 0, T1)
    got1, ref1 = _scores_both_ways(layer, w, q, k, v)
    assert np.isfinite(ref1).all()
    np.testing.assert_array_equal(got1.view(np.uint32), ref1.view(np.uint32))
    q, k, v = synth.tokens(w, T1, T1 + T2)
    got2, ref2 = _scores_both_ways(layer, w, q, k, v)
    assert np.isfinite(ref2).all()
    np.testing.assert_array_equal(got2.view(np.uint32), ref2.view(np.uint32))
    layer.close()


def test_static_scratch_limit_and_argument_errors():
    # 64 hidden blocks x 8 heads x 4096 tokens = 2 Mi partial scores: beyond the array
    w = synth.tiny(name="static_big", dtype="bf16", h=8, h_kv=8, d=64, N=4096, B=4096, b=4096, n_s=0, d_R=8192,
                   theta=10000.0)
    layer, W1, W2 = make_layer(w)
    q, k, v = synth.tokens(w, 0, 4096)
    dq, dk, dv = dev(q, w), dev(k, w), dev(v, w)
    sc = torch.zeros((w.h_kv, 4096), dtype=torch.float32, device=DEV)
    call = B.lib.locret_score_static
    assert call(layer.ctx, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), 4096, sc.data_ptr(), None) == B.LOCRET_ELIMIT
    assert b"static scratch" in B.lib.locret_strerror(B.LOCRET_ELIMIT)
    # half the tokens fit exactly, and agree with the workspace path
    h2 = [x[:2048].contiguous() for x in (dq, dk, dv)]
    sc2 = torch.zeros((w.h_kv, 2048), dtype=torch.float32, device=DEV)
    assert call(layer.ctx, h2[0].data_ptr(), h2[1].data_ptr(), h2[2].data_ptr(), 2048, sc2.data_ptr(), None) == B.LOCRET_OK
    ref = layer.score(*h2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(sc2.cpu().numpy().view(np.uint32), ref.cpu().numpy().view(np.uint32))
    assert call(layer.ctx, None, dk.data_ptr(), dv.data_ptr(), 16, sc.data_ptr(), None) == B.LOCRET_EINVAL
    assert call(layer.ctx, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), 0, sc.data_ptr(), None) == B.LOCRET_ESHAPE
    assert call(layer.ctx, dq.data_ptr() + 2, dk.data_ptr(), dv.data_ptr(), 16, sc.data_ptr(), None) == B.LOCRET_EALIGN
    layer.close()
    cfg = B.config_from_workload(w)
    ws = torch.empty(B.locret_workspace_bytes(cfg), dtype=torch.uint8, device=DEV)
    ctx = B.locret_create(cfg, ws)
    assert call(ctx, dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), 16, sc.data_ptr(), None) == B.LOCRET_ESTATE   # no weights
    B.locret_destroy(ctx)
