"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/locret.h declares, and turns bad arguments into error codes before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2410_01805_amd import binding as B
from paper_2410_01805_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "locret.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(locret_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert sorted(B.EXPORTS) == names
    for n in names:
        assert getattr(B.lib, n) is not None


def _cfg(**kw):
    base = dict(n_q_heads=8, n_kv_heads=2, head_dim=64, chunk_max=512, budget=1024, d_hidden=256, rh_kv_expand=1,
                dtype=B.LOCRET_F32, rope_mode=0, rope_theta=0.0, softmax_scale=0.0)
    base.update(kw)
    return B.locret_config(**base)


def test_workspace_bytes_covers_both_cache_copies():
    cfg = _cfg()
    n = B.locret_workspace_bytes(cfg)
    cap = 1024 + 512
    two_copies_kv = 2 * 2 * (2 * cap * 64 * 4)
    assert n >= two_copies_kv and n < 4 * two_copies_kv
    w = synth.WORKLOADS["cfg3_llama_128k"]
    n3 = B.locret_workspace_bytes(B.config_from_workload(w))
    cap3 = w.b + w.B
    assert n3 >= 2 * 3 * (8 * cap3 * 128 * 2)           # K, V and the rotated shadow, two copies
    assert n3 < 1 << 30


BAD = [
    dict(n_q_heads=0), dict(n_kv_heads=0), dict(n_q_heads=8, n_kv_heads=3), dict(head_dim=80), dict(head_dim=0),
    dict(chunk_max=0), dict(budget=0), dict(d_hidden=0), dict(dtype=2), dict(rope_mode=2), dict(rh_kv_expand=5),
    dict(rope_mode=1, rope_theta=0.0), dict(rope_mode=1, rope_theta=-3.0), dict(softmax_scale=-1.0),
    dict(softmax_scale=float("nan")), dict(budget=1 << 30),
]


@pytest.mark.parametrize("kw", BAD)
def test_bad_config_is_rejected_on_the_host(kw):
    cfg = _cfg(**kw)
    assert B.locret_workspace_bytes(cfg) == 0
    h = C.c_void_p()
    rc = B.lib.locret_create(C.byref(cfg), 0x1000, 1 << 40, C.byref(h))
    assert rc in (B.LOCRET_EINVAL, B.LOCRET_ESHAPE)
    assert h.value is None


def test_create_argument_errors():
    cfg = _cfg()
    h = C.c_void_p()
    assert B.lib.locret_create(None, 0x1000, 1 << 40, C.byref(h)) == B.LOCRET_EINVAL
    assert B.lib.locret_create(C.byref(cfg), None, 1 << 40, C.byref(h)) == B.LOCRET_EINVAL
    assert B.lib.locret_create(C.byref(cfg), 0x1000, 1 << 40, None) == B.LOCRET_EINVAL
    assert B.lib.locret_create(C.byref(cfg), 0x1010, 1 << 40, C.byref(h)) == B.LOCRET_EALIGN
    assert B.lib.locret_create(C.byref(cfg), 0x1000, 16, C.byref(h)) == B.LOCRET_ENOMEM
    assert B.locret_workspace_bytes(None) == 0


def test_null_context_is_an_error_everywhere():
    assert B.lib.locret_reset(None) == B.LOCRET_EINVAL
    assert B.lib.locret_set_weights(None, 16, 16, None) == B.LOCRET_EINVAL
    assert B.lib.locret_prefill_chunk(None, 16, 16, 16, 1, 0, 1, None, 16, None, None, None) == B.LOCRET_EINVAL
    assert B.lib.locret_score(None, 16, 16, 16, 1, 16, None) == B.LOCRET_EINVAL
    assert B.lib.locret_evict_compact(None, 16, 16, 16, 1, 0, None, None) == B.LOCRET_EINVAL
    assert B.lib.locret_cache_len(None) == B.LOCRET_EINVAL
    assert B.lib.locret_set_head_budgets(None, None) == B.LOCRET_EINVAL
    assert B.lib.locret_cache_lens(None, None) == B.LOCRET_EINVAL
    assert B.lib.locret_cache_view(None, None, None, None, None, None, None) == B.LOCRET_EINVAL
    B.lib.locret_destroy(None)


def test_strerror_names_every_code():
    seen = set()
    for code in range(0, -7, -1):
        s = B.locret_strerror(code)
        assert s and s != "unknown error code"
        seen.add(s)
    assert len(seen) == 7
    assert B.locret_strerror(-99) == "unknown error code"
    with pytest.raises(B.LocretError) as e:
        B._check(B.LOCRET_ESTATE, "x")
    assert e.value.code == B.LOCRET_ESTATE
