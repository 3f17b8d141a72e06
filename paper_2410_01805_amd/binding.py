"""ctypes binding of liblocret.so (the C ABI of include/locret.h), same names, marshalling only.

PyTorch supplies device memory and streams; every step of the chunk path runs in the library's
HIP kernels.  Importing this module fails loudly if the library has not been built
(python -m paper_2410_01805_amd.build, or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes as C
import os

# PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  It must be in the process before
# liblocret.so is opened so that the dynamic loader binds the library to that same runtime:
# two runtimes in one process do not share device allocations or streams.
import torch  # noqa: F401  (memory and streams come from here as well)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "liblocret.so")

LOCRET_OK, LOCRET_EINVAL, LOCRET_ESHAPE, LOCRET_EALIGN, LOCRET_ESTATE, LOCRET_EHIP, LOCRET_ENOMEM, LOCRET_ELIMIT = 0, -1, -2, -3, -4, -5, -6, -7
LOCRET_F32, LOCRET_BF16 = 0, 1

EXPORTS = [
    "locret_workspace_bytes", "locret_create", "locret_set_weights", "locret_set_pinned_prefix", "locret_reset", "locret_prefill_chunk",
    "locret_score", "locret_decode_step", "locret_evict_compact", "locret_cache_len", "locret_tokens_seen", "locret_cache_view",
    "locret_destroy", "locret_strerror", "locret_profile_mode", "locret_profile_enable", "locret_profile_read",
    "locret_set_head_budgets", "locret_cache_lens", "locret_score_static", "locret_cache_view_q4",
]
LOCRET_PROF_STAGES = 5
LOCRET_MAX_HEAD_BUDGETS = 64
PROF_STAGE_NAMES = ("append", "attention", "retaining_head", "select", "compact")


class locret_config(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("chunk_max", C.c_int32),
        ("budget", C.c_int32), ("d_hidden", C.c_int32), ("rh_kv_expand", C.c_int32), ("dtype", C.c_int32),
        ("rope_mode", C.c_int32), ("rope_theta", C.c_float), ("softmax_scale", C.c_float), ("kv_bits", C.c_int32),
    ]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build the HIP library first "
                          "(python -m paper_2410_01805_amd.build); there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    vp, i32, f32p, i32p = C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p
    lib.locret_workspace_bytes.restype = C.c_size_t
    lib.locret_workspace_bytes.argtypes = [C.POINTER(locret_config)]
    lib.locret_create.restype = C.c_int
    lib.locret_create.argtypes = [C.POINTER(locret_config), vp, C.c_size_t, C.POINTER(vp)]
    lib.locret_set_weights.restype = C.c_int
    lib.locret_set_weights.argtypes = [vp, vp, vp, vp]
    lib.locret_reset.restype = C.c_int
    lib.locret_reset.argtypes = [vp]
    lib.locret_prefill_chunk.restype = C.c_int
    lib.locret_prefill_chunk.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32p, vp, f32p, i32p, vp]
    lib.locret_score.restype = C.c_int
    lib.locret_score.argtypes = [vp, vp, vp, vp, i32, f32p, vp]
    lib.locret_score_static.restype = C.c_int
    lib.locret_score_static.argtypes = [vp, vp, vp, vp, i32, f32p, vp]
    lib.locret_decode_step.restype = C.c_int
    lib.locret_decode_step.argtypes = [vp, vp, vp, vp, i32, vp, f32p, vp]
    lib.locret_evict_compact.restype = C.c_int
    lib.locret_evict_compact.argtypes = [vp, f32p, vp, vp, i32, i32, i32p, vp]
    lib.locret_profile_mode.restype = C.c_int
    lib.locret_profile_mode.argtypes = [vp, i32]
    lib.locret_set_pinned_prefix.restype = C.c_int
    lib.locret_set_pinned_prefix.argtypes = [vp, i32]
    lib.locret_set_head_budgets.restype = C.c_int
    lib.locret_set_head_budgets.argtypes = [vp, C.POINTER(i32)]
    lib.locret_cache_lens.restype = C.c_int
    lib.locret_cache_lens.argtypes = [vp, C.POINTER(i32)]
    lib.locret_cache_len.restype = C.c_int32
    lib.locret_cache_len.argtypes = [vp]
    lib.locret_tokens_seen.restype = C.c_int64
    lib.locret_tokens_seen.argtypes = [vp]
    lib.locret_cache_view.restype = C.c_int
    lib.locret_cache_view.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                      C.POINTER(i32), C.POINTER(i32)]
    lib.locret_cache_view_q4.restype = C.c_int
    lib.locret_cache_view_q4.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(i32), C.POINTER(i32),
                                         C.POINTER(i32), C.POINTER(i32)]
    lib.locret_profile_enable.restype = C.c_int
    lib.locret_profile_enable.argtypes = [vp, i32]
    lib.locret_profile_read.restype = C.c_int
    lib.locret_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
    lib.locret_destroy.restype = None
    lib.locret_destroy.argtypes = [vp]
    lib.locret_strerror.restype = C.c_char_p
    lib.locret_strerror.argtypes = [C.c_int]
    return lib


lib = _load()


class LocretError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {locret_strerror(code)} ({code})")


def _check(code: int, where: str) -> None:
    if code != LOCRET_OK:
        raise LocretError(code, where)


def _ptr(t) -> int | None:
    """Device address of a torch tensor (None -> NULL); ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors cross the boundary as dense row-major buffers"
    return t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ---- the C ABI, one Python function per entry point -------------------------------------------------
def locret_strerror(code: int) -> str:
    return lib.locret_strerror(code).decode()


def locret_workspace_bytes(cfg: locret_config) -> int:
    return lib.locret_workspace_bytes(C.byref(cfg) if cfg is not None else None)


def locret_create(cfg: locret_config, workspace, workspace_bytes: int | None = None) -> int:
    handle = C.c_void_p()
    nbytes = workspace_bytes if workspace_bytes is not None else (
        workspace.numel() * workspace.element_size() if workspace is not None and not isinstance(workspace, int) else 0)
    _check(lib.locret_create(C.byref(cfg) if cfg is not None else None, _ptr(workspace), nbytes, C.byref(handle)),
           "locret_create")
    return handle.value


def locret_set_weights(ctx, W1, W2, stream=None) -> None:
    _check(lib.locret_set_weights(ctx, _ptr(W1), _ptr(W2), _stream(stream)), "locret_set_weights")


def locret_reset(ctx) -> None:
    _check(lib.locret_reset(ctx), "locret_reset")


def locret_prefill_chunk(ctx, q, k, v, T, n_stab, evict, scores_in, attn_out, scores_out, kept_idx_out,
                         stream=None) -> None:
    _check(lib.locret_prefill_chunk(ctx, _ptr(q), _ptr(k), _ptr(v), T, n_stab, evict, _ptr(scores_in),
                                    _ptr(attn_out), _ptr(scores_out), _ptr(kept_idx_out), _stream(stream)),
           "locret_prefill_chunk")


def locret_profile_mode(ctx, mode: int) -> None:
    _check(lib.locret_profile_mode(ctx, mode), "locret_profile_mode")


def locret_set_pinned_prefix(ctx, n_pin: int) -> None:
    _check(lib.locret_set_pinned_prefix(ctx, n_pin), "locret_set_pinned_prefix")


def locret_set_head_budgets(ctx, budgets) -> None:
    """budgets: a sequence of n_kv_heads ints (host), or None for the config's single budget."""
    arr = None if budgets is None else (C.c_int32 * len(budgets))(*[int(b) for b in budgets])
    _check(lib.locret_set_head_budgets(ctx, arr), "locret_set_head_budgets")


def locret_cache_lens(ctx, n_kv_heads: int) -> list:
    arr = (C.c_int32 * n_kv_heads)()
    _check(lib.locret_cache_lens(ctx, arr), "locret_cache_lens")
    return list(arr)


def locret_decode_step(ctx, q, k, v, with_score, attn_out, scores_out=None, stream=None) -> None:
    _check(lib.locret_decode_step(ctx, _ptr(q), _ptr(k), _ptr(v), 1 if with_score else 0, _ptr(attn_out),
                                  _ptr(scores_out), _stream(stream)), "locret_decode_step")


def locret_score(ctx, q, k, v, T, scores, stream=None) -> None:
    _check(lib.locret_score(ctx, _ptr(q), _ptr(k), _ptr(v), T, _ptr(scores), _stream(stream)), "locret_score")


def locret_score_static(ctx, q, k, v, T, scores, stream=None) -> None:
    _check(lib.locret_score_static(ctx, _ptr(q), _ptr(k), _ptr(v), T, _ptr(scores), _stream(stream)),
           "locret_score_static")


def locret_evict_compact(ctx, chunk_scores, k_chunk, v_chunk, T, n_stab, kept_idx_out, stream=None) -> None:
    _check(lib.locret_evict_compact(ctx, _ptr(chunk_scores), _ptr(k_chunk), _ptr(v_chunk), T, n_stab,
                                    _ptr(kept_idx_out), _stream(stream)), "locret_evict_compact")


def locret_cache_len(ctx) -> int:
    return lib.locret_cache_len(ctx)


def locret_tokens_seen(ctx) -> int:
    return lib.locret_tokens_seen(ctx)


def locret_cache_view(ctx) -> dict:
    K, V, S, P = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
    n, stride = C.c_int32(), C.c_int32()
    _check(lib.locret_cache_view(ctx, C.byref(K), C.byref(V), C.byref(S), C.byref(P), C.byref(n), C.byref(stride)),
           "locret_cache_view")
    return dict(K=K.value, V=V.value, score=S.value, orig_pos=P.value, len=n.value, row_stride=stride.value)


def locret_cache_view_q4(ctx) -> dict:
    Kq, Vq = C.c_void_p(), C.c_void_p()
    n, stride, rb, rsb = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib.locret_cache_view_q4(ctx, C.byref(Kq), C.byref(Vq), C.byref(n), C.byref(stride), C.byref(rb), C.byref(rsb)),
           "locret_cache_view_q4")
    return dict(Kq=Kq.value, Vq=Vq.value, len=n.value, row_stride=stride.value, row_bytes=rb.value,
                row_stride_bytes=rsb.value)


def locret_profile_enable(ctx, max_calls: int) -> None:
    _check(lib.locret_profile_enable(ctx, max_calls), "locret_profile_enable")


def locret_profile_read(ctx):
    """(per-stage milliseconds summed over the recorded calls, number of calls)."""
    ms = (C.c_double * LOCRET_PROF_STAGES)()
    n = C.c_int32()
    _check(lib.locret_profile_read(ctx, ms, C.byref(n)), "locret_profile_read")
    return list(ms), n.value


def locret_destroy(ctx) -> None:
    lib.locret_destroy(ctx)


# ---- convenience: config from a synth.Workload, a context that owns its workspace tensor -----------------
def config_from_workload(w) -> locret_config:
    return locret_config(w.h, w.h_kv, w.d, w.B, w.b, w.d_R, w.rh_kv_expand,
                         LOCRET_BF16 if w.dtype == "bf16" else LOCRET_F32, 1 if w.rope else 0,
                         float(w.theta) if w.rope else 0.0, 0.0, getattr(w, "kv_bits", 0))


class LocretLayer:
    """Owns a workspace tensor and a context; methods forward to the C ABI (no arithmetic here)."""

    def __init__(self, cfg: locret_config, device="cuda:0"):
        import torch
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = locret_workspace_bytes(cfg)
        if nbytes == 0:
            raise LocretError(LOCRET_EINVAL, "locret_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.ctx = locret_create(cfg, self.workspace)
        self.tdtype = torch.bfloat16 if cfg.dtype == LOCRET_BF16 else torch.float32

    def set_weights(self, W1, W2):
        locret_set_weights(self.ctx, W1, W2)

    def reset(self):
        locret_reset(self.ctx)

    def prefill_chunk(self, q, k, v, n_stab, evict=True, scores_in=None, want_scores=True, want_kept=True):
        import torch
        T = q.shape[0]
        out = torch.empty_like(q)
        sc = torch.empty((self.cfg.n_kv_heads, T), dtype=torch.float32, device=self.device) if want_scores else None
        kept = torch.full((self.cfg.n_kv_heads, self.cfg.budget), -1, dtype=torch.int32, device=self.device) \
            if (want_kept and evict) else None
        locret_prefill_chunk(self.ctx, q, k, v, T, n_stab, 1 if evict else 0, scores_in, out, sc, kept)
        return out, sc, kept

    def score(self, q, k, v):
        import torch
        T = q.shape[0]
        sc = torch.empty((self.cfg.n_kv_heads, T), dtype=torch.float32, device=self.device)
        locret_score(self.ctx, q, k, v, T, sc)
        return sc

    def set_pinned_prefix(self, n_pin: int) -> None:
        locret_set_pinned_prefix(self.ctx, n_pin)

    def set_head_budgets(self, budgets) -> None:
        if budgets is not None and len(budgets) != self.cfg.n_kv_heads:
            raise LocretError(LOCRET_EINVAL, "locret_set_head_budgets")
        locret_set_head_budgets(self.ctx, budgets)

    @property
    def cache_lens(self) -> list:
        return locret_cache_lens(self.ctx, self.cfg.n_kv_heads)

    def decode_step(self, q, k, v, with_score=False):
        """One generated token: q [1][h][d], k, v [1][h_kv][d] -> (attn_out [1][h][d], scores [h_kv] or None)."""
        import torch
        out = torch.empty_like(q)
        sc = torch.empty((self.cfg.n_kv_heads,), dtype=torch.float32, device=self.device) if with_score else None
        locret_decode_step(self.ctx, q, k, v, with_score, out, sc)
        return out, sc

    def evict_compact(self, scores, k, v, n_stab):
        import torch
        kept = torch.full((self.cfg.n_kv_heads, self.cfg.budget), -1, dtype=torch.int32, device=self.device)
        locret_evict_compact(self.ctx, scores, k, v, k.shape[0], n_stab, kept)
        return kept

    @property
    def cache_len(self) -> int:
        return locret_cache_len(self.ctx)

    def cache_tensors(self):
        """Copies of the live cache (K, V in storage dtype, score float32, orig_pos int32), each
        [h_kv][len][...], taken from the workspace through locret_cache_view (with head-wise budgets
        len is the longest head's: row m is meaningful up to cache_lens[m])."""
        import torch
        view = locret_cache_view(self.ctx)
        base = self.workspace.data_ptr()
        h_kv, d, n, stride = self.cfg.n_kv_heads, self.cfg.head_dim, view["len"], view["row_stride"]
        es = 2 if self.cfg.dtype == LOCRET_BF16 else 4

        def grab(addr, dtype, inner, esize):
            off = addr - base
            raw = self.workspace[off: off + h_kv * stride * inner * esize].view(dtype)
            return raw.view(h_kv, stride, inner)[:, :n].clone()
        K = grab(view["K"], self.tdtype, d, es) if view["K"] else None
        V = grab(view["V"], self.tdtype, d, es)
        S = grab(view["score"], torch.float32, 1, 4)[..., 0]
        P = grab(view["orig_pos"], torch.int32, 1, 4)[..., 0]
        if self.cfg.kv_bits:
            # packed rows instead of K, V: uint8 [h_kv][len][row_bytes] (padding bytes dropped)
            vq = locret_cache_view_q4(self.ctx)
            rb, rsb = vq["row_bytes"], vq["row_stride_bytes"]
            Kq = grab(vq["Kq"], torch.uint8, rsb, 1)[..., :rb].contiguous()
            Vq = grab(vq["Vq"], torch.uint8, rsb, 1)[..., :rb].contiguous()
            return Kq, Vq, S, P
        return K, V, S, P

    def close(self):
        if self.ctx:
            locret_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
