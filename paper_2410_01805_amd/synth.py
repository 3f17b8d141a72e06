"""Seeded synthetic inputs for the Locret chunk step (workload shapes + tensors).

This module is the only code shared by the GPU path's tests/bench and the CPU
oracle's tests.  It holds no arithmetic of the method itself: only a
counter-based random generator, the workload table, and bf16 rounding of the
generated values (a storage-format conversion).

Every value is a pure function of (seed, tensor id, flat element index), so any
chunk of a stream can be generated on its own, in any order, on any machine.

Workloads follow the layer shapes of the two backbones the paper evaluates
(Section 4 "Experiments": an MHA model with 32 heads of 96 and a GQA model with
32 query / 8 KV heads of 128) and the scale of its inference hyper-parameters
(Appendix A.2, the table of b, B, n_s, n_loc).  The paper's own prompts come
from public long-context benchmarks; these seeded Gaussians stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from functools import lru_cache

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)

# tensor ids (mixed into the hash so tensors are independent streams)
TID_Q, TID_K, TID_V, TID_W1, TID_W2, TID_PLANT = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" or "bf16": storage type of q, k, v, W, out, cache
    h: int                # query heads
    h_kv: int             # KV heads (h % h_kv == 0)
    d: int                # head dim
    N: int                # tokens in the stream
    B: int                # chunk size
    b: int                # cache budget, units per KV head
    n_s: int              # stabilizer length
    d_R: int              # retaining-head hidden width
    rh_kv_expand: int     # 0: d_in = (h + 2 h_kv) d ; 1: d_in = 3 h d (K, V blocks repeated g times)
    rope: bool
    theta: float
    seed: int
    planted_frac: float = 0.0   # fraction of positions whose keys are scaled
    planted_scale: float = 1.0
    w_std: float = 0.02
    kv_bits: int = 0            # 0: cache rows as given; 4: 4-bit cache rows

    @property
    def g(self) -> int:
        return self.h // self.h_kv

    @property
    def d_in(self) -> int:
        return 3 * self.h * self.d if self.rh_kv_expand else (self.h + 2 * self.h_kv) * self.d

    @property
    def n_chunks(self) -> int:
        return (self.N + self.B - 1) // self.B

    def chunk_range(self, c: int) -> tuple[int, int]:
        lo = c * self.B
        return lo, min(self.N, lo + self.B)


_SEED0 = 20241001

WORKLOADS: dict[str, Workload] = {
    # the five named benchmark configurations
    "cfg1_f32_gqa_4k": Workload("cfg1_f32_gqa_4k", "f32", 8, 2, 64, 4096, 512, 1024, 64, 256, 1,
                                False, 0.0, _SEED0 + 1),
    "cfg2_llama_32k": Workload("cfg2_llama_32k", "bf16", 32, 8, 128, 32768, 2048, 6144, 2048, 1024, 0,
                               True, 500000.0, _SEED0 + 2),
    "cfg3_llama_128k": Workload("cfg3_llama_128k", "bf16", 32, 8, 128, 131072, 4096, 16384, 2048, 1024, 0,
                                True, 500000.0, _SEED0 + 3, planted_frac=0.01, planted_scale=4.0),
    "cfg4_phi3_128k": Workload("cfg4_phi3_128k", "bf16", 32, 32, 96, 131072, 4096, 8192, 1024, 1024, 0,
                               True, 10000.0, _SEED0 + 4),
    "cfg5_stream_1m": Workload("cfg5_stream_1m", "bf16", 32, 8, 128, 1048576, 4096, 8192, 2048, 1024, 0,
                               True, 500000.0, _SEED0 + 5),
    # the paper's own inference settings (Appendix "Hyperparameters, Environment and Baselines", inference
    # table: budget b, chunk B, stabilizers n_s) on the two backbones' layer shapes, 128K tokens
    "paper_llama31_row": Workload("paper_llama31_row", "bf16", 32, 8, 128, 131072, 1024, 16384, 2500, 1024, 0,
                                  True, 500000.0, _SEED0 + 6),
    "paper_phi3_row": Workload("paper_phi3_row", "bf16", 32, 32, 96, 131072, 3072, 6000, 2500, 1024, 0,
                               True, 10000.0, _SEED0 + 7),
}


def tiny(name: str = "tiny", **kw) -> Workload:
    """A small workload for tests; any field can be overridden."""
    base = Workload(name, "f32", 4, 2, 16, 96, 16, 24, 4, 32, 0, True, 10000.0, 7)
    return replace(base, **kw)


# ----------------------------------------------------------------------------
# counter-based generator
# ----------------------------------------------------------------------------

def _mix(x: np.ndarray) -> np.ndarray:
    """64-bit finaliser (xor-shift-multiply), elementwise on uint64."""
    x = x.copy()
    x ^= x >> np.uint64(30)
    x *= np.uint64(0xBF58476D1CE4E5B9)
    x ^= x >> np.uint64(27)
    x *= np.uint64(0x94D049BB133111EB)
    x ^= x >> np.uint64(31)
    return x


def _stream_key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.array([(seed * 0x9E3779B97F4A7C15 + tensor_id * 0xD1B54A32D192ED03) & 0xFFFFFFFFFFFFFFFF],
                     dtype=np.uint64)
        return _mix(k)[0]


def hash_u64(seed: int, tensor_id: int, start: int, count: int, lane: int = 0) -> np.ndarray:
    """uint64 hash of flat indices [start, start+count) of one tensor stream."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        key = _stream_key(seed, tensor_id * 2 + lane)
        return _mix((idx * np.uint64(0x9E3779B97F4A7C15)) ^ key)


def standard_normal(seed: int, tensor_id: int, start: int, count: int) -> np.ndarray:
    """float64 N(0,1) samples for flat indices [start, start+count) (Box-Muller, one per index)."""
    h1 = hash_u64(seed, tensor_id, start, count, 0)
    h2 = hash_u64(seed, tensor_id, start, count, 1)
    u1 = ((h1 >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)  # (0, 1]
    u2 = (h2 >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)          # [0, 1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)


# ----------------------------------------------------------------------------
# bf16 storage rounding
# ----------------------------------------------------------------------------

def bf16_bits(x32: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def storage_round(x64: np.ndarray, dtype: str) -> np.ndarray:
    """Values as the chosen storage type holds them, returned as float32."""
    x32 = x64.astype(np.float32)
    if dtype == "bf16":
        return bf16_to_f32(bf16_bits(x32))
    return x32


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------

@lru_cache(maxsize=8)
def planted_positions(w: Workload) -> np.ndarray:
    """Sorted token positions whose keys are scaled: the floor(frac*N) smallest hash keys."""
    n = int(np.floor(w.planted_frac * w.N))
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    keys = hash_u64(w.seed, TID_PLANT, 0, w.N)
    pos = np.argpartition(keys, n - 1)[:n]
    return np.sort(pos.astype(np.int64))


def tokens(w: Workload, lo: int, hi: int):
    """q [T][h][d], k [T][h_kv][d], v [T][h_kv][d] for tokens [lo, hi): float32 arrays holding
    values exactly representable in w.dtype.  q and k are NOT rotated (no RoPE applied)."""
    T = hi - lo
    q = standard_normal(w.seed, TID_Q, lo * w.h * w.d, T * w.h * w.d).reshape(T, w.h, w.d)
    k = standard_normal(w.seed, TID_K, lo * w.h_kv * w.d, T * w.h_kv * w.d).reshape(T, w.h_kv, w.d)
    v = standard_normal(w.seed, TID_V, lo * w.h_kv * w.d, T * w.h_kv * w.d).reshape(T, w.h_kv, w.d)
    if w.planted_frac > 0.0:
        pp = planted_positions(w)
        sel = pp[(pp >= lo) & (pp < hi)] - lo
        k[sel] *= w.planted_scale
    return storage_round(q, w.dtype), storage_round(k, w.dtype), storage_round(v, w.dtype)


def chunk(w: Workload, c: int):
    lo, hi = w.chunk_range(c)
    return tokens(w, lo, hi)


def weights(w: Workload):
    """W1 [d_in][d_R], W2 [d_R][h_kv] ~ N(0, w_std^2), float32 holding w.dtype-representable values."""
    W1 = standard_normal(w.seed, TID_W1, 0, w.d_in * w.d_R).reshape(w.d_in, w.d_R) * w.w_std
    W2 = standard_normal(w.seed, TID_W2, 0, w.d_R * w.h_kv).reshape(w.d_R, w.h_kv) * w.w_std
    return storage_round(W1, w.dtype), storage_round(W2, w.dtype)
