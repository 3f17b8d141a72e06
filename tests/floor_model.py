"""Error floor of Eq. 1 (Section 3.1) on bf16 matrix cores, for setting test tolerances.

Not an oracle and not the product: the chunk attention evaluated in float64 with ONLY the operand
roundings that bf16 matrix-core arithmetic forces on any kernel, whatever its design:
  * the rotated, pre-scaled query and the rotated key are matrix operands, so each is rounded to bf16 once;
  * the probabilities are the left operand of the P V product, so they are rounded to bf16 (the normaliser
    is summed from the unrounded values);
  * the output is stored as bf16.
Products and sums are exact (float64).  The difference between this and the oracle is the part of a
kernel's error that belongs to the arithmetic; what a kernel adds on top is its own.
"""
from __future__ import annotations

import numpy as np

from oracle.locret_oracle import rope_rotate
from paper_2410_01805_amd import synth

LOG2E = 1.4426950408889634


def bf16(x: np.ndarray) -> np.ndarray:
    return synth.bf16_to_f32(synth.bf16_bits(np.asarray(x, dtype=np.float32))).astype(np.float64)


def floor_attention(o, q, k, v, rows, heads, round_qk=True, round_p=True, round_out=True) -> dict:
    """{query head j: out[len(rows)][d]} for the oracle state `o` (cache before the chunk) and the chunk q, k, v."""
    T = q.shape[0]
    rows = np.asarray(rows)
    out = {}
    for j in heads:
        m = j // o.g
        n_c = o.n_c_of(m)
        keys = np.concatenate([o.K[m], np.asarray(k[:, m, :], dtype=np.float64)], axis=0)
        vals = np.concatenate([o.V[m], np.asarray(v[:, m, :], dtype=np.float64)], axis=0)
        qj = np.asarray(q[rows, j, :], dtype=np.float64)
        if o.rope:
            keys = rope_rotate(keys, np.arange(n_c + T), o.theta)
            qj = rope_rotate(qj, n_c + rows, o.theta)
        qj = qj * (o.scale * LOG2E)
        if round_qk:
            keys, qj = bf16(keys), bf16(qj)
        s = qj @ keys.T
        visible = np.arange(n_c + T)[None, :] <= (n_c + rows)[:, None]
        s = np.where(visible, s, -np.inf)
        s -= s.max(axis=1, keepdims=True)
        p = np.exp2(s)
        den = p.sum(axis=1, keepdims=True)
        if round_p:
            p = bf16(p)
        r = (p @ vals) / den
        out[j] = bf16(r) if round_out else r
    return out


def ratio_to_unit_bound(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """|got - ref| over the element-wise bf16 bound of the GPU tests at kappa = 1: 2e-2 |ref| + 2e-2 rms(row)."""
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    return np.abs(got - ref) / (2e-2 * np.abs(ref) + 2e-2 * rms)
