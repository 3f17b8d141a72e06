#!/usr/bin/env python3
"""Benchmark of the Locret chunk step on one MI355X.

A step is one locret_prefill_chunk call (attention + retaining head + select + compact) on one
chunk of the synthetic 128K-token stream.  The timed region is exactly K consecutive steps that start
from an empty cache at chunk 0 and wrap to a new pass (empty cache again) after the last chunk; K
defaults to one whole pass (32 chunks), and then `value` is whole-stream prefill tokens/s per layer
at 131072 tokens.  For any other K the line says which tokens were timed (`config.tokens`,
`config.chunks_timed`) and carries figures that do not depend on K: `whole_stream` (one complete pass,
timed on its own) and `steady_state` (steps with the cache at its budget).  Inputs are generated on
the host from the seeded recipe and are resident in HBM before the clock starts.  SETTLE_STEPS untimed steps run
in front of the W warm-up steps (`settle_steps` in the line): a GPU that idled through the input generation needs
more than a handful of calls before its clocks settle.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
SETTLE_STEPS = 64             # untimed steps in front of the warm-up steps (clocks and caches of an idle GPU)
PEAK_F32_TFLOPS = 157.3



def measured_attention_traffic(workload_name):
    """(HBM bytes of one steady-state attention launch, source) from the committed rocprofv3 counter summary
    of this workload (profiles/chunk_step_<workload>_hbm_traffic.txt: FETCH_SIZE and WRITE_SIZE, scaled by what
    the same counters read for a plain copy), or (None, None) when no summary covers the workload.  It is a
    figure measured in those profiling runs, not in this run."""
    rel = os.path.join("profiles", f"chunk_step_{workload_name}_hbm_traffic.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        if line.startswith("locret::attn_") and "merge" not in line:
            try:
                return float(line.split()[-1]) * 1e6, rel + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, separate runs)"
            except ValueError:
                return None, None
    return None, None


def attention_flops(w, n_c, T):
    """QK^T + PV over the keys each query really sees (cache + causal part of the chunk)."""
    return 4.0 * w.h * w.d * (T * n_c + T * (T + 1) / 2.0)


def score_flops(w, T):
    K = (w.h + 2 * w.h_kv) * w.d
    return 2.0 * T * K * w.d_R + 2.0 * T * w.d_R * w.h_kv


def evict_bytes(w, n_c, T):
    """scores in; kept scores + positions out; K and V rows read and written once; rotated-K shadow written."""
    s = 2 if w.dtype == "bf16" else 4
    L = n_c + T
    n_keep = min(L, w.b)
    moved = n_keep if L > w.b else 0
    return w.h_kv * (L * 4 + n_keep * 8 * (1 if moved else 0) + 4 * moved * w.d * s + (moved * w.d * s if w.rope else 0))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="cfg3_llama_128k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-head-budgets", action="store_true",
                    help="skip the head-wise-budget leg (profiling runs: keeps the launch counts those of the chunk step)")
    ap.add_argument("--no-quant", action="store_true", help="skip the 4-bit-cache-rows leg")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain elementwise pass over 256 MiB (read 256 MiB, write 256 MiB): the "
                         "reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="measured HBM bytes per steady-state attention launch (from the counter runs), "
                         "reported as roofline.traffic")
    ap.add_argument("--cpu-rows", type=int, default=600, help="query rows per head in the oracle's attention sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus above 1 is not supported (no collectives are built)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2410_01805_amd import binding as B
    from paper_2410_01805_amd import synth

    w = synth.WORKLOADS[args.workload]
    n_chunks = w.n_chunks
    K = args.steps if args.steps is not None else n_chunks
    if K < 1:
        print("bench.py: --steps must be at least 1", file=sys.stderr)
        sys.exit(2)
    W = args.warmup
    dev = torch.device("cuda:0")
    td = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    # ---- inputs: generated per chunk on host threads, uploaded, resident before timing ------------------
    need = n_chunks                      # the whole stream: the K-independent figures need every chunk
    t_gen = time.time()
    with ThreadPoolExecutor(max_workers=min(16, len(os.sched_getaffinity(0)))) as ex:
        host_chunks = list(ex.map(lambda c: synth.chunk(w, c), range(need)))
    chunks = [tuple(torch.from_numpy(x).to(dev).to(td).contiguous() for x in hc) for hc in host_chunks]
    W1h, W2h = synth.weights(w)
    layer = B.LocretLayer(B.config_from_workload(w), dev)
    layer.set_weights(torch.from_numpy(W1h).to(dev).to(td), torch.from_numpy(W2h).to(dev).to(td))
    out = torch.empty((w.B, w.h, w.d), dtype=td, device=dev)
    scores = torch.empty((w.h_kv, w.B), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen

    def step(i):
        c = i % need
        if c == 0:
            B.locret_reset(layer.ctx)
        q, k, v = chunks[c]
        T = q.shape[0]
        B.locret_prefill_chunk(layer.ctx, q, k, v, T, w.n_s, 1, None, out, scores, None)
        return T

    # The GPU has idled through the input generation above; its clocks and caches need more than a handful of
    # calls to settle (measured: 32 timed steps behind 8 untimed ones run 2 % slower than the same steps behind
    # 72).  So a fixed number of untimed steps precedes the W warm-up steps, whatever W is.
    for i in range(SETTLE_STEPS):
        step(i)
    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    if args.calibrate:
        x = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        y = torch.empty_like(x)
        torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        del x, y

    # ---- timed region ---------------------------------------------------------------------------------
    # Inside it only the dominant kernel (attention) is timed, through its own dispatch, which puts no
    # extra packets into the stream; the other stages are timed in a second pass over the same steps below
    # (with the selection as a kernel of its own, which the timed region does not have).
    B.locret_reset(layer.ctx)
    B.locret_profile_mode(layer.ctx, 1)
    B.locret_profile_enable(layer.ctx, K)
    plan = []           # (n_c before the call, T) per timed step, for the work model
    n_c = 0
    for i in range(K):
        c = i % need
        if c == 0:
            n_c = 0
        T = chunks[c][0].shape[0]
        plan.append((n_c, T))
        n_c = min(n_c + T, w.b)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    tokens = 0
    for i in range(K):
        tokens += step(i)
    e1.record()
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)
    attn_ms, n_attn = B.locret_profile_read(layer.ctx)
    B.locret_profile_enable(layer.ctx, 0)

    # ---- figures that do not depend on K ------------------------------------------------------------------
    # (a) one complete pass over the stream from an empty cache, timed on its own the same way
    plan_full = []
    n_c = 0
    for c in range(n_chunks):
        T = chunks[c][0].shape[0]
        plan_full.append((n_c, T))
        n_c = min(n_c + T, w.b)
    B.locret_profile_enable(layer.ctx, n_chunks)
    f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    f0.record()
    for c in range(n_chunks):
        step(c)
    f1.record()
    torch.cuda.synchronize()
    full_ms = f0.elapsed_time(f1)
    full_attn_ms, n_full = B.locret_profile_read(layer.ctx)
    # (b) steady state: the cache is at its budget after that pass; the stream's last full chunk again and again
    c_steady = max(c for c in range(n_chunks) if chunks[c][0].shape[0] == w.B)
    qs, ks, vs = chunks[c_steady]
    n_steady = 20
    steady_possible = B.locret_cache_len(layer.ctx) == w.b
    for _ in range(2):
        B.locret_prefill_chunk(layer.ctx, qs, ks, vs, w.B, w.n_s, 1, None, out, scores, None)
    B.locret_profile_enable(layer.ctx, n_steady)
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s0.record()
    for _ in range(n_steady):
        B.locret_prefill_chunk(layer.ctx, qs, ks, vs, w.B, w.n_s, 1, None, out, scores, None)
    s1.record()
    torch.cuda.synchronize()
    steady_ms = s0.elapsed_time(s1) / n_steady
    steady_attn_ms, n_st = B.locret_profile_read(layer.ctx)
    B.locret_profile_enable(layer.ctx, 0)

    # ---- second pass over the same steps, every stage timed (not part of `value`) ------------------------
    # In the timed region the selection rides in the first workgroups of the attention launch; here a second
    # context, created with LOCRET_FUSE_SELECT=0 (the library reads its launch switches when a context is
    # created), launches it on its own so that it has a duration of its own: the stage figures below are
    # those of the separate kernels.
    fuse_before = os.environ.get("LOCRET_FUSE_SELECT")
    os.environ["LOCRET_FUSE_SELECT"] = "0"
    layer_st = B.LocretLayer(B.config_from_workload(w), dev)
    if fuse_before is None:
        del os.environ["LOCRET_FUSE_SELECT"]
    else:
        os.environ["LOCRET_FUSE_SELECT"] = fuse_before
    layer_st.set_weights(torch.from_numpy(W1h).to(dev).to(td), torch.from_numpy(W2h).to(dev).to(td))

    def step_st(i):
        c = i % need
        if c == 0:
            B.locret_reset(layer_st.ctx)
        q, k, v = chunks[c]
        B.locret_prefill_chunk(layer_st.ctx, q, k, v, q.shape[0], w.n_s, 1, None, out, scores, None)

    B.locret_profile_mode(layer_st.ctx, 2)      # every stage through its kernels' own dispatches: pure kernel durations
    for i in range(min(K, 6)):           # untimed: the selection kernels are loaded on their first launch
        step_st(i)
    torch.cuda.synchronize()
    B.locret_profile_enable(layer_st.ctx, K)
    for i in range(K):
        step_st(i)
    torch.cuda.synchronize()
    stage_ms, n_prof = B.locret_profile_read(layer_st.ctx)
    B.locret_profile_enable(layer_st.ctx, 0)
    layer_st.close()
    del layer_st
    stage_ms = list(stage_ms)
    if n_attn == K:                      # the live figure of the timed region (else: a kernel that is timed with events)
        stage_ms[1] = attn_ms[1]

    fl_attn = sum(attention_flops(w, nc, T) for nc, T in plan)
    fl_score = sum(score_flops(w, T) for nc, T in plan)
    by_evict = sum(evict_bytes(w, nc, T) for nc, T in plan)
    ms = dict(zip(B.PROF_STAGE_NAMES, stage_ms))
    peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_F32_TFLOPS
    attn_tflops = fl_attn / (ms["attention"] * 1e-3) / 1e12
    traffic, traffic_source = measured_attention_traffic(w.name)
    if args.traffic_bytes is not None:
        traffic, traffic_source = args.traffic_bytes, "--traffic-bytes"
    steady_attn_tflops = (attention_flops(w, w.b, w.B) * n_steady / (steady_attn_ms[1] * 1e-3) / 1e12
                          if (n_st == n_steady and steady_possible) else None)
    roofline = {
        "kernel": "attention", "bound": "mfma", "achieved": round(attn_tflops, 2), "peak": peak, "unit": "TFLOP/s",
        "frac": round(attn_tflops / peak, 4),
        "steady_achieved": round(steady_attn_tflops, 2) if steady_attn_tflops else None,
        "steady_frac": round(steady_attn_tflops / peak, 4) if steady_attn_tflops else None,
        "steady_launch_ms": round(steady_attn_ms[1] / n_steady, 4) if steady_attn_tflops else None,
        "traffic": traffic, "traffic_source": traffic_source,
        "algorithmic_bytes_steady": (2 * w.h_kv * (w.b + w.B) + 2 * w.B * w.h) * w.d * (2 if w.dtype == "bf16" else 4),
        "avg_launch_ms": round(ms["attention"] / max(1, n_prof), 4),
        "timed_by": "kernel dispatch timestamps, inside the timed region" if n_attn == K else "events around the launch, second pass",
        "flops_per_launch_steady": attention_flops(w, w.b, w.B),
    }
    mlp_tflops = fl_score / (ms["retaining_head"] * 1e-3) / 1e12
    evict_ms = ms["select"] + ms["compact"]
    evict_gbs = by_evict / (evict_ms * 1e-3) / 1e9 if evict_ms > 0 else 0.0
    # in the step as it runs (timed region) only the compaction's own time is exposed: the same bytes over that
    compact_gbs = by_evict / (ms["compact"] * 1e-3) / 1e9 if ms["compact"] > 0 else 0.0
    # the library carries the selection inside the attention launch for bf16 head dims 128 and 96 while the
    # candidates of a head fit the register-resident form (24576)
    sel_fused = fuse_before != "0" and w.dtype == "bf16" and w.d in (96, 128) and (w.b + w.B - w.n_s) <= 24576
    extra = {
        "stage_ms_per_step": {k: round(v / max(1, n_prof), 4) for k, v in ms.items()},
        "retaining_head": {"achieved": round(mlp_tflops, 2), "unit": "TFLOP/s", "frac": round(mlp_tflops / peak, 4)},
        "attention_plus_retaining_head_frac": round((fl_attn + fl_score) / ((ms["attention"] + ms["retaining_head"]) * 1e-3) / 1e12 / peak, 4),
        "select_compact": {"bound": "hbm", "achieved": round(evict_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": round(evict_gbs / PEAK_HBM_GBS, 4),
                           **({"in_step": {"achieved": round(compact_gbs, 1), "frac": round(compact_gbs / PEAK_HBM_GBS, 4),
                                           "what": "the same bytes over the compaction kernel's time alone, which is what "
                                                   "the step spends on the pair when the selection rides in the attention launch"}}
                              if sel_fused else {}),
                           "note": "both as kernels of their own (second pass); in the timed region the selection runs "
                                   "inside the attention launch" if sel_fused else "both as kernels of their own"},
        "input_gen_s": round(t_gen, 1),
        "whole_stream": {"tokens": w.N, "steps": n_chunks, "ms": round(full_ms, 3),
                         "tokens_per_s": round(w.N / (full_ms * 1e-3), 1),
                         "attention_frac": (round(sum(attention_flops(w, nc, T) for nc, T in plan_full)
                                                  / (full_attn_ms[1] * 1e-3) / 1e12 / peak, 4) if n_full == n_chunks else None)},
        "steady_state": ({"n_c": w.b, "T": w.B, "steps": n_steady, "ms_per_step": round(steady_ms, 4),
                          "tokens_per_s": round(w.B / (steady_ms * 1e-3), 1)} if steady_possible else None),
    }

    # ---- decode step (Eq. 1 with B = 1): one generated token over the full budget ----------
    # the cache is at the budget after the timed region; 64 generated tokens, plain generation (no score)
    n_dec = min(64, w.B)
    q1 = chunks[0][0][:1].contiguous(); k1 = chunks[0][1][:1].contiguous(); v1 = chunks[0][2][:1].contiguous()
    o1 = torch.empty_like(q1)
    for _ in range(8):
        B.locret_decode_step(layer.ctx, q1, k1, v1, 0, o1, None)
    d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_units = B.locret_cache_len(layer.ctx)
    torch.cuda.synchronize()
    d0.record()
    for _ in range(n_dec):
        B.locret_decode_step(layer.ctx, q1, k1, v1, 0, o1, None)
    d1.record()
    torch.cuda.synchronize()
    dec_ms = d0.elapsed_time(d1) / n_dec
    es = 2 if w.dtype == "bf16" else 4
    dec_bytes = 2 * w.h_kv * (n_units + n_dec / 2) * w.d * es          # one pass over (rotated) K and V
    dec_gbs = dec_bytes / (dec_ms * 1e-3) / 1e9
    extra["decode_step"] = {"units": n_units, "ms_per_token": round(dec_ms, 4), "bound": "hbm",
                            "achieved": round(dec_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": round(dec_gbs / PEAK_HBM_GBS, 4), "timed": "split-K attention (rotates the query, appends the token) + merge"}

    # ---- head-wise budgets (one budget per KV head): the same layer with a pyramid of budgets of the
    # same total, steady state (every head at its budget), against equal budgets measured the same way
    import dataclasses

    def steady_ms(lay, n_fill, n_timed=20):
        qc, kc, vc = chunks[min(1, need - 1)]
        for _ in range(n_fill):
            B.locret_prefill_chunk(lay.ctx, qc, kc, vc, qc.shape[0], w.n_s, 1, None, out, scores, None)
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        s0.record()
        for _ in range(n_timed):
            B.locret_prefill_chunk(lay.ctx, qc, kc, vc, qc.shape[0], w.n_s, 1, None, out, scores, None)
        s1.record()
        torch.cuda.synchronize()
        return s0.elapsed_time(s1) / n_timed

    if w.h_kv >= 2 and w.h_kv <= B.LOCRET_MAX_HEAD_BUDGETS and not args.no_head_budgets:
        B.locret_reset(layer.ctx)                               # the decode steps above left it over its budget
        equal_ms = steady_ms(layer, (w.b + w.B - 1) // w.B + 4)
        lo_b = max(w.n_s, w.b // 4)
        pyr = [int(round(lo_b + (2 * w.b - 2 * lo_b) * (w.h_kv - 1 - m) / (w.h_kv - 1))) for m in range(w.h_kv)]
        pyr[-1] += w.h_kv * w.b - sum(pyr)                      # exactly the same total
        lay2 = B.LocretLayer(B.config_from_workload(dataclasses.replace(w, b=max(pyr))), dev)
        lay2.set_weights(torch.from_numpy(W1h).to(dev).to(td), torch.from_numpy(W2h).to(dev).to(td))
        lay2.set_head_budgets(pyr)
        pyr_ms = steady_ms(lay2, (max(pyr) + w.B - 1) // w.B + 4)
        assert lay2.cache_lens == pyr
        lay2.close()
        extra["head_budgets"] = {"budgets": pyr, "steady_ms_per_step": round(pyr_ms, 4),
                                 "equal_budgets_steady_ms_per_step": round(equal_ms, 4),
                                 "tokens_per_s": round(w.B / (pyr_ms * 1e-3), 1)}

    # ---- 4-bit cache rows (the appendix's combination with KV-cache quantization): the same layer with
    # kv_bits = 4, steady state; stage figures are pure kernel durations (profile mode 2)
    if w.dtype == "bf16" and w.d in (64, 96, 128) and not args.no_quant:
        wq = dataclasses.replace(w, kv_bits=4)
        cfgq = B.config_from_workload(wq)
        layq = B.LocretLayer(cfgq, dev)
        layq.set_weights(torch.from_numpy(W1h).to(dev).to(td), torch.from_numpy(W2h).to(dev).to(td))
        q_ms = steady_ms(layq, (w.b + w.B - 1) // w.B + 4)
        B.locret_profile_mode(layq.ctx, 2)
        B.locret_profile_enable(layq.ctx, 20)
        steady_ms(layq, 0)
        qst, nq = B.locret_profile_read(layq.ctx)
        B.locret_profile_enable(layq.ctx, 0)
        for _ in range(8):
            B.locret_decode_step(layq.ctx, q1, k1, v1, 0, o1, None)
        dq0, dq1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        dq0.record()
        for _ in range(n_dec):
            B.locret_decode_step(layq.ctx, q1, k1, v1, 0, o1, None)
        dq1.record()
        torch.cuda.synchronize()
        layq.close()
        rowb = w.d // 2 + 4 * (w.d // 32)
        # per unit: packed K, V rows read and written, staging K, V rows written, score + position read and written, index read
        cq_bytes = w.h_kv * w.b * (4 * rowb + 2 * w.d * 2 + 16 + 4)
        cq_ms = qst[4] / max(1, nq)
        extra["quantized_rows"] = {
            "kv_bits": 4, "row_bytes": rowb, "steady_ms_per_step": round(q_ms, 4),
            "tokens_per_s": round(w.B / (q_ms * 1e-3), 1),
            "stage_ms_per_step": {k: round(v / max(1, nq), 4) for k, v in zip(B.PROF_STAGE_NAMES, qst)},
            "compact": {"algorithmic_bytes": cq_bytes, "achieved": round(cq_bytes / (cq_ms * 1e-3) / 1e9, 1) if cq_ms > 0 else None,
                        "unit": "GB/s", "frac": round(cq_bytes / (cq_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if cq_ms > 0 else None,
                        "bytes_vs_bf16_rows": round(cq_bytes / (w.h_kv * w.b * (5 * w.d * 2 + 16 + 4)), 3)},
            "decode_ms_per_token": round(dq0.elapsed_time(dq1) / n_dec, 4),
            "workspace_bytes": B.locret_workspace_bytes(cfgq), "workspace_bytes_bf16_rows": B.locret_workspace_bytes(B.config_from_workload(w)),
        }

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, host_chunks, args.cpu_rows)

    line = {
        "metric": "prefill tokens/sec per layer at 128K ctx", "value": round(tokens / (total_ms * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "settle_steps": SETTLE_STEPS, "ms_per_step": round(total_ms / K, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "tokens": tokens, "stream_tokens": w.N,
                   "chunks_timed": (f"{K // n_chunks} whole pass(es) of {n_chunks} chunks" if K % n_chunks == 0 else
                                    f"{K // n_chunks} whole pass(es) + chunks 0-{K % n_chunks - 1} of {n_chunks}, each pass from an empty cache"),
                   "chunk": w.B, "budget": w.b, "stabilizers": w.n_s,
                   "heads": f"{w.h}q/{w.h_kv}kv x{w.d}", "d_R": w.d_R},
        "roofline": roofline, "cpu_baseline": cpu, **extra,
    }
    print(json.dumps(line))


def cpu_baseline(w, host_chunks, rows_per_head):
    """The oracle, as it stands, on one steady-state chunk of the same workload: retaining head,
    selection and compaction in full; attention on a sample of query rows (rows are independent),
    extrapolated linearly to the whole chunk from two sample sizes."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle.locret_oracle import LocretLayerOracle
    from paper_2410_01805_amd import synth

    W1, W2 = synth.weights(w)
    o = LocretLayerOracle(w.h, w.h_kv, w.d, w.b, W1, W2, w.rh_kv_expand, w.rope, w.theta)
    # fill the cache to the budget with the first chunks (scores come from the oracle itself; untimed)
    c = 0
    while o.n_c < w.b and c < len(host_chunks) - 1:
        q, k, v = host_chunks[c]
        o.prefill_chunk(q, k, v, w.n_s, want_attn=False)
        c += 1
    q, k, v = host_chunks[c]
    T = q.shape[0]
    rng = np.random.default_rng(0)
    r1 = np.sort(rng.choice(T, size=min(T, rows_per_head), replace=False))
    r2 = np.sort(rng.choice(T, size=min(T, 3 * rows_per_head), replace=False))
    t0 = time.time(); o.attention(q, k, v, rows=r1); t1 = time.time()
    o.attention(q, k, v, rows=r2); t2 = time.time()
    ta, tb = t1 - t0, t2 - t1
    per_row = max(0.0, (tb - ta) / max(1, len(r2) - len(r1)))
    fixed = max(0.0, ta - per_row * len(r1))
    t_attn_full = fixed + per_row * T if len(r1) < T else ta
    t3 = time.time()
    sc = o.score(q, k, v)
    o.evict_compact(sc, k, v, w.n_s)
    t_rest = time.time() - t3
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    # the small configuration (config 1: float32 inputs, 4096 tokens as 8 chunks of 512) through the oracle in full
    w1 = synth.WORKLOADS["cfg1_f32_gqa_4k"]
    W1a, W2a = synth.weights(w1)
    o1 = LocretLayerOracle(w1.h, w1.h_kv, w1.d, w1.b, W1a, W2a, w1.rh_kv_expand, w1.rope, w1.theta)
    c1 = [synth.chunk(w1, c) for c in range(w1.n_chunks)]
    t4 = time.time()
    for q1, k1, v1 in c1:
        o1.prefill_chunk(q1, k1, v1, w1.n_s)
    t_cfg1 = time.time() - t4
    return {
        "config1_full_stream": {"workload": w1.name, "tokens": w1.N, "seconds": round(t_cfg1, 3),
                                "tokens_per_s": round(w1.N / t_cfg1, 1)},
        "value": round(T / (t_attn_full + t_rest), 1), "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": f"one steady-state chunk (n_c={w.b}, T={T}): retaining head + select + compact in full "
                  f"({t_rest:.2f}s); attention on {len(r1)} and {len(r2)} query rows x {w.h} heads "
                  f"({ta:.2f}s, {tb:.2f}s), extrapolated linearly to {T} rows ({t_attn_full:.1f}s)",
    }


if __name__ == "__main__":
    main()
