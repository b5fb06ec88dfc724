#!/usr/bin/env python3
"""Benchmark of the SWA decode hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch: append, scores,
softmax, importance accumulation, selection, sparse output and in-place
compaction, for all b*h (sequence, head) pairs of one layer.  By default that is
ONE kernel (swa_decode_step with SWA_FUSE_COMPACTION | SWA_UNORDERED); --step-mode
fused keeps the cache in token order, --step-mode split runs swa_decode_step
followed by swa_compact_kv.

The job is the workload's decode trajectory from the prompt on (the step right
after the prompt, which evicts most of the prompt, then the steady state with
compaction every step).  To keep the data HBM-cold the way a multi-layer model
does, R independent replicas of the layer state are stepped round-robin (replica
= one layer's cache): step i works on replica i % R at trajectory step i // R.  R
follows from BYTES, never from --steps: the R consecutive steps of one sweep
must touch at least SWEEP_MIN_BYTES of distinct cache (four times the 256 MB
Infinity Cache), and R >= 2.  Inputs are resident in HBM before the timed
region starts.

Without --steps the timed region is whole trajectories on every replica (the
step after the prompt at its true weight, 1 of 512).  With --steps K --warmup W
the schedule's first W steps run untimed and the next K are timed: a short
stretch of the steady state (W >= R puts every replica's step after the prompt
into the warm-up); the whole-trajectory figures, with the first step's own rate,
are printed beside it in `whole_trajectory`.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
SWEEP_MIN_BYTES = 1 << 30   # distinct bytes one sweep over the replicas must touch (4 x the Infinity Cache)
HEADLINE = "c5_llama7b_sp80"   # the largest single-GPU workload (b = 256, mixed prompts 512..2048)


def simulate_lengths(B, wl, lens, compact_every=1):
    """Host-side replay of the budget: per step, cached length m and kept count per sequence.
    The cache shrinks to the kept set only on the steps that compact (every step by default;
    0 = never)."""
    cur = list(lens)
    ms, keeps = [], []
    for t in range(wl.steps):
        m_t, k_t = [], []
        for s, L in enumerate(cur):
            n = lens[s] + t + 1
            m = L + 1
            keep, _, _ = B.swa_budget(n, m, wl.w, wl.sparsity_bp)
            m_t.append(m)
            k_t.append(keep)
            cur[s] = keep if (compact_every > 0 and (t + 1) % compact_every == 0) else m
        ms.append(m_t)
        keeps.append(k_t)
    return ms, keeps


def torch_zeros(shape, device):
    import torch
    return torch.zeros(shape, dtype=torch.float32, device=device)


class Replica:
    """One layer's device state plus the per-step logical lengths."""

    def __init__(self, B, W, wl, prompt, torch, len_bounds, fused, kv_int8=False, compact_every=1, split_rows=False):
        self.compact_every = compact_every
        self.fused = bool(fused)
        flags = {False: 0, True: B.SWA_FUSE_COMPACTION, "fused": B.SWA_FUSE_COMPACTION, "split": 0,
                 "unordered": B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED,
                 "shared": B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED | B.SWA_HEAD_SHARED,
                 "window": B.SWA_FUSE_COMPACTION | B.SWA_UNORDERED}[fused]
        if split_rows:
            assert flags == 0, "SWA_SPLIT_ROWS goes with the two-call form"
            flags = B.SWA_SPLIT_ROWS
        self.window_rows = min(max(wl.w, 1), B.SWA_MAX_WINDOW_ROWS) if fused == "window" else 0
        self.ring = None
        self.fused = (flags & B.SWA_FUSE_COMPACTION) != 0
        params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype, flags=flags)
        st = B.DecodeState(params, device="cuda", debug_probs=False)
        st.K.copy_(prompt["K"])
        st.V.copy_(prompt["V"])
        st.pos.copy_(prompt["pos"])
        st.cache_len.copy_(prompt["cache_len"])
        self.st = st
        base = prompt["cache_len"].to(torch.int32)
        self.seq_lens = torch.stack([base + (t + 1) for t in range(wl.steps)]).contiguous()  # [T, b]
        # per-step params: the host knows an upper bound on the cached length of every step
        self.kv_int8 = kv_int8
        self.B = B
        qf = B.SWA_KV_INT8 if kv_int8 else 0
        self.params = [B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype,
                                     len_bound=lb, flags=flags | qf) for lb in len_bounds]

    def finish_prompt(self, q_tail):
        """End of the prompt: importance seed (if the workload has one), then KV compression."""
        if self.window_rows:
            st, R = self.st, self.window_rows
            self.ring = torch_zeros((st.K.shape[0], st.K.shape[1], R, st.K.shape[2]), st.K.device)
            if q_tail is not None:
                self.B.swa_prefill_rows(st.params, q_tail[:, :, -R:].contiguous(), R, st.K, st.cache_len, self.ring,
                                        st.workspace)
        elif q_tail is not None:
            self.st.prefill_scores(q_tail)
        if self.kv_int8:
            self.st.quantize()

    def decode(self, B, t, q, kn, vn):
        st = self.st
        if self.fused:
            # one kernel: the new lengths come back in kept_cnt, so the two arrays alternate
            self._call(B, t, q, kn, vn, None)
            st.cache_len, st.kept_cnt = st.kept_cnt, st.cache_len
        else:
            self._call(B, t, q, kn, vn, st.kept_idx)

    def _call(self, B, t, q, kn, vn, kept_idx):
        st = self.st
        if self.window_rows:
            B.swa_decode_step_window(self.params[t], q, kn, vn, st.K, st.V, self.ring, self.window_rows,
                                     t % self.window_rows, st.score, st.pos, st.cache_len, self.seq_lens[t],
                                     kept_idx, st.kept_cnt, st.out, None, st.workspace)
        elif self.kv_int8:
            B.swa_decode_step_q8(self.params[t], q, kn, vn, st.K, st.V, st.qparams, st.score, st.pos,
                                 st.cache_len, self.seq_lens[t], kept_idx, st.kept_cnt, st.out, None,
                                 st.workspace)
        else:
            B.swa_decode_step(self.params[t], q, kn, vn, st.K, st.V, st.score, st.pos, st.cache_len,
                              self.seq_lens[t], kept_idx, st.kept_cnt, st.out, None, st.workspace)

    def compact(self, B, t):
        st = self.st
        if not self.fused and self.compact_every > 0 and (t + 1) % self.compact_every == 0:
            B.swa_compact_kv(self.params[t], st.K, st.V, st.score, st.pos, st.kept_idx, st.kept_cnt,
                             st.cache_len, st.workspace)

    def step(self, B, t, q, kn, vn):
        self.decode(B, t, q, kn, vn)
        self.compact(B, t)


_PROMPTS = {}


def prompt_of(wl, W):
    """Prompt state of a workload; the three sparsities of config 5 share one prompt."""
    key = (wl.config_id, wl.seed, wl.b, wl.h, wl.d, wl.dtype, wl.prompt_lo, wl.prompt_hi, wl.steps, wl.w, wl.hh_frac)
    if key not in _PROMPTS:
        _PROMPTS.clear()                      # one prompt resident at a time (config 5: 10 GB)
        _PROMPTS[key] = W.make_prompt(wl, "cuda")
    return _PROMPTS[key]


# Device memory stays with torch's caching allocator for the whole process: a serving stack allocates its
# caches once, and memory handed back to the driver and acquired again between workloads measured 1.5-3 %
# slower on this GPU than the blocks of the first allocation.


def replicas_for(step_bytes):
    """Replica count from bytes alone: the R steps of one sweep touch R x (one step's working set) of
    distinct memory, which must reach SWEEP_MIN_BYTES even for the lightest step; at least two."""
    return max(2, math.ceil(SWEEP_MIN_BYTES / max(1, min(step_bytes))))


def bench_workload(wl, steps, warmup, mode, torch, B, W, fused=True, want_kernel_times=True, kv_int8=False,
                   compact_every=1, split_rows=False):
    """Times `steps` decode steps (None = whole trajectories on every replica) after `warmup` untimed ones."""
    dev = "cuda"
    T = wl.steps
    prompt = prompt_of(wl, W)
    lens = prompt["lengths"]
    inputs = [W.make_step(wl, t, prompt["mu"]) for t in range(T)]
    q_tail = W.make_q_tail(wl, prompt["mu"], wl.prefill_R) if wl.prefill_R > 0 else None
    ms, keeps = simulate_lengths(B, wl, lens, compact_every)
    len_bounds = [max(m_t) for m_t in ms]
    window_rows = min(max(wl.w, 1), B.SWA_MAX_WINDOW_ROWS) if fused == "window" else 0

    def abp(m, k):
        return W.algorithmic_bytes_per_pair(wl.d, wl.elem_bytes, m, k, kv_int8, window_rows)

    step_bytes = [sum(wl.h * abp(m, k) for m, k in zip(ms[t], keeps[t])) for t in range(T)]
    R = replicas_for(step_bytes)
    whole = steps is None
    if whole:
        # whole trajectories, from the prompt on, on every replica; the warm-up runs on replicas of its own
        steps, start = T * R, 0
        warmup = min(warmup, T * R)
    else:
        # one continuous job: the `warmup` untimed steps are the FIRST steps of the same round-robin schedule
        # (they hold the step after the prompt of every replica once warmup >= R), the timed steps follow them
        steps = min(steps, T * R)             # a trajectory has T steps; more would need more replicas
        start = max(0, min(warmup, T * R - steps))
        warmup = start
    stop = start + steps

    def fresh(n):
        reps = [Replica(B, W, wl, prompt, torch, len_bounds, fused, kv_int8, compact_every, split_rows) for _ in range(n)]
        for r in reps:
            r.finish_prompt(q_tail)
        return reps

    def run(reps, lo, hi):
        n = len(reps)
        for i in range(lo, hi):
            t, r = divmod(i, n)
            q, kn, vn = inputs[t]
            reps[r].step(B, t, q, kn, vn)

    if whole and warmup > 0:
        wreps = fresh(min(R, warmup))          # fewer steps than replicas: every one is a first step
        run(wreps, 0, warmup)
        torch.cuda.synchronize()
        del wreps

    # -------- prefill seed timing (separate from the decode metric)
    prefill_ms = None
    if q_tail is not None:
        tmp = Replica(B, W, wl, prompt, torch, len_bounds, fused, False)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        tmp.st.prefill_scores(q_tail)
        e1.record()
        torch.cuda.synchronize()
        prefill_ms = e0.elapsed_time(e1)
        del tmp
    quantize_ms = None
    if kv_int8:
        tmp = Replica(B, W, wl, prompt, torch, len_bounds, fused, False).st
        ck, cv = torch.zeros_like(tmp.K, dtype=torch.uint8), torch.zeros_like(tmp.V, dtype=torch.uint8)
        qp = torch.zeros((4, wl.b, wl.h, wl.d), dtype=torch.float32, device=dev)
        B.swa_quantize_kv(tmp.params, tmp.K, tmp.V, tmp.cache_len, ck, cv, qp)       # warm
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        B.swa_quantize_kv(tmp.params, tmp.K, tmp.V, tmp.cache_len, ck, cv, qp)
        e1.record()
        torch.cuda.synchronize()
        quantize_ms = e0.elapsed_time(e1)
        del tmp, ck, cv, qp

    # -------- timed region: exactly `steps` steps; an event between the steps right after a prompt (the first
    # R of the schedule) and the steady ones splits the time without bracketing single launches
    reps = fresh(R)
    run(reps, 0, start)                        # untimed: the schedule's first steps
    torch.cuda.synchronize()
    split = min(max(start, R), stop)
    e0, em, e1 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    if mode == "graph":
        graphs = []
        for lo, hi in ((start, split), (split, stop)):
            if hi > lo:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    run(reps, lo, hi)
                graphs.append((lo, g))
        torch.cuda.synchronize()
        t_wall0 = time.perf_counter()
        e0.record()
        for lo, g in graphs:
            if lo == split:
                em.record()
            g.replay()
        if split == stop:
            em.record()
        e1.record()
        torch.cuda.synchronize()
        t_wall1 = time.perf_counter()
        del graphs
    else:
        t_wall0 = time.perf_counter()
        e0.record()
        run(reps, start, split)
        em.record()
        run(reps, split, stop)
        e1.record()
        torch.cuda.synchronize()
        t_wall1 = time.perf_counter()
    total_ms = e0.elapsed_time(e1)
    first_ms = e0.elapsed_time(em) / (split - start) if split > start else None
    steady_ms = em.elapsed_time(e1) / (stop - split) if stop > split else None
    wall_ms = (t_wall1 - t_wall0) * 1e3
    for r in reps:
        assert r.st.check_status() == 0
    del reps

    # -------- accounting
    timed = range(start, stop)
    kv_tokens = sum(sum(ms[i // R]) for i in timed)
    alg_bytes = sum(step_bytes[i // R] for i in timed)
    sweep = [step_bytes[i // R] for i in timed]
    min_sweep = min(sum(sweep[j:j + R]) for j in range(0, max(1, steps - R + 1)))

    res = {
        "workload": wl.name, "steps": steps, "warmup": warmup, "replicas": R, "mode": mode, "fused": fused,
        "trajectory_steps": [start // R, (stop - 1) // R], "first_step_timed": start < R,
        "min_sweep_bytes": min_sweep,
        "cold": bool(min_sweep >= 2 * (256 << 20) or steps < R),
        "ms_per_step": total_ms / steps, "total_ms": total_ms, "host_wall_ms": wall_ms,
        "kv_tokens_per_s": kv_tokens / (total_ms * 1e-3),
        "generated_tokens_per_s": wl.b * steps / (total_ms * 1e-3),
        "alg_bytes_per_step": alg_bytes / steps,
        "alg_gbs_whole_step": alg_bytes / (total_ms * 1e-3) / 1e9,
        "prefill_seed_ms": prefill_ms, "quantize_kv_ms": quantize_ms,
        # whole steps (every launch of the step), from the event between the two stretches of the timed region
        "first_step_ms": first_ms, "steady_step_ms": steady_ms,
        "first_step_gbs": (step_bytes[0] / (first_ms * 1e-3) / 1e9) if first_ms else None,
        "steady_step_gbs": (sum(step_bytes[i // R] for i in range(split, stop)) / (stop - split) / (steady_ms * 1e-3) / 1e9)
                           if steady_ms else None,
    }

    # -------- per-kernel durations with HIP events on the launch stream (separate pass)
    if want_kernel_times:
        reps = fresh(R)
        torch.cuda.synchronize()
        # cost of an empty event pair, to be subtracted
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
        for a, b_ in pairs:
            a.record()
            b_.record()
        torch.cuda.synchronize()
        empty_ms = sorted(a.elapsed_time(b_) for a, b_ in pairs)[len(pairs) // 2]
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(stop)]
        n = len(reps)
        for i in range(stop):                  # the untimed first steps too: they hold the step after the prompt
            t, r = divmod(i, n)
            q, kn, vn = inputs[t]
            ev[i][0].record()
            reps[r].decode(B, t, q, kn, vn)
            ev[i][1].record()
            reps[r].compact(B, t)
            ev[i][2].record()
        torch.cuda.synchronize()
        dec = [max(0.0, e[0].elapsed_time(e[1]) - empty_ms) for e in ev]
        cmp_ = [max(0.0, e[1].elapsed_time(e[2]) - empty_ms) if not fused else 0.0 for e in ev]
        res["decode_kernel_ms_avg"] = sum(dec[start:stop]) / steps
        res["compact_kernel_ms_avg"] = sum(cmp_[start:stop]) / steps
        res["event_pair_overhead_ms"] = empty_ms
        first = [dec[i] for i in range(stop) if i // n == 0]
        steady = [dec[i] for i in timed if i // n > 0]
        res["decode_first_step_ms"] = sum(first) / max(1, len(first))
        res["decode_steady_ms"] = sum(steady) / max(1, len(steady)) if steady else None
        res["decode_first_step_gbs"] = step_bytes[0] / (res["decode_first_step_ms"] * 1e-3) / 1e9
        res["decode_steady_gbs"] = None
        if steady:
            sb = [step_bytes[i // n] for i in timed if i // n > 0]
            res["decode_steady_gbs"] = sum(sb) / (sum(steady) * 1e-3) / 1e9
        del reps
    return res


def bench_prefill_attention(wl, torch, B, W):
    """swa_prefill_attention over the workload's prompts: time and MFMA rate (dense causal attention,
    4 d flops per visible (query, key) pair) of the attention kernel, seed included in the time."""
    prompt = W.make_prompt(wl, "cuda")
    lens = prompt["lengths"]
    g = torch.Generator(device="cuda").manual_seed(wl.seed)
    Q = torch.randn((wl.b, wl.h, wl.cap, wl.d), generator=g, device="cuda", dtype=torch.float32).to(wl.torch_dtype)
    out = torch.zeros_like(Q)
    score = torch.zeros((wl.b, wl.h, wl.cap), dtype=torch.float32, device="cuda")
    R = wl.prefill_R if wl.prefill_R > 0 else min(max(wl.w, 1), B.SWA_MAX_PREFILL_ROWS)
    params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype, len_bound=max(lens))
    ws = torch.zeros((B.swa_workspace_bytes(params),), dtype=torch.uint8, device="cuda")
    times = []
    for it in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        B.swa_prefill_attention(params, Q, prompt["K"], prompt["V"], prompt["cache_len"], out, R, score, ws)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    ms = min(times[1:])
    flops = sum(4.0 * wl.d * L * (L + 1) / 2 for L in lens) * wl.h
    peak = 157.3 if wl.dtype == "f32" else 2500.0          # dense MFMA peak of the dtype, TFLOP/s
    return {"ms": ms, "tflops": flops / (ms * 1e-3) / 1e12, "mfma_peak_tflops": peak,
            "frac": flops / (ms * 1e-3) / 1e12 / peak, "seed_rows": R,
            "note": "dense causal attention over the prompts + importance seed, one call"}


def prewarm(torch, B, seconds):
    """Keeps the GPU streaming for `seconds` before anything is timed (clocks and power state settle over a
    much longer time than a few warm-up steps last).  Untimed, and nothing of the workload is touched."""
    if seconds <= 0:
        return 0
    x = torch.ones((1 << 28,), dtype=torch.float32, device="cuda")        # 1 GiB
    sink = torch.zeros((1,), dtype=torch.int32, device="cuda")
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(16):
            B.swa_probe_stream_read(x, x.numel() * 4, sink)
        torch.cuda.synchronize()
        n += 16
    del x
    return n


def bench_offload_tier(wl, torch, B, W, steps=4):
    """swa_offload_evicted between swa_decode_step and swa_compact_kv (Section V-A, Algorithm 2, the store half of
    the GPU-CPU caching phase): the step after the prompt evicts most of the prompt, the following ones one
    token per pair.  Rows cross the host link, so the bound is that link (PCIe 5.0 x16: 64 GB/s per direction),
    not HBM; this is the PCIe-inclusive leg and never part of `value`.  Then a reload of 64 tokens per pair."""
    prompt = prompt_of(wl, W)
    params = B.make_params(wl.b, wl.h, wl.d, wl.cap, wl.w, wl.sparsity_bp, wl.torch_dtype)
    st = B.DecodeState(params, device="cuda", debug_probs=False)
    st.K.copy_(prompt["K"]); st.V.copy_(prompt["V"]); st.pos.copy_(prompt["pos"])
    st.cache_len.copy_(prompt["cache_len"]); st.seq_len.copy_(prompt["cache_len"])
    store = B.HostStore(params, host_cap=wl.prompt_hi + steps)
    row_bytes = 2 * wl.d * wl.elem_bytes + 8                      # K row, V row, importance, position
    out = []
    for t in range(steps):
        q, kn, vn = W.make_step(wl, t, prompt["mu"])
        st.seq_len += 1
        st.decode_step(q, kn, vn)
        before = int(store.len.sum())
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.swa_offload_evicted(params, st.K, st.V, st.score, st.pos, st.kept_idx, st.kept_cnt, st.cache_len, store,
                              st.workspace)
        e1.record()
        torch.cuda.synchronize()
        rows = int(store.len.sum()) - before
        ms = e0.elapsed_time(e1)
        out.append({"step": t, "tokens": rows, "bytes": rows * row_bytes, "ms": ms, "gbs": rows * row_bytes / (ms * 1e-3) / 1e9})
        st.compact()
    # load the 64 oldest stored tokens of every pair back
    n_req = int(min(64, int(store.len.min())))
    req = torch.arange(n_req, dtype=torch.int32, device="cuda").expand(wl.b, wl.h, n_req).contiguous()
    cnt = torch.full((wl.b,), n_req, dtype=torch.int32, device="cuda")
    new_len = torch.zeros_like(st.cache_len)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    B.swa_reload_tokens(params, store, req, cnt, max(n_req, 1), st.K, st.V, st.score, st.pos, st.cache_len, new_len,
                        st.workspace)
    e1.record()
    torch.cuda.synchronize()
    assert st.check_status() == 0
    ms = e0.elapsed_time(e1)
    nbytes = n_req * wl.b * wl.h * row_bytes
    return {"bound": "host link", "peak_gbs": 64.0, "offload_steps": out,
            "frac_first_step": out[0]["gbs"] / 64.0,
            "reload": {"tokens": n_req * wl.b * wl.h, "bytes": nbytes, "ms": ms, "gbs": nbytes / (ms * 1e-3) / 1e9},
            "note": "device-initiated copies to and from pinned host memory; events on the launch stream"}


def stream_read_ceiling(torch, B):
    """Streaming-read rate of this GPU on a 4 GiB buffer (plain 128-bit loads, nothing else)."""
    x = torch.ones((1 << 30,), dtype=torch.float32, device="cuda")
    sink = torch.zeros((1,), dtype=torch.int32, device="cuda")
    best = None
    for _ in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.swa_probe_stream_read(x, x.numel() * 4, sink)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    del x
    return (1 << 32) / (best * 1e-3) / 1e9


def cpu_baseline(wl, W, torch, budget_s=10.0):
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample."""
    import numpy as np
    from oracle import swa_oracle as O
    O.build()
    sub_b = min(wl.b, 16)
    wls = wl.replace(b=sub_b)
    prompt = W.make_prompt(wls, "cpu")
    K = prompt["K"].double().numpy().copy()
    V = prompt["V"].double().numpy().copy()
    pos = prompt["pos"].numpy().copy()
    cache_len = prompt["cache_len"].numpy().copy()
    score = np.zeros(K.shape[:3])
    seq_len = cache_len.copy()
    max_steps = wl.steps
    inputs = [[x.double().numpy() for x in W.make_step(wls, t, prompt["mu"])] for t in range(max_steps)]
    state0 = (K.copy(), V.copy(), pos.copy(), cache_len.copy())
    kv_tokens, elapsed, done, passes = 0, 0.0, 0, 0
    # whole trajectories from the prompt on, repeated until about budget_s of oracle time is spent
    while elapsed < budget_s:
        K[...], V[...], pos[...], cache_len[...] = state0
        score[...] = 0.0
        seq_len = cache_len.copy()
        for t in range(max_steps):
            q, kn, vn = inputs[t]
            seq_len = seq_len + 1
            t0 = time.perf_counter()
            kept_idx, kept_cnt, out, _ = O.decode_step(q, kn, vn, K, V, score, pos, cache_len, seq_len,
                                                       wl.w, wl.sparsity_bp, wl.scale, want_probs=False)
            kv_tokens += int(cache_len.sum())
            O.compact(K, V, score, pos, kept_idx, kept_cnt, cache_len)
            elapsed += time.perf_counter() - t0
            done += 1
            if elapsed > 3 * budget_s:
                break
        passes += 1
        if elapsed > 3 * budget_s:
            break
    return {
        "value": kv_tokens / elapsed, "unit": "KV tokens/s", "cores": O.num_threads(), "kind": "oracle",
        "sample": f"{done} decode steps ({passes} passes over the {wl.steps}-step trajectory, from the "
                  f"prompt on) of {sub_b} of {wl.b} sequences x {wl.h} heads of {wl.name}, fp64, "
                  f"{elapsed:.1f} s of oracle time",
    }


def load_traffic(name, alg_bytes):
    """The counter record of this workload and step form whose timed launches are the ones timed here: the
    records are keyed by workload (whole trajectories) or workload + "_steps<K>" (a stretch of K steps), and the
    one whose algorithmic bytes per launch agree with this run's to 2 % is taken; none agreeing: no figure."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if not os.path.exists(path):
        return None
    try:
        records = json.load(open(path))
    except Exception:
        return None
    best = None
    for key, rec in records.items():
        if key != name and not key.startswith(name + "_steps"):
            continue
        err = abs(rec["algorithmic_bytes_per_launch"] - alg_bytes) / alg_bytes
        if err <= 0.02 and (best is None or err < best[0]):
            best = (err, dict(rec, record=key))
    return best[1] if best else None


STEP_TEXT = {
    "unordered": "swa_decode_step with SWA_FUSE_COMPACTION|SWA_UNORDERED (one kernel, hole-filling compaction, "
                 "kept_idx not requested)",
    "fused": "swa_decode_step with SWA_FUSE_COMPACTION (one kernel, token-ordered compaction, kept_idx not "
             "requested)",
    "shared": "swa_decode_step with SWA_HEAD_SHARED (three launches around the head-summed importance, "
              "hole-filling compaction)",
    "window": "swa_decode_step_window (strict local attention sum over min(w, 64) rows, hole-filling compaction)",
    "split": "swa_decode_step + swa_compact_kv",
}


def roofline_of(res, step_mode, kv_int8, wl_name):
    """Roofline object of the decode kernel for one timed run.  One-kernel forms: the step IS the
    kernel, so the HIP-event time of the timed region divided by the number of launches is its
    average launch duration (inter-kernel gaps included, hence an upper bound).  Two-call form:
    per-launch event brackets around swa_decode_step."""
    one_kernel = step_mode in ("unordered", "fused", "window")
    dec_ms = res["ms_per_step"] if one_kernel else res["decode_kernel_ms_avg"]
    achieved = res["alg_bytes_per_step"] / (dec_ms * 1e-3) / 1e9
    tag = ("" if step_mode == "unordered" else "_" + step_mode) + ("_q8" if kv_int8 else "")
    traffic = load_traffic(wl_name + tag, res["alg_bytes_per_step"]) if one_kernel else None
    # one-kernel forms: the step is the kernel, so the timed region's own split applies; two calls: the
    # per-launch event brackets (which read a few microseconds low: an empty bracket costs more than a full one)
    first_gbs = res.get("first_step_gbs") if one_kernel else res.get("decode_first_step_gbs")
    steady_gbs = res.get("steady_step_gbs") if one_kernel else res.get("decode_steady_gbs")
    first_frac = first_gbs / HBM_PEAK_GBS if first_gbs else None
    steady_frac = steady_gbs / HBM_PEAK_GBS if steady_gbs else None
    return {
        "bound": "hbm", "kernel": "swa_decode_kernel",
        "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
        "traffic": (traffic["fetch_bytes_per_launch"] + traffic["write_bytes_per_launch"]) if traffic else None,
        "traffic_source": ("profiles/pmc_traffic.json: rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE runs of this "
                           "workload, step form and timed steps (record `traffic_detail.record`), scaled by a "
                           "1 GiB copy (not measured in this run)") if traffic else None,
        "traffic_detail": traffic,
        "alg_bytes_per_launch": res["alg_bytes_per_step"], "avg_launch_ms": dec_ms,
        "timing": ("HIP events around the timed region on the launch stream / launches" if one_kernel
                   else "HIP events around every swa_decode_step launch"),
        "first_step_gbs": first_gbs, "steady_gbs": steady_gbs,
        "first_step_frac": first_frac, "steady_frac": steady_frac,
    }


def summary_of(res, step_mode, kv_int8, wl_name):
    r = roofline_of(res, step_mode, kv_int8, wl_name)
    return {"step_mode": step_mode, "steps": res["steps"], "replicas": res["replicas"], "cold": res["cold"],
            "kv_tokens_per_s": res["kv_tokens_per_s"], "ms_per_step": res["ms_per_step"],
            "decode_kernel_ms_avg": res.get("decode_kernel_ms_avg"),
            "compact_kernel_ms_avg": res.get("compact_kernel_ms_avg"),
            "whole_step_alg_gbs": res["alg_gbs_whole_step"], "prefill_seed_ms": res["prefill_seed_ms"],
            "roofline": {k: r[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic", "alg_bytes_per_launch",
                                           "avg_launch_ms", "first_step_frac", "steady_frac")}}


def other_workload_in_a_process_of_its_own(name, args):
    """Times one further workload by running this script on it in a child process (whole trajectories, the same
    step forms), before this process has touched the GPU.  Memory that a process acquires late, after
    gigabytes were allocated and released, measured 2-3 % slower on this GPU than the first allocations of a
    fresh process; one workload per process keeps every figure on the same footing as the headline's and as
    the rocprofv3 runs under profiles/, which are one workload per process too.  Returns the entry for
    other_workloads, or None (the caller then times the workload in-process)."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--gpus", "1", "--config", name, "--others", "none",
           "--no-cpu-baseline", "--ordered-forms", args.ordered_forms, "--step-mode", args.step_mode, "--mode", args.mode,
           "--prewarm-s", str(args.prewarm_s), "--compact-every", str(args.compact_every)]
    if args.kv_int8:
        cmd.append("--kv-int8")
    if args.split_rows:
        cmd.append("--split-rows")
    try:
        out = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
        c = json.loads(out.stdout.strip().splitlines()[-1])
    except Exception:
        return None
    entry = {"workload": name, "step_mode": args.step_mode, "steps": c["steps"], "replicas": c["config"]["replicas"],
             "cold": c["config"]["cold"], "kv_tokens_per_s": c["value"], "ms_per_step": c["ms_per_step"],
             "decode_kernel_ms_avg": c["detail"].get("decode_kernel_ms_avg"),
             "compact_kernel_ms_avg": c["detail"].get("compact_kernel_ms_avg"),
             "whole_step_alg_gbs": c["whole_step_alg_gbs"], "prefill_seed_ms": c["detail"].get("prefill_seed_ms"),
             "roofline": {k: c["roofline"].get(k) for k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                                            "alg_bytes_per_launch", "avg_launch_ms", "first_step_frac",
                                                            "steady_frac")},
             "measured_in": "a process of its own"}
    if c["detail"].get("prefill_seed"):
        entry["prefill_seed"] = c["detail"]["prefill_seed"]
    if c.get("other_step_forms"):
        entry["other_step_forms"] = c["other_step_forms"]
    return entry


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps of the headline workload; they follow the --warmup untimed steps of the same "
                         "round-robin schedule, which starts at the prompt (default: whole trajectories on every "
                         "replica, from the prompt on)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default=HEADLINE)
    ap.add_argument("--mode", choices=["graph", "stream"], default="graph")
    ap.add_argument("--step-mode", choices=["unordered", "fused", "split", "shared", "window"], default="unordered",
                    help="fused: one kernel per step, cache kept in token order; unordered: one kernel per "
                         "step, compaction fills holes (SWA_UNORDERED); shared: unordered with one token set per "
                         "sequence from the head-summed importance (SWA_HEAD_SHARED); window: unordered with "
                         "the strict local attention sum over a ring of w attention rows "
                         "(swa_decode_step_window); "
                         "split: swa_decode_step + swa_compact_kv")
    ap.add_argument("--kv-int8", action="store_true",
                    help="compress the cache to 8-bit channel-wise codes after the prompt (swa_quantize_kv) "
                         "and step with swa_decode_step_q8 (fp16 workloads)")
    ap.add_argument("--compact-every", type=int, default=1,
                    help="with --step-mode split: call swa_compact_kv only every C-th step (0 = never); between "
                         "compactions the cache keeps every token and the selection runs over all of them")
    ap.add_argument("--split-rows", action="store_true",
                    help="with --step-mode split: SWA_SPLIT_ROWS, the rows of a pair spread over several workgroups "
                         "(for few pairs with long caches, e.g. --compact-every 0)")
    ap.add_argument("--prefill-attention", action="store_true",
                    help="also time swa_prefill_attention over the workload's prompts")
    ap.add_argument("--prewarm-s", type=float, default=1.5,
                    help="seconds of plain streaming reads before anything is timed (0 = none)")
    ap.add_argument("--offload-tier", action="store_true",
                    help="also time swa_offload_evicted / swa_reload_tokens on the workload (host link, not HBM)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 1 GiB device copies (known traffic, for scaling rocprofv3 counters)")
    ap.add_argument("--others", default="c5_llama7b_sp50,c5_llama7b_sp90,c4_opt30b,c3_opt13b,c2_opt6p7b",
                    help="comma list of further workloads summarised in the same line ('none' = none)")
    ap.add_argument("--others-in-process", action="store_true",
                    help="time the further workloads in this process instead of one child process each")
    ap.add_argument("--no-whole-trajectory", action="store_true",
                    help="with --steps: do not also time whole trajectories of the headline workload")
    ap.add_argument("--ordered-forms", default="fused,split",
                    help="further step forms timed beside --step-mode for every workload ('none' = none)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 "
              "(the path shards over (sequence, head) pairs with no exchange between GPUs)",
              file=sys.stderr)
        sys.exit(2)

    # the other workloads first, each in a process of its own, while this process has not touched the GPU
    none = ("", "none")
    other_names = [x for x in args.others.split(",") if x not in none and x != args.config]
    child_entries = {}
    whole_child = None
    if not args.others_in_process:
        for name in other_names:
            child_entries[name] = other_workload_in_a_process_of_its_own(name, args)
        if args.steps is not None and not args.no_whole_trajectory:
            # the headline workload over whole trajectories, on the same footing
            saved = args.ordered_forms
            args.ordered_forms = "none"
            whole_child = other_workload_in_a_process_of_its_own(args.config, args)
            args.ordered_forms = saved

    import torch
    from paper_2403_17312_amd import binding as B
    from paper_2403_17312_amd import workload as W
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()
    torch.cuda.set_device(0)
    B.swa_prepare()                      # LDS limits raised before anything is captured
    prewarm(torch, B, args.prewarm_s)

    wl = W.CONFIGS.get(args.config) or W.EXTRA[args.config]
    warmup = args.warmup if args.warmup is not None else 8
    fused_of = lambda sm: sm if sm != "split" else False
    if args.compact_every != 1 and args.step_mode != "split":
        print("bench.py: --compact-every needs --step-mode split (the fused forms compact every step)", file=sys.stderr)
        sys.exit(2)
    if args.split_rows and (args.step_mode != "split" or args.kv_int8):
        print("bench.py: --split-rows needs --step-mode split and the uncompressed cache", file=sys.stderr)
        sys.exit(2)
    none = ("", "none")
    extra_forms = [x for x in args.ordered_forms.split(",") if x not in none and x != args.step_mode]
    if args.compact_every != 1 or args.split_rows or args.step_mode in ("shared", "window"):
        extra_forms = []
    res = bench_workload(wl, args.steps, warmup, args.mode, torch, B, W, fused=fused_of(args.step_mode),
                         kv_int8=args.kv_int8, compact_every=args.compact_every, split_rows=args.split_rows)
    steps = res["steps"]
    roof = roofline_of(res, args.step_mode, args.kv_int8, wl.name)
    line = {
        "metric": "SWA decode-step KV tokens/s",
        "value": res["kv_tokens_per_s"],
        "unit": "KV tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": res["warmup"],
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype + ("+u8kv" if args.kv_int8 else ""), "data": "synthetic",
        "config": {"workload": wl.name, "b": wl.b, "h": wl.h, "d": wl.d, "prompt": [wl.prompt_lo, wl.prompt_hi],
                   "decode_steps_per_trajectory": wl.steps, "w": wl.w, "sparsity_bp": wl.sparsity_bp,
                   "replicas": res["replicas"], "cold": res["cold"], "min_sweep_bytes": res["min_sweep_bytes"],
                   "timed": f"steps {res['trajectory_steps'][0]}..{res['trajectory_steps'][1]} of the decode trajectories of "
                            f"{res['replicas']} replicas stepped round-robin"
                            + ("; from the prompt on" if res["first_step_timed"] else
                               f"; the {res['warmup']} untimed warm-up steps are the first steps of the same schedule and "
                               "hold every replica's step after the prompt, which whole_trajectory and "
                               "roofline.first_step_frac report"),
                   "launch": args.mode, "compact_every": args.compact_every,
                   "step": STEP_TEXT[args.step_mode]
                           + ("; 8-bit compressed cache (swa_quantize_kv once, then swa_decode_step_q8)"
                              if args.kv_int8 else "")
                           + ("; SWA_SPLIT_ROWS (a pair's rows over several workgroups, four launches)"
                              if args.split_rows else "")},
        "roofline": roof,
        "whole_step_alg_gbs": res["alg_gbs_whole_step"],
        "generated_tokens_per_s": res["generated_tokens_per_s"],
        "detail": {k: res.get(k) for k in ("decode_kernel_ms_avg", "compact_kernel_ms_avg", "decode_first_step_ms",
                                           "decode_steady_ms", "event_pair_overhead_ms", "host_wall_ms",
                                           "prefill_seed_ms", "quantize_kv_ms", "first_step_ms", "steady_step_ms")},
    }
    ceil_gbs = stream_read_ceiling(torch, B)
    line["roofline"]["measured_stream_read_gbs"] = ceil_gbs
    line["roofline"]["frac_of_measured_stream_read"] = roof["achieved"] / ceil_gbs
    line["pair_rows_per_s"] = res["kv_tokens_per_s"] * wl.h

    def seed_detail(o, r):
        # one read of the prompt's keys and 2 R s d flops per pair
        lens = W.prompt_lengths(o).tolist()
        kb = sum(lens) * o.h * o.d * o.elem_bytes
        fl = 2.0 * o.prefill_R * sum(lens) * o.h * o.d
        sec = r["prefill_seed_ms"] * 1e-3
        return {"ms": r["prefill_seed_ms"], "gbs_one_read_of_K": kb / sec / 1e9, "frac_of_hbm_peak": kb / sec / 1e9 / HBM_PEAK_GBS,
                "tflops_one_pass": fl / sec / 1e12}

    if res["prefill_seed_ms"]:
        line["detail"]["prefill_seed"] = seed_detail(wl, res)
    if args.prefill_attention:
        line["detail"]["prefill_attention"] = bench_prefill_attention(wl, torch, B, W)
    if args.offload_tier:
        line["detail"]["offload_tier"] = bench_offload_tier(wl, torch, B, W)

    # --steps covers a short stretch of the trajectory: the same workload over whole trajectories (the step
    # after the prompt included, at its true weight), for reference
    if args.steps is not None and not args.no_whole_trajectory and res["steps"] < wl.steps * res["replicas"]:
        if whole_child is not None:
            line["whole_trajectory"] = {k: v for k, v in whole_child.items() if k != "workload"}
        else:
            r = bench_workload(wl, None, warmup, args.mode, torch, B, W, fused=fused_of(args.step_mode),
                               kv_int8=args.kv_int8, compact_every=args.compact_every, split_rows=args.split_rows)
            line["whole_trajectory"] = summary_of(r, args.step_mode, args.kv_int8, wl.name)
        if line["roofline"]["first_step_frac"] is None:      # the timed stretch held no step after a prompt
            line["roofline"]["first_step_frac"] = line["whole_trajectory"]["roofline"]["first_step_frac"]
            line["roofline"]["first_step_gbs"] = line["whole_trajectory"]["roofline"]["first_step_frac"] * HBM_PEAK_GBS
            line["roofline"]["first_step_from"] = "whole_trajectory"

    # the same workload in the forms that keep the cache in token order
    forms = []
    for sm in extra_forms:
        r = bench_workload(wl, args.steps, warmup, args.mode, torch, B, W, fused=fused_of(sm), kv_int8=args.kv_int8)
        forms.append(summary_of(r, sm, args.kv_int8, wl.name))
    if forms:
        line["other_step_forms"] = forms

    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl, W, torch)

    others = []
    for name in other_names:
        o = W.CONFIGS[name]
        if args.kv_int8 and o.dtype != "f16":
            continue
        if child_entries.get(name) is not None:
            others.append(child_entries[name])
            continue
        entry = {"workload": name, "measured_in": "this process, after the headline workload"}
        for sm in [args.step_mode] + extra_forms:
            r = bench_workload(o, None, min(o.steps, 8), args.mode, torch, B, W, fused=fused_of(sm),
                               kv_int8=args.kv_int8, compact_every=args.compact_every, split_rows=args.split_rows)
            sm_sum = summary_of(r, sm, args.kv_int8, name)
            if sm == args.step_mode:
                entry.update(sm_sum)
                if r["prefill_seed_ms"]:
                    entry["prefill_seed"] = seed_detail(o, r)
            else:
                entry.setdefault("other_step_forms", []).append(sm_sum)
        others.append(entry)
    if others:
        line["other_workloads"] = others
    if args.copy_calibration:
        x = torch.zeros((1 << 29,), dtype=torch.float16, device="cuda")      # 1 GiB
        y = torch.empty_like(x)
        for _ in range(4):
            torch.add(x, 1.0, out=y)          # reads 1 GiB, writes 1 GiB, one elementwise kernel
        torch.cuda.synchronize()
        line["copy_calibration"] = "4 x torch.add(x, 1, out=y) on 1 GiB fp16 tensors"
    print(json.dumps(line))


if __name__ == "__main__":
    main()
