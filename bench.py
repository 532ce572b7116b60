#!/usr/bin/env python3
"""Benchmark of the bounded-cache rollout decode path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen7b]

A step is one pass of the whole hot path (evict-and-encode where a window is full, ring append,
windowed GQA decode attention) over one batch of B rollouts.  The headline workload is the
Qwen2.5-7B-shaped layer (bf16, 28 query / 4 KV heads, head_dim 128, window 4096, chunk 128,
128 rollouts, 8192 decode steps); inputs are synthetic, seeded, and resident in HBM before any
timed region starts.

What is timed.  The metric is quoted on the whole T-step run of the workload, most of which runs
with full rings.  With --steps K < T the timed region is the LAST K steps of that run: steps
1 .. T-K are decoded first, untimed, through the same entry point (the last W of them are the
warm-up), so the K timed steps find the rings as the real run leaves them.  --steps 0 (or K >= T)
times the whole run from an empty cache.  Beside it the same JSON line carries

  full_run             the whole T-step run from an empty cache, timed in the same process
  staggered_evictions  full-ring steps with the rollouts' evictions in the same step / spread over the steps
  workloads            the other configurations (3B-, 8B-shaped, ragged, tiny fp32): last-K-step and whole-run figures
  roofline             algorithmic bytes of the timed launches / their HIP-event time, against the HBM peak
  cpu_baseline         the CPU oracle on the host cores, on a bounded sample of the same workload

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

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth


def n_live_at(t: int, W: int, C: int) -> int:
    """Live thinking tokens the attention of decode step t (1-based) reads, lazy chunk eviction."""
    return t if t <= W else W - C + ((t - W - 1) % C) + 1


def path_bytes(wl, lengths, t0: int, t1: int, prompt_len=None):
    """Algorithmic bytes and decoded tokens of decode steps t0+1 .. t1 (1-based) of the workload: per active
    rollout and step the K and V stream over question tokens and live window, q in and out out, the
    append; per eviction the chunk re-read and the read-modify-write of S."""
    import numpy as np
    s = wl.elem_bytes
    Wr, C = wl.window - wl.n_sink, wl.chunk
    per_tok, qo, app = 2 * wl.d_kv * s, 2 * wl.d_q * s, 2 * wl.d_kv * s
    per_evict = 2 * C * wl.d_kv * s + 2 * wl.n_global * wl.rank * 4
    steps = np.arange(t0 + 1, t1 + 1, dtype=np.int64)
    nl = np.array([n_live_at(int(t), Wr, C) for t in steps], dtype=np.float64)
    evicts = ((steps > Wr) & ((steps - Wr - 1) % C == 0)).astype(np.float64)
    uniq = {}
    pls = [0] * len(lengths) if prompt_len is None else list(np.asarray(prompt_len).tolist())
    for L, P in zip(np.asarray(lengths).tolist(), pls):
        uniq[(L, P)] = uniq.get((L, P), 0) + 1
    total, tokens = 0.0, 0
    for (L, P), cnt in uniq.items():
        alive = steps <= L
        total += cnt * float(((per_tok * (nl + P) + qo + app + per_evict * evicts) * alive).sum())
        tokens += cnt * int(alive.sum())
    return total, tokens


def cpu_baseline(wl, budget_s: float = 15.0):
    """The fp64 oracle, as it stands, on the host: one rollout of the workload's true per-token shape
    with the window pre-filled to capacity, so the first timed step evicts and encodes a chunk."""
    import numpy as np
    import psutil
    import torch

    from oracle import pte_oracle as po
    from paper_2602_16839_amd import inputs as I

    one = wl.replace(batch=1)
    enc = {k: v.to(torch.float64).numpy() for k, v in I.encoder_params(one).items()}
    orc = po.OracleLayer(1, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                         enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    W = wl.window
    _, k, v = I.qkv_steps(one, 0, W)
    k, v = k.to(torch.float64).numpy(), v.to(torch.float64).numpy()
    for t in range(W):
        orc.append(0, k[t, 0], v[t, 0])
    max_steps = 16 * wl.chunk
    q, k, v = (x.to(torch.float64).numpy() for x in I.qkv_steps(one, W, W + max_steps))
    proc = psutil.Process()
    c0 = proc.cpu_times()
    t0 = time.perf_counter()
    n = 0
    while n < max_steps:
        orc.step(q[n], k[n], v[n])
        n += 1
        if time.perf_counter() - t0 > budget_s:
            break
    wall = time.perf_counter() - t0
    c1 = proc.cpu_times()
    cpu = (c1.user - c0.user) + (c1.system - c0.system)
    return {
        "value": n / wall, "unit": "tokens/s", "cores": max(1, int(round(cpu / wall))), "kind": "oracle",
        "sample": "1 rollout x %d decode steps of the %s shape (H_q %d, H_kv %d, d %d), window pre-filled to "
                  "W=%d so that step 1 evicts and encodes a %d-token chunk; numpy fp64, %.1f s wall, "
                  "%d host cores visible" % (n, wl.name, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, W, wl.chunk,
                                             wall, len(os.sched_getaffinity(0))),
    }


class Timer:
    """HIP events on torch's current stream (the stream every library call is issued to) plus the host clock."""

    def __init__(self, torch):
        self.torch = torch

    def __call__(self, fn):
        t = self.torch
        t.cuda.synchronize()
        e0, e1 = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        w0 = time.perf_counter()
        e0.record()
        fn()
        e1.record()
        t.cuda.synchronize()
        return e0.elapsed_time(e1), (time.perf_counter() - w0) * 1e3


class Bench:
    """One workload on one context: inputs by segments of the step axis, the run in pieces."""

    def __init__(self, wl, args, torch, np, I, ptenc, resident: bool):
        self.wl, self.args, self.torch, self.np, self.I, self.ptenc = wl, args, torch, np, I, ptenc
        self.dev = torch.device("cuda:0")
        self.lengths = I.rollout_lengths(wl)
        self.T = int(self.lengths.max()) if wl.ragged else wl.steps
        self.compact = wl.ragged and args.ragged_mode == "compact"
        self.resident = resident or wl.ragged     # the whole run's inputs in HBM at once (else per segment)
        self.timer = Timer(torch)
        self.layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                                 dtype=wl.torch_dtype, n_global=wl.n_global, rank=wl.rank, n_sink=wl.n_sink)
        self.prompt_len = I.prompt_lengths(wl) if wl.n_sink else None
        if wl.n_sink:
            self.pk, self.pv = I.prompt_kv(wl, device=self.dev)
        layer = self.layer
        if args.splits:
            layer.set_option(ptenc.OPT_SPLITS, args.splits)
        if args.encode_parts:
            layer.set_option(ptenc.OPT_ENCODE_PARTS, args.encode_parts)
        if args.encode_inline >= 0:
            layer.set_option(ptenc.OPT_ENCODE_INLINE, args.encode_inline)
        if args.policy == "scored":
            layer.set_option(ptenc.OPT_RECENT, args.recent)
            layer.set_option(ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED)
        self.enc = I.encoder_params(wl, device=self.dev)
        e = self.enc
        layer.set_encoder(e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"])
        self.attn_kernel, self.n_splits, _ = layer.plan()
        self.seg = None          # (t0, t1, q, k, v, out, active, ids, row_offsets)
        if self.resident:
            self.seg = self._make_segment(0, self.T)

    # ---- inputs ----
    def _make_segment(self, t0, t1):
        torch, np, I, wl, dev = self.torch, self.np, self.I, self.wl, self.dev
        n = t1 - t0
        active = ids = row_offsets = None
        blk = max(1, (1 << 26) // (wl.batch * wl.d_q))
        if self.compact:
            # what a rollout engine feeds: only the rollouts still running, with their ids (rows of step t, then
            # of step t + 1, ...); built block by block so that no full [steps, B] tensor ever exists
            counts = np.array([(self.lengths > t).sum() for t in range(t0, t1)], dtype=np.int64)
            row_offsets = np.concatenate([[0], np.cumsum(counts)])
            rows = int(row_offsets[-1])
            q = torch.empty((rows, wl.n_q_heads, wl.head_dim), dtype=wl.torch_dtype, device=dev)
            k = torch.empty((rows, wl.n_kv_heads, wl.head_dim), dtype=wl.torch_dtype, device=dev)
            v = torch.empty_like(k)
            ids = torch.empty(rows, dtype=torch.int32, device=dev)
            len_dev = torch.from_numpy(self.lengths).to(dev).view(1, -1)
            for a in range(0, n, blk):
                b = min(n, a + blk)
                r0, r1 = int(row_offsets[a]), int(row_offsets[b])
                if r1 == r0:
                    continue
                alive = torch.arange(t0 + a, t0 + b, device=dev).view(-1, 1) < len_dev          # [b - a, B]
                qb, kb, vb = I.qkv_steps(wl, t0 + a, t0 + b, device=dev)
                q[r0:r1], k[r0:r1], v[r0:r1] = qb[alive], kb[alive], vb[alive]
                ids[r0:r1] = torch.nonzero(alive)[:, 1].to(torch.int32)
        else:
            q = torch.empty((n, wl.batch, wl.n_q_heads, wl.head_dim), dtype=wl.torch_dtype, device=dev)
            k = torch.empty((n, wl.batch, wl.n_kv_heads, wl.head_dim), dtype=wl.torch_dtype, device=dev)
            v = torch.empty_like(k)
            for a in range(0, n, blk):
                b = min(n, a + blk)
                q[a:b], k[a:b], v[a:b] = I.qkv_steps(wl, t0 + a, t0 + b, device=dev)
            if wl.ragged:
                tt = torch.arange(t0, t1, device=dev).view(-1, 1)
                active = (tt < torch.from_numpy(self.lengths).to(dev).view(1, -1)).to(torch.uint8).contiguous()
        out = torch.empty_like(q)
        torch.cuda.synchronize()
        return (t0, t1, q, k, v, out, active, ids, row_offsets)

    def _segment_for(self, t0, t1):
        if self.seg is not None and self.seg[0] <= t0 and t1 <= self.seg[1]:
            return self.seg
        self.seg = None                       # free the old one first
        self.seg = self._make_segment(t0, t1)
        return self.seg

    # ---- the run ----
    def start(self):
        """An empty cache; question tokens (if the workload has any) prefilled: not part of the timed steps."""
        self.layer.reset()
        if self.wl.n_sink:
            self.layer.prefill(self.pk, self.pv, self.prompt_len)

    def prepared(self, t0, t1):
        """Decode steps t0+1 .. t1 as a function that only makes the library call (no synchronisation; the
        arguments are marshalled here, outside any timed region); the inputs must be in the current segment."""
        s0, _, q, k, v, out, active, ids, ro = self.seg
        a, b = t0 - s0, t1 - s0
        if self.compact:
            r0, r1 = int(ro[a]), int(ro[b])
            return self.layer.prepared_run_ids(q[r0:r1], k[r0:r1], v[r0:r1], ids[r0:r1], ro[a:b + 1] - r0, out[r0:r1])
        return self.layer.prepared_run(q[a:b], k[a:b], v[a:b], out[a:b], None if active is None else active[a:b])

    def launch(self, t0, t1):
        self.prepared(t0, t1)()

    def run_timed(self, t0, t1, seg_steps=0):
        """Steps t0+1 .. t1; returns (GPU ms by HIP events, host ms), summed over the segments the inputs come in."""
        gpu = wall = 0.0
        step = seg_steps if (seg_steps and not self.resident) else (t1 - t0)
        a = t0
        while a < t1:
            b = min(t1, a + step)
            self._segment_for(a, b)
            g, w = self.timer(self.prepared(a, b))
            gpu, wall = gpu + g, wall + w
            a = b
        return gpu, wall

    def check_counters(self, t):
        ln, _ = self.layer.counters()
        assert self.np.array_equal(ln, self.np.minimum(self.lengths, t)), "counters after the run are not the step count"
        assert self.layer.poll_error() == 0

    def figures(self, t0, t1, gpu_ms, wall_ms):
        nbytes, tokens = path_bytes(self.wl, self.lengths, t0, t1, self.prompt_len)
        ms = max(gpu_ms, wall_ms)
        return {
            "steps": t1 - t0, "first_step": t0 + 1, "last_step": t1, "tokens": tokens,
            "ms": ms, "gpu_ms": gpu_ms, "us_per_step": ms * 1e3 / max(1, t1 - t0),
            "tokens_per_s": tokens / (ms * 1e-3),
            "algorithmic_gbytes": nbytes / 1e9,
            "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "hbm_frac_by_gpu_events": nbytes / (gpu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }

    def window_words(self, t0, t1):
        wl = self.wl
        Wr, C = wl.window - wl.n_sink, wl.chunk
        nl = [n_live_at(t, Wr, C) for t in range(t0 + 1, t1 + 1)]
        return "steps %d..%d of the %d-step run, %d..%d thinking tokens live per rollout" % (
            t0 + 1, t1, self.T, min(nl), max(nl))

    def describe(self):
        wl = self.wl
        return "%s-shaped layer: B %d rollouts, %d Q / %d KV heads, head_dim %d, window %d, chunk %d%s%s" % (
            wl.name, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
            (", ragged lengths (lognormal, median 3000, capped at %d), finished rollouts %s" % (
                wl.steps, "dropped from the batch (rollout-id lists)" if self.compact else "masked")) if wl.ragged else "",
            ", %d slots reserved for question tokens (128..%d per rollout, prefilled)" % (wl.n_sink, wl.n_sink)
            if wl.n_sink else "")

    def staggered(self, n_steps):
        """Full-ring steps with every rollout evicting in the same step, and with the rollouts' rings filled at
        different steps so that every step has its share of evictions.  The cache keeps what the last run
        left and the counters are re-based, so positions and contents no longer correspond: timing only."""
        np, wl, layer = self.np, self.wl, self.layer
        Wr, C, B = wl.window, wl.chunk, wl.batch
        ns = min(n_steps, self.T)
        self._segment_for(0, ns)
        zeros = np.zeros(B, dtype=np.int64)

        def timed_from(ln):
            best = None
            for _ in range(3):
                layer.set_counters(ln, zeros)
                g, _ = self.timer(self.prepared(0, ns))
                us = g * 1e3 / ns
                best = us if best is None else min(best, us)
            return best

        together = timed_from(np.full(B, Wr - C // 2, dtype=np.int64))
        spread = timed_from((Wr - (np.arange(B) * C // B) % C).astype(np.int64))
        return {"steps": ns, "us_per_step_all_evicting_together": together,
                "us_per_step_evictions_spread_over_steps": spread,
                "spread_over_together": spread / together}


def steady_and_full(b: Bench, K: int, W: int, seg_steps: int):
    """The whole run from an empty cache, timed in pieces: steps 1..T-K (the last W of them are the warm-up of the
    K-step region), then the last K steps as a timed region of their own.  Returns (steady, full) figures."""
    T = b.T
    K = min(K, T)
    b.start()
    g0 = w0 = 0.0
    if T - K > 0:
        g0, w0 = b.run_timed(0, T - K, seg_steps)
    b._segment_for(T - K, T)
    g1, w1 = b.run_timed(T - K, T)
    b.check_counters(T)
    steady = b.figures(T - K, T, g1, w1)
    steady["window"] = b.window_words(T - K, T)
    full = b.figures(0, T, g0 + g1, w0 + w1)
    full["timed_as"] = "steps 1..%d%s, then the last %d" % (
        T - K, "" if b.resident else " in segments of %d (inputs generated per segment, outside the timing)" % seg_steps, K)
    return steady, full


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20,
                    help="decode steps in the timed region: the last K steps of the workload's run (0 = the whole run)")
    ap.add_argument("--warmup", type=int, default=5,
                    help="warm-up steps: the last W of the untimed steps 1..T-K that precede the timed region")
    ap.add_argument("--workload", default="qwen7b")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--encode-parts", type=int, default=0,
                    help="workgroups that share one evicted chunk's encoding (0 = the library's heuristic)")
    ap.add_argument("--encode-inline", type=int, default=-1, choices=[-1, 0, 1],
                    help="who folds evicted chunks into the state: 0 encoding workgroups of their own, 1 the rollouts' own "
                         "workgroups ahead of time, -1 the library's choice by launch size")
    ap.add_argument("--chunk", type=int, default=0,
                    help="override the workload's eviction chunk C (eviction-ratio sweeps; 0 = the workload's own)")
    ap.add_argument("--ragged-mode", choices=["compact", "masked"], default="compact",
                    help="ragged workloads: drop finished rollouts from the batch (rollout-id lists) or mask them")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the untimed steps 1..T-K and the K timed steps (profiler runs): no full run, no "
                         "staggered evictions, no other workloads, no CPU baseline")
    ap.add_argument("--no-workloads", action="store_true", help="skip the other configurations")
    ap.add_argument("--progress", action="store_true",
                    help="decode the untimed steps in pieces of 1024 and report each on stderr (runs under a profiler's "
                         "counters take minutes)")
    ap.add_argument("--no-stagger", action="store_true", help="skip the staggered-evictions figures")
    ap.add_argument("--extras", action="store_true",
                    help="also time the state-as-weight-delta application (and the question-token prefill)")
    ap.add_argument("--policy", choices=["sliding", "scored"], default="sliding",
                    help="which tokens an eviction takes: the oldest chunk, or the lowest accumulated attention probability")
    ap.add_argument("--recent", type=int, default=-1, help="scored policy: most recent ring entries never taken (-1 = half the ring)")
    ap.add_argument("--layers", type=int, default=0,
                    help="also time a stack of this many layers (each with its own cache) over the run's first steps: "
                         "eager launches, then replays of the recorded one-step HIP graph")
    ap.add_argument("--layer-steps", type=int, default=512, help="steps of the stack timing")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the plain copy / read kernels on 1 GiB (scale for the profiler's byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on ONE GPU (rollouts are independent; several GPUs would each take a "
              "slice of the batch with no exchange). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2602_16839_amd import inputs as I
    from paper_2602_16839_amd import ptenc

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    wl = I.WORKLOADS[args.workload]
    if args.chunk:
        wl = wl.replace(chunk=args.chunk)
    Wu = max(0, args.warmup)

    # ---- the headline workload: inputs of the whole run resident in HBM where they fit comfortably ----
    in_bytes = wl.steps * wl.batch * (2 * wl.d_q + 2 * wl.d_kv) * wl.elem_bytes
    hb = Bench(wl, args, torch, np, I, ptenc, resident=in_bytes <= (40 << 30))
    T = hb.T
    K = T if (args.steps <= 0 or args.steps >= T) else args.steps
    seg_steps = 512

    # untimed: steps 1 .. T-K through the same entry point (the last Wu of them are the warm-up)
    hb.start()
    if T - K > 0:
        a = 0
        while a < T - K:
            b_ = (T - K) if (hb.resident and not args.progress) else min(T - K, a + (1024 if hb.resident else seg_steps))
            hb._segment_for(a, b_)
            hb.launch(a, b_)
            if args.progress:
                torch.cuda.synchronize()
                print("bench.py: steps 1..%d of %d decoded (untimed)" % (b_, T), file=sys.stderr, flush=True)
            a = b_
    else:
        hb._segment_for(0, min(T, max(Wu, 1)))
        hb.launch(0, min(T, Wu))          # whole-run timing: a few steps to warm up, then from an empty cache again
        hb.start()
    hb._segment_for(T - K, T)
    # the timed region: exactly K steps, synchronised on both sides, HIP events on the launch stream
    gpu_ms, wall_ms = hb.timer(hb.prepared(T - K, T))
    hb.check_counters(T)
    total_ms = max(gpu_ms, wall_ms)
    head = hb.figures(T - K, T, gpu_ms, wall_ms)
    fused = hb.attn_kernel == 1

    # ---- roofline of the dominant kernel over the same K launches.  On the MFMA path one launch of the step
    #      kernel is one whole decode step and nothing else runs between the launches, so the HIP events
    #      around the timed region bracket exactly K back-to-back launches of it. ----
    launch_bytes = head["algorithmic_gbytes"] * 1e9 / K
    mean_s = gpu_ms * 1e-3 / K
    traffic, traffic_note = None, "no HBM byte counters were collected for this window"
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % wl.name)
    if os.path.exists(tpath):
        with open(tpath) as fh:
            tj = json.load(fh)
        if tj.get("first_step") == T - K + 1 and tj.get("last_step") == T and not args.chunk and args.policy == "sliding":
            traffic, traffic_note = tj.get("traffic_bytes_per_launch"), tj.get("source")
        else:
            traffic_note = "profiles/hbm_traffic_%s.txt covers steps %s..%s, not this window" % (
                wl.name, tj.get("first_step"), tj.get("last_step"))
    roofline = {
        "bound": "hbm", "achieved": launch_bytes / mean_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": launch_bytes / mean_s / 1e9 / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_note,
        "kernel": "decode_mfma_kernel (evict-encode + append + attention in one launch)" if fused
                  else "attn_generic / step kernels of the plain path (all launches of the step)",
        "launches": K, "mean_launch_us": mean_s * 1e6, "algorithmic_bytes_per_launch": launch_bytes,
        "timed_with": "HIP events on the launch stream around the K back-to-back launches of the timed region",
    }

    res = {
        "metric": "rollout decode tokens/s per layer (bounded window)",
        "value": head["tokens"] / (total_ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wu,
        "ms_per_step": total_ms / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {
            "workload": "%s; timed: %s%s" % (
                hb.describe(), hb.window_words(T - K, T),
                (" (steps 1..%d decoded first, untimed, through the same entry point; the last %d of them are the "
                 "warm-up)" % (T - K, min(Wu, T - K))) if K < T else " from an empty cache"),
            "name": wl.name, "batch": wl.batch, "window": wl.window, "chunk": wl.chunk, "tokens": head["tokens"],
            "run_steps": T, "first_timed_step": T - K + 1, "last_timed_step": T,
            "attn_kernel": "mfma" if fused else "generic", "window_splits": hb.n_splits,
            "evict_policy": args.policy, "parallelism": "single GPU",
        },
        "gpu_ms": gpu_ms, "wall_ms": wall_ms,
        "hbm_frac_whole_path": head["hbm_frac"],
        "algorithmic_gbytes": head["algorithmic_gbytes"],
        "roofline": roofline,
    }

    if not args.headline_only:
        # ---- the whole run from an empty cache, in the same process ----
        if K < T:
            hb.start()
            g, w = hb.run_timed(0, T, seg_steps)
            hb.check_counters(T)
            res["full_run"] = hb.figures(0, T, g, w)
            res["full_run"]["what"] = "all %d steps from an empty cache%s" % (
                T, "" if hb.resident else ", in segments of %d steps (inputs generated per segment, untimed)" % seg_steps)
        if not args.no_stagger and not wl.ragged and not wl.n_sink and args.policy == "sliding":
            res["staggered_evictions"] = hb.staggered(2 * wl.chunk)

    if args.extras:
        layer = hb.layer
        # y += ((x A) S) B at the model's hidden size (the query projection width stands in for it)
        ex = {}
        d_h = wl.d_q
        ad = I.adapter_inputs(wl, d_h, d_h, device=dev)
        yb = ad["y"].clone()
        for _ in range(10):
            layer.apply_delta(ad["x"], ad["At"], ad["Bt"], yb)
        g, _ = hb.timer(lambda: [layer.apply_delta(ad["x"], ad["At"], ad["Bt"], yb) for _ in range(200)])
        us = g * 1e3 / 200
        s_ = wl.elem_bytes
        nbytes_ad = wl.batch * (d_h * s_ + 2 * d_h * s_ + wl.n_global * wl.rank * 4) + (wl.n_global + wl.rank) * d_h * s_
        ex["apply_delta"] = {"d_in": d_h, "d_out": d_h, "us_per_call": us, "algorithmic_bytes": nbytes_ad,
                             "GB_per_s": nbytes_ad / us / 1e3, "hbm_frac": nbytes_ad / us / 1e3 / HBM_PEAK_GBS}
        if wl.n_sink:
            g, _ = hb.timer(lambda: [layer.prefill(hb.pk, hb.pv, hb.prompt_len) for _ in range(20)])
            us = g * 1e3 / 20
            nb = float(hb.prompt_len.sum()) * 2 * wl.d_kv * s_ * 2          # read once, written once
            ex["prefill"] = {"us_per_call": us, "algorithmic_bytes": nb, "GB_per_s": nb / us / 1e3}
        res["extras"] = ex

    if args.layers > 0 and not wl.ragged:
        # L layers, each with its own cache, counters and state; layer l reads the inputs of step t + 7 l
        L, KL = args.layers, min(args.layer_steps, T)
        hb._segment_for(0, KL)
        _, _, q, k, v, out, _, _, _ = hb.seg
        enc = hb.enc
        st = ptenc.Stack(L, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                         dtype=wl.torch_dtype, n_global=wl.n_global, rank=wl.rank, n_sink=wl.n_sink)
        for lay in st.layers:
            lay.set_encoder(enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
            if args.splits:
                lay.set_option(ptenc.OPT_SPLITS, args.splits)

        def stack_start():
            st.reset()
            if wl.n_sink:
                for lay in st.layers:
                    lay.prefill(hb.pk, hb.pv, hb.prompt_len)

        outs = [out[l % KL] for l in range(L)]

        def eager(t):
            idx = [(t + 7 * l) % KL for l in range(L)]
            st.step([q[i] for i in idx], [k[i] for i in idx], [v[i] for i in idx], outs)

        def timed(fn):
            stack_start()
            for t in range(min(Wu, 8)):
                fn(t)
            stack_start()
            g, w = hb.timer(lambda: [fn(t) for t in range(KL)])
            return max(g, w)

        ms_eager = timed(eager)
        ln0, _ = st.layers[L - 1].counters()
        assert np.array_equal(ln0, np.full(wl.batch, KL)) and st.layers[0].poll_error() == 0
        st.graph_capture([q[l % KL] for l in range(L)], [k[l % KL] for l in range(L)],
                         [v[l % KL] for l in range(L)], outs)
        ms_graph = timed(lambda t: st.graph_launch())
        ln0, _ = st.layers[L - 1].counters()
        assert np.array_equal(ln0, np.full(wl.batch, KL)) and st.layers[0].poll_error() == 0
        best = min(ms_eager, ms_graph)
        nb, toks = path_bytes(wl, hb.lengths, 0, KL, hb.prompt_len)
        res["stack"] = {
            "layers": L, "steps": KL, "cache_gbytes": st.cache.numel() / 1e9, "plan": list(st.layers[0].plan()),
            "metric": "rollout decode tokens/s per model of %d layers (bounded window), first %d steps of the run" % (L, KL),
            "value": toks / (best * 1e-3), "unit": "tokens/s",
            "ms_per_step_eager": ms_eager / KL, "ms_per_step_graph": ms_graph / KL,
            "hbm_frac_whole_path": L * nb / (best * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }
        del st

    if args.calibrate or not args.headline_only:
        # what a plain streaming read of 1 GiB reaches on this GPU, measured here: the practical ceiling beside the
        # published peak (and, under a profiler's counters, the kernels of known size that scale its byte counters)
        nbytes = 1 << 30
        src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=dev)
        sink = torch.zeros(4, dtype=torch.uint8, device=dev)
        if args.calibrate:
            dst = torch.empty_like(src)
        for _ in range(5):
            if args.calibrate:
                ptenc.ptenc_util_copy(dst, src, nbytes, 2048)
            ptenc.ptenc_util_stream_read(src, nbytes, sink, 2048)

        def gbs(fn, iters=20):
            g, _ = hb.timer(lambda: [fn() for _ in range(iters)])
            return nbytes * iters / (g * 1e-3) / 1e9
        ceiling = {"stream_read_GB_per_s": gbs(lambda: ptenc.ptenc_util_stream_read(src, nbytes, sink, 2048)),
                   "stream_read_nontemporal_GB_per_s": gbs(lambda: ptenc.ptenc_util_stream_read_nt(src, nbytes, sink, 2048)),
                   "bytes_per_launch": nbytes, "launches_each": 20,
                   "what": "the library's plain read kernel over 1 GiB, 2048 workgroups, back to back"}
        res["measured_stream_ceiling"] = ceiling
        res["roofline"]["frac_of_measured_stream_ceiling"] = res["roofline"]["achieved"] / max(
            ceiling["stream_read_GB_per_s"], ceiling["stream_read_nontemporal_GB_per_s"])
        if args.calibrate:
            res["calibration"] = {"copy_kernel_bytes_read": nbytes, "copy_kernel_bytes_written": nbytes,
                                  "read_kernel_bytes_read": nbytes, "launches_each": 5}
            del dst
        del src

    # ---- the other configurations: last-K-step and whole-run figures, same process ----
    if not args.headline_only and not args.no_workloads and args.workload == "qwen7b" and not args.chunk \
            and args.policy == "sliding":
        del hb
        torch.cuda.empty_cache()
        others = {}
        for name in ("qwen3b", "llama8b", "ragged", "tiny_f32"):
            w2 = I.WORKLOADS[name]
            nb2 = w2.steps * w2.batch * (2 * w2.d_q + 2 * w2.d_kv) * w2.elem_bytes
            ob = Bench(w2, args, torch, np, I, ptenc, resident=nb2 <= (40 << 30))
            # two eviction periods at a full ring: long enough for the shorter steps of these shapes to be timed
            # as a region of their own, and every rollout evicts twice in it
            K2 = max(20, 2 * w2.chunk)
            if w2.ragged:
                # steady state of a ragged batch is not one window size: the K steps right after every ring that
                # will fill has filled (most rollouts still running), and the whole run
                t_a = w2.window + 2 * w2.chunk
                ob.start()
                ob.launch(0, t_a)
                g1, w1 = ob.timer(ob.prepared(t_a, t_a + K2))
                steady = ob.figures(t_a, t_a + K2, g1, w1)
                steady["window"] = "steps %d..%d of the run (every ring that fills has filled; %d of %d rollouts still running)" % (
                    t_a + 1, t_a + K2, int((ob.lengths > t_a).sum()), w2.batch)
                ob.start()
                g, w = ob.run_timed(0, ob.T)
                ob.check_counters(ob.T)
                full = ob.figures(0, ob.T, g, w)
            else:
                steady, full = steady_and_full(ob, K2, Wu, seg_steps)
            others[name] = {"workload": ob.describe(), "attn_kernel": "mfma" if ob.attn_kernel == 1 else "generic",
                            "window_splits": ob.n_splits, "last_steps": steady, "full_run": full}
            del ob
            torch.cuda.empty_cache()
        res["workloads"] = others

    if not args.no_cpu_baseline and not args.headline_only:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
