#!/usr/bin/env python3
"""Benchmark of the bounded-cache rollout decode path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen7b] [--splits S]

A step is one pass of the whole hot path (evict-and-encode where a window is full, ring append,
windowed GQA decode attention) over one batch of B rollouts.  The default workload is the
Qwen2.5-7B-shaped layer (bf16, 28 query / 4 KV heads, head_dim 128, window 4096, chunk 128,
128 rollouts) decoded for 8192 steps from an empty cache; inputs are synthetic, seeded, and
resident in HBM before the timed region starts.

Prints ONE JSON line: whole-job decode tokens/s, the HBM roofline of the step kernel
(algorithmic bytes per launch / mean launch time measured with HIP events on the launch
stream), and the CPU oracle timed on the host cores on a bounded sample of the same workload.
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
    """Live tokens the attention of decode step t (1-based) reads, lazy chunk eviction."""
    return t if t <= W else W - C + ((t - W - 1) % C) + 1


def attention_bytes_per_step(wl, lengths, steps: int, prompt_len=None):
    """Algorithmic bytes of the attention launch of every step: K and V stream over the question
    tokens and the live window plus q in and out out, for every active rollout."""
    import numpy as np
    s = wl.elem_bytes
    per_tok = 2 * wl.d_kv * s
    qo = 2 * wl.d_q * s
    out = np.zeros(steps, dtype=np.float64)
    act = np.zeros(steps, dtype=np.int64)
    uniq = {}
    pls = [0] * len(lengths) if prompt_len is None else prompt_len.tolist()
    for L, P in zip(lengths.tolist(), pls):
        uniq[(L, P)] = uniq.get((L, P), 0) + 1
    nl = np.array([n_live_at(t, wl.window - wl.n_sink, wl.chunk) for t in range(1, steps + 1)], dtype=np.float64)
    for (L, P), cnt in uniq.items():
        n = min(L, steps)
        out[:n] += cnt * (per_tok * (nl[:n] + P) + qo)
        act[:n] += cnt
    return out, act


def prologue_bytes_total(wl, lengths, steps: int) -> float:
    """Algorithmic bytes of append (every active step) and of evict-and-encode (chunk re-read plus
    the read-modify-write of S) over the run."""
    s = wl.elem_bytes
    tot = 0.0
    for L in lengths.tolist():
        n = min(L, steps)
        tot += n * 2 * wl.d_kv * s
        ring = wl.window - wl.n_sink
        ev = 0 if n <= ring else math.ceil((n - ring) / wl.chunk)
        tot += ev * (2 * wl.chunk * wl.d_kv * s + 2 * wl.n_global * wl.rank * 4)
    return tot


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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="decode steps to time (0 = the workload's full run)")
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="qwen7b")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--encode-parts", type=int, default=0,
                    help="workgroups that share one evicted chunk's encoding (0 = the library's heuristic)")
    ap.add_argument("--chunk", type=int, default=0,
                    help="override the workload's eviction chunk C (eviction-ratio sweeps; 0 = the workload's own)")
    ap.add_argument("--ragged-mode", choices=["compact", "masked"], default="compact",
                    help="ragged workloads: drop finished rollouts from the batch (rollout-id lists) or mask them")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true", help="skip the per-launch HIP-event pass")
    ap.add_argument("--extras", action="store_true",
                    help="also time the state-as-weight-delta application (and the question-token prefill)")
    ap.add_argument("--policy", choices=["sliding", "scored"], default="sliding",
                    help="which tokens an eviction takes: the oldest chunk, or the lowest accumulated attention probability")
    ap.add_argument("--recent", type=int, default=-1, help="scored policy: most recent ring entries never taken (-1 = half the ring)")
    ap.add_argument("--layers", type=int, default=0,
                    help="also time a stack of this many layers (each with its own cache) over the same steps: "
                         "eager launches, then replays of the recorded one-step HIP graph")
    ap.add_argument("--stagger", action="store_true",
                    help="also time steady-state steps with the rollouts' evictions spread evenly over the steps "
                         "(a running batch whose rollouts started at different times) next to all evicting together")
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
    K = args.steps if args.steps > 0 else wl.steps
    Wu = max(0, args.warmup)
    lengths = I.rollout_lengths(wl)
    if wl.ragged:
        K = min(K, int(lengths.max()))

    # ---- synthetic inputs, resident in HBM ----
    T_gen = max(K, Wu)
    q = torch.empty((T_gen, wl.batch, wl.n_q_heads, wl.head_dim), dtype=wl.torch_dtype, device=dev)
    k = torch.empty((T_gen, wl.batch, wl.n_kv_heads, wl.head_dim), dtype=wl.torch_dtype, device=dev)
    v = torch.empty_like(k)
    blk = max(1, (1 << 26) // (wl.batch * wl.d_q))
    for t0 in range(0, T_gen, blk):
        t1 = min(T_gen, t0 + blk)
        q[t0:t1], k[t0:t1], v[t0:t1] = I.qkv_steps(wl, t0, t1, device=dev)
    active = None
    compact = wl.ragged and args.ragged_mode == "compact"
    row_offsets = None
    if wl.ragged:
        tt = torch.arange(T_gen, device=dev).view(-1, 1)
        alive = tt < torch.from_numpy(lengths).to(dev).view(1, -1)          # [T, B]
        if compact:
            # what a rollout engine feeds: only the rollouts still running, with their ids
            ids = torch.nonzero(alive)[:, 1].to(torch.int32).contiguous()
            q, k, v = q[alive].contiguous(), k[alive].contiguous(), v[alive].contiguous()
            counts = np.array([(lengths > t).sum() for t in range(T_gen)], dtype=np.int64)
            row_offsets = np.concatenate([[0], np.cumsum(counts)])
        else:
            active = alive.to(torch.uint8).contiguous()
    out = torch.empty_like(q)
    enc = I.encoder_params(wl, device=dev)

    layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                        dtype=wl.torch_dtype, n_global=wl.n_global, rank=wl.rank, n_sink=wl.n_sink)
    prompt_len = I.prompt_lengths(wl) if wl.n_sink else None
    if wl.n_sink:
        pk, pv = I.prompt_kv(wl, device=dev)

    def start_run():
        # an empty cache, question tokens (if the workload has any) prefilled: not part of the timed steps
        layer.reset()
        if wl.n_sink:
            layer.prefill(pk, pv, prompt_len)

    if args.splits:
        layer.set_option(ptenc.OPT_SPLITS, args.splits)
    if args.encode_parts:
        layer.set_option(ptenc.OPT_ENCODE_PARTS, args.encode_parts)
    if args.policy == "scored":
        layer.set_option(ptenc.OPT_RECENT, args.recent)
        layer.set_option(ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED)
    layer.set_encoder(enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    attn_kernel, n_splits, _ = layer.plan()

    # ---- warmup, then the timed run from an empty cache ----
    def run_steps(t0, t1):
        if compact:
            r0, r1 = int(row_offsets[t0]), int(row_offsets[t1])
            layer.run_ids(q[r0:r1], k[r0:r1], v[r0:r1], ids[r0:r1], row_offsets[t0:t1 + 1] - r0, out[r0:r1])
        else:
            layer.run(q[t0:t1], k[t0:t1], v[t0:t1], out[t0:t1], None if active is None else active[t0:t1])

    start_run()
    if Wu:
        run_steps(0, Wu)
    start_run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0 = time.perf_counter()
    e0.record()
    run_steps(0, K)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - w0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    total_ms = max(gpu_ms, wall_ms)
    assert layer.poll_error() == 0
    ln, base = layer.counters()
    assert np.array_equal(ln, np.minimum(lengths, K)), "counters after the run are not the step count"

    abytes, act = attention_bytes_per_step(wl, lengths, K, prompt_len)
    tokens = int(act.sum())
    value = tokens / (total_ms * 1e-3)
    all_bytes = float(abytes.sum()) + prologue_bytes_total(wl, lengths, K)

    # ---- launch time of the dominant kernel with HIP events on the launch stream (second pass over the
    #      same steps).  On the MFMA path one launch is one whole decode step and nothing else runs in
    #      between, so the events bracket runs of EV_EVERY back-to-back launches: an event pair around
    #      every single launch adds about 2 us to each (it breaks the back-to-back dispatch), which is
    #      not kernel time.  The plain path's attention launches are bracketed one by one. ----
    roofline = None
    fused = attn_kernel == 1
    EV_EVERY = 32
    if not args.no_kernel_timing:
        start_run()
        evs = []
        if fused:
            for t0 in range(0, K, EV_EVERY):
                pair = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                pair[0].record()
                run_steps(t0, min(K, t0 + EV_EVERY))
                pair[1].record()
                evs.append(pair)
        else:
            for t in range(K):
                a = None if active is None else active[t]
                pair = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                layer.evict_encode(a)
                layer.append(k[t], v[t], a)
                pair[0].record()
                layer.attend(q[t], out[t], a)
                pair[1].record()
                evs.append(pair)
        torch.cuda.synchronize()
        kern_ms = float(sum(a.elapsed_time(b) for a, b in evs))
        mean_s = kern_ms * 1e-3 / K
        launch_bytes = (all_bytes if fused else float(abytes.sum())) / K
        achieved = launch_bytes / mean_s / 1e9
        traffic = None
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % wl.name)
        if os.path.exists(tpath) and K == wl.steps:
            with open(tpath) as fh:
                traffic = json.load(fh).get("traffic_bytes_per_launch")
        roofline = {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "kernel": "decode_mfma_kernel (evict-encode + append + attention in one launch)" if fused
                      else "attn_generic_kernel + combine_kernel",
            "launches": K, "mean_launch_us": mean_s * 1e6, "algorithmic_bytes_per_launch": launch_bytes,
            "launches_per_event_pair": EV_EVERY if fused else 1,
        }

    res = {
        "metric": "rollout decode tokens/s per layer (bounded window)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wu,
        "ms_per_step": total_ms / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {
            "workload": "%s-shaped layer: B %d rollouts, %d Q / %d KV heads, head_dim %d, window %d, chunk %d, "
                        "%d decode steps from an empty cache%s%s" % (
                            wl.name, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk, K,
                            (", ragged lengths, finished rollouts %s" % ("dropped from the batch (rollout-id lists)"
                                                                        if compact else "masked")) if wl.ragged else "",
                            ", %d slots reserved for question tokens (128..%d per rollout, prefilled)" % (
                                wl.n_sink, wl.n_sink) if wl.n_sink else ""),
            "name": wl.name, "batch": wl.batch, "window": wl.window, "chunk": wl.chunk, "tokens": tokens,
            "attn_kernel": "mfma" if attn_kernel == 1 else "generic", "window_splits": n_splits,
            "evict_policy": args.policy,
            "parallelism": "single GPU",
        },
        "gpu_ms": gpu_ms, "wall_ms": wall_ms,
        "hbm_frac_whole_path": all_bytes / (total_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "algorithmic_gbytes": all_bytes / 1e9,
        "roofline": roofline,
    }
    if args.stagger and not wl.ragged and not wl.n_sink and args.policy == "sliding":
        # steady state, rings nearly full: the cache keeps what the run left (the counters are re-based, so
        # positions and contents no longer correspond: timing only)
        Wr, C, B = wl.window, wl.chunk, wl.batch
        ns = min(2 * C, K)
        zeros = np.zeros(B, dtype=np.int64)

        def timed_from(ln):
            best = None
            for _ in range(3):
                layer.set_counters(ln, zeros)
                torch.cuda.synchronize()
                a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a0.record()
                layer.run(q[:ns], k[:ns], v[:ns], out[:ns])
                a1.record()
                torch.cuda.synchronize()
                us = a0.elapsed_time(a1) * 1e3 / ns
                best = us if best is None else min(best, us)
            return best

        together = timed_from(np.full(B, Wr - C // 2, dtype=np.int64))
        spread = timed_from((Wr - (np.arange(B) * C // B) % C).astype(np.int64))
        res["staggered_evictions"] = {"steps": ns, "us_per_step_all_evicting_together": together,
                                      "us_per_step_evictions_spread_over_steps": spread}
    if args.extras:
        # y += ((x A) S) B at the model's hidden size (the query projection width stands in for it)
        ex = {}
        d_h = wl.d_q
        ad = I.adapter_inputs(wl, d_h, d_h, device=dev)
        yb = ad["y"].clone()
        for _ in range(10):
            layer.apply_delta(ad["x"], ad["At"], ad["Bt"], yb)
        torch.cuda.synchronize()
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record()
        for _ in range(200):
            layer.apply_delta(ad["x"], ad["At"], ad["Bt"], yb)
        a1.record()
        torch.cuda.synchronize()
        us = a0.elapsed_time(a1) * 1e3 / 200
        s_ = wl.elem_bytes
        nbytes_ad = wl.batch * (d_h * s_ + 2 * d_h * s_ + wl.n_global * wl.rank * 4) + (wl.n_global + wl.rank) * d_h * s_
        ex["apply_delta"] = {"d_in": d_h, "d_out": d_h, "us_per_call": us, "algorithmic_bytes": nbytes_ad,
                             "GB_per_s": nbytes_ad / us / 1e3, "hbm_frac": nbytes_ad / us / 1e3 / HBM_PEAK_GBS}
        if wl.n_sink:
            torch.cuda.synchronize()
            a0.record()
            for _ in range(20):
                layer.prefill(pk, pv, prompt_len)
            a1.record()
            torch.cuda.synchronize()
            us = a0.elapsed_time(a1) * 1e3 / 20
            nb = float(prompt_len.sum()) * 2 * wl.d_kv * s_ * 2          # read once, written once
            ex["prefill"] = {"us_per_call": us, "algorithmic_bytes": nb, "GB_per_s": nb / us / 1e3}
        res["extras"] = ex
    if args.layers > 0 and not wl.ragged:
        # L layers, each with its own cache, counters and state; layer l reads the inputs of step t + 7 l
        L = args.layers
        del layer
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
                    lay.prefill(pk, pv, prompt_len)

        outs = [out[l % T_gen] for l in range(L)]

        def eager(t):
            idx = [(t + 7 * l) % T_gen for l in range(L)]
            st.step([q[i] for i in idx], [k[i] for i in idx], [v[i] for i in idx], outs)

        def timed(fn):
            stack_start()
            for t in range(min(Wu, 8)):
                fn(t)
            stack_start()
            torch.cuda.synchronize()
            s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0 = time.perf_counter()
            s0.record()
            for t in range(K):
                fn(t)
            s1.record()
            torch.cuda.synchronize()
            return max(s0.elapsed_time(s1), (time.perf_counter() - c0) * 1e3)

        ms_eager = timed(eager)
        ln0, _ = st.layers[L - 1].counters()
        assert np.array_equal(ln0, np.full(wl.batch, K)) and st.layers[0].poll_error() == 0
        st.graph_capture([q[l % T_gen] for l in range(L)], [k[l % T_gen] for l in range(L)],
                         [v[l % T_gen] for l in range(L)], outs)
        ms_graph = timed(lambda t: st.graph_launch())
        ln0, _ = st.layers[L - 1].counters()
        assert np.array_equal(ln0, np.full(wl.batch, K)) and st.layers[0].poll_error() == 0
        best = min(ms_eager, ms_graph)
        res["stack"] = {
            "layers": L, "cache_gbytes": st.cache.numel() / 1e9, "plan": list(st.layers[0].plan()),
            "metric": "rollout decode tokens/s per model of %d layers (bounded window)" % L,
            "value": tokens / (best * 1e-3), "unit": "tokens/s",
            "ms_per_step_eager": ms_eager / K, "ms_per_step_graph": ms_graph / K,
            "hbm_frac_whole_path": L * all_bytes / (best * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }
        del st
    if args.calibrate:
        nbytes = 1 << 30
        src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        sink = torch.zeros(4, dtype=torch.uint8, device=dev)
        for _ in range(5):
            ptenc.ptenc_util_copy(dst, src, nbytes, 2048)
            ptenc.ptenc_util_stream_read(src, nbytes, sink, 2048)
        torch.cuda.synchronize()
        def gbs(fn, iters=20):
            torch.cuda.synchronize()
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record()
            for _ in range(iters):
                fn()
            c1.record()
            torch.cuda.synchronize()
            return nbytes * iters / (c0.elapsed_time(c1) * 1e-3) / 1e9
        res["calibration"] = {"copy_kernel_bytes_read": nbytes, "copy_kernel_bytes_written": nbytes,
                              "read_kernel_bytes_read": nbytes, "launches_each": 5,
                              "stream_read_GB_per_s": gbs(lambda: ptenc.ptenc_util_stream_read(src, nbytes, sink, 2048)),
                              "stream_read_nontemporal_GB_per_s": gbs(lambda: ptenc.ptenc_util_stream_read_nt(src, nbytes, sink, 2048))}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
