"""Where a decode step's time goes, workgroup by workgroup.

Runs against the profiling build of the library (``python -m paper_2602_16839_amd.build --timeline``,
-DPTENC_TIMELINE), in which thread 0 of every workgroup of the step kernel notes the 100 MHz wall clock at the
boundaries of the step's phases.  A workload's run is decoded up to a full ring, then single steps are launched
one at a time (synchronised in between) and their stamps read back:

    python -m paper_2602_16839_amd.step_timeline --workload qwen7b [--policy scored] [--splits N] [--steps 32]
    python -m paper_2602_16839_amd.step_timeline --workload ragged --listed 8     # a compact list of 8 rollouts

(with --listed the rings are not decoded up to their size: the counters are set to a window one chunk short of
full over whatever the cache holds, which is all a timing needs).

Times are microseconds from the first workgroup's entry.  Synthetic inputs (paper_2602_16839_amd.inputs).
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
os.environ.setdefault("PTENC_LIB", os.path.join(PKG_DIR, "libptenc_timeline.so"))

import numpy as np   # noqa: E402
import torch         # noqa: E402

from . import inputs as I, ptenc   # noqa: E402

NAMES = {0: "entry", 1: "counters and queries there, walk begins", 2: "walk ends (wavefront 0)", 3: "wavefronts merged",
         4: "scores folded (scored policy)", 6: "window splits: partial handed over, ticket taken", 5: "result out"}


def timeline_region(cfg):
    fn = getattr(ptenc.lib(), "ptenc_timeline_region", None)
    if fn is None:
        raise RuntimeError("%s is not the profiling build: build it with `python -m paper_2602_16839_amd.build --timeline`"
                           % os.environ["PTENC_LIB"])
    off, nb, slots = C.c_size_t(), C.c_size_t(), C.c_int()
    fn.argtypes = [C.POINTER(ptenc.Config), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_int)]
    if fn(C.byref(cfg), C.byref(off), C.byref(nb), C.byref(slots)) != 0:
        raise RuntimeError("ptenc_timeline_region failed")
    return off.value, nb.value, slots.value


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="qwen7b")
    ap.add_argument("--policy", choices=["sliding", "scored"], default="sliding")
    ap.add_argument("--splits", type=int, default=0, help="window splits (0 = the library's plan)")
    ap.add_argument("--steps", type=int, default=32, help="single steps measured, at a full ring")
    ap.add_argument("--listed", type=int, default=0,
                    help="launch the steps for a compact list of this many rollouts (0 = the full batch)")
    args = ap.parse_args()

    wl = I.WORKLOADS[args.workload]
    if wl.torch_dtype != torch.bfloat16 or (wl.ragged and not args.listed):
        print("step_timeline: the bf16 path only; a ragged workload through --listed", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk, dtype=wl.torch_dtype,
                        n_global=wl.n_global, rank=wl.rank, n_sink=wl.n_sink)
    if args.splits:
        layer.set_option(ptenc.OPT_SPLITS, args.splits)
    if args.policy == "scored":
        layer.set_option(ptenc.OPT_RECENT, -1)
        layer.set_option(ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED)
    e = I.encoder_params(wl, device=dev)
    layer.set_encoder(e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"])
    off, nbytes, slots = timeline_region(layer.cfg)
    stamps_dev = layer.state[off: off + nbytes].view(torch.int64).view(-1, slots)

    # up to a full ring that has evicted at least once, in pieces (inputs generated per piece)
    W, Cc = wl.window - wl.n_sink, wl.chunk
    t_full = W + 2 * Cc + 3              # two evictions behind it, not an evicting step itself for a few steps
    layer.reset()
    if wl.n_sink:
        pk, pv = I.prompt_kv(wl, device=dev)
        layer.prefill(pk, pv, I.prompt_lengths(wl))
    t = 0
    n_meas = min(args.steps, Cc - 8)      # stay clear of the next evicting step
    ids = None
    if args.listed:
        n_l = min(args.listed, wl.batch)
        ids = torch.arange(n_l, dtype=torch.int32, device=dev)
        layer.cache.zero_()
        layer.set_counters(np.full(wl.batch, W - Cc - n_meas - 1, dtype=np.int64), np.zeros(wl.batch, dtype=np.int64))
    else:
        while t < t_full:
            n = min(512, t_full - t)
            q, k, v = I.qkv_steps(wl, t, t + n, device=dev)
            layer.run(q, k, v, torch.empty_like(q))
            t += n
    torch.cuda.synchronize()
    q, k, v = I.qkv_steps(wl, t, t + n_meas, device=dev)
    if ids is not None:
        q, k, v = q[:, :n_l].contiguous(), k[:, :n_l].contiguous(), v[:, :n_l].contiguous()
    out = torch.empty_like(q)
    per_step, waves, ev_us = [], [], []
    for j in range(n_meas):
        stamps_dev.zero_()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        if ids is None:
            layer.step(q[j], k[j], v[j], out[j])
        else:
            layer.step_ids(q[j], k[j], v[j], ids, out[j])
        e1.record()
        torch.cuda.synchronize()
        st = stamps_dev.cpu().numpy().astype(np.float64) / 100.0        # 100 MHz -> us
        used = (st[:, 0] > 0) & (st[:, 5] > 0)      # attention workgroups (encoding workgroups of their own stamp their entry only)
        st = st[used]
        st = np.where(st > 0, st - st[:, 0].min(), np.nan)
        per_step.append(st[:, :8])
        waves.append(st[:, 8:16])
        ev_us.append(e0.elapsed_time(e1) * 1e3)
    assert layer.poll_error() == 0
    if len({x.shape[0] for x in per_step}) != 1:
        print("step_timeline: the measured steps differ in their launch shape", file=sys.stderr)
        return 1
    r = np.stack(per_step[4:])            # [steps, workgroups, 8]; the first few steps warm up
    wv = np.stack(waves[4:])
    print("workload %s, policy %s: %s, %d attention workgroups stamped; %d single steps (window %s), %.1f us each by HIP "
          "events (a single launch between two synchronisations)" % (
              args.workload, args.policy,
              "%d rollouts x %d KV heads" % (wl.batch, wl.n_kv_heads) if ids is None
              else "a compact list of %d of %d rollouts x %d KV heads" % (n_l, wl.batch, wl.n_kv_heads),
              r.shape[1], r.shape[0], "full, %d" % W if ids is None else "about %d" % (W - Cc), float(np.mean(ev_us[4:]))))
    print("%-52s %10s %10s %10s %24s" % ("phase boundary (us from the first workgroup's entry)", "mean", "median", "p95",
                                        "latest workgroup (mean)"))
    for kk in (0, 1, 2, 3, 4, 6, 5):
        x = r[:, :, kk]
        if np.all(np.isnan(x)):
            continue
        print("%-52s %10.2f %10.2f %10.2f %24.2f" % (NAMES[kk], np.nanmean(x), np.nanmedian(x), np.nanpercentile(x, 95),
                                                     float(np.mean(np.nanmax(x, axis=1)))))
    end = np.nanmean(r[:, :, 5], axis=0)
    n_wg = end.shape[0]
    idx = np.arange(n_wg)
    print("result out, by workgroup index: even %.1f, odd %.1f; first half of the grid %.1f, second half %.1f" % (
        end[idx % 2 == 0].mean(), end[idx % 2 == 1].mean(), end[: n_wg // 2].mean(), end[n_wg // 2:].mean()))
    hist, edges = np.histogram(end, bins=12)
    print("result out, histogram over workgroups: " + "  ".join("%.1f-%.1f us: %d" % (edges[i], edges[i + 1], hist[i])
                                                                for i in range(len(hist)) if hist[i]))
    nw = 8 if np.any(wv[:, :, 4:] > 0) else 4
    print("walk ends, by wavefront of the workgroup (mean): " + "  ".join("%.2f" % x for x in np.nanmean(wv[:, :, :nw], axis=(0, 1))))
    return 0


if __name__ == "__main__":
    sys.exit(main())
