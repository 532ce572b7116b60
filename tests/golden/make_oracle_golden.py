#!/usr/bin/env python3
"""Writes tests/golden/oracle_small_case.json and tests/golden/scored_small_case.json: outputs of the
CPU oracles (and nothing else) on small seeded cases.  Run from the repository root:
python tests/golden/make_oracle_golden.py

The file is a regression anchor: the oracle must keep reproducing it (a CPU test), and the HIP path is
compared with it as well (a GPU test).  The paper prints no numeric values for this path, so these are
the oracle's numbers, not the paper's; what pins the oracle itself is tests/test_oracle_pins.py.
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402
import torch  # noqa: E402

from oracle import pte_oracle as po  # noqa: E402
from oracle import scored_oracle as so  # noqa: E402
from paper_2602_16839_amd import inputs as I  # noqa: E402

# bf16 inputs, 2 rollouts, 4 query / 2 KV heads, head_dim 128, window 64, chunk 24 (wraps), 100 steps
CASE = dict(batch=2, n_q_heads=4, n_kv_heads=2, window=64, chunk=24, steps=100, n_global=8, rank=16)
SAMPLE_STEPS = [1, 2, 40, 64, 65, 89, 100]


def compute():
    wl = I.WORKLOADS["qwen3b"].replace(**CASE)
    enc = {k: v.to(torch.float64).numpy() for k, v in I.encoder_params(wl).items()}
    orc = po.OracleLayer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                         enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    q, k, v = (x.to(torch.float64).numpy() for x in I.qkv_steps(wl, 0, wl.steps))
    outs = {}
    for t in range(wl.steps):
        o = orc.step(q[t], k[t], v[t])
        if t + 1 in SAMPLE_STEPS:
            outs[str(t + 1)] = o[:, :, :8].tolist()          # first 8 columns of every (rollout, head)
    ln, base = orc.counters()
    return {
        "case": CASE, "workload_base": "qwen3b", "sample_steps": SAMPLE_STEPS,
        "out_first8": outs, "len": ln.tolist(), "base": base.tolist(),
        "S0": orc.S0.tolist(), "S_final": orc.state().tolist(),
    }


# importance-based eviction: bf16, 2 rollouts, 14 query / 2 KV heads, window 96, chunk 32, 24 recent entries
# protected, queries scaled by 48 so that the attention is peaked and the scores spread out
SCORED_CASE = dict(batch=2, n_q_heads=14, n_kv_heads=2, window=96, chunk=32, steps=170, n_global=8, rank=16)
SCORED_RECENT, SCORED_GAIN = 24, 48.0


def compute_scored():
    wl = I.WORKLOADS["qwen7b"].replace(**SCORED_CASE)
    enc = {k: v.to(torch.float64).numpy() for k, v in I.encoder_params(wl).items()}
    orc = so.ScoredOracleLayer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk, SCORED_RECENT,
                               enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    q = (q.float() * SCORED_GAIN).to(q.dtype)
    q, k, v = (x.to(torch.float64).numpy() for x in (q, k, v))
    victims = []                                   # [eviction][rollout] -> positions, ring order
    for t in range(wl.steps):
        before = list(orc.evicted)
        orc.step(q[t], k[t], v[t])
        if list(orc.evicted) != before:
            victims.append([list(map(int, orc.last_victims[b])) for b in range(wl.batch)])
    ln, base = orc.counters()
    return {
        "case": SCORED_CASE, "workload_base": "qwen7b", "n_recent": SCORED_RECENT, "q_gain": SCORED_GAIN,
        "victims": victims, "len": ln.tolist(), "base": base.tolist(), "min_margin": orc.min_margin,
        "positions": [orc.positions(b).tolist() for b in range(wl.batch)],
        "scores": [orc.scores(b).tolist() for b in range(wl.batch)],
        "S_final": orc.state().tolist(),
    }


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    for name, fn in (("oracle_small_case.json", compute), ("scored_small_case.json", compute_scored)):
        with open(os.path.join(here, name), "w") as f:
            json.dump(fn(), f)
        print("wrote", os.path.join(here, name))
