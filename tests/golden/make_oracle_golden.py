#!/usr/bin/env python3
"""Writes tests/golden/oracle_small_case.json: outputs of the CPU oracle (and nothing else) on a small
seeded case.  Run from the repository root:  python tests/golden/make_oracle_golden.py

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


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_case.json")
    with open(path, "w") as f:
        json.dump(compute(), f)
    print("wrote", path)
