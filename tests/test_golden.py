"""The stored oracle outputs (tests/golden/oracle_small_case.json, written by make_oracle_golden.py from
the oracle alone): the oracle still reproduces them, and the HIP path matches them."""
import importlib.util
import json
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
GOLDEN = os.path.join(HERE, "golden", "oracle_small_case.json")


def _load():
    with open(GOLDEN) as f:
        return json.load(f)


def test_oracle_reproduces_its_golden_file():
    spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(HERE, "golden", "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now, then = mod.compute(), _load()
    assert now["len"] == then["len"] == [100, 100] and now["base"] == then["base"] == [48, 48]   # 24 * ceil(36 / 24)
    assert np.allclose(now["S_final"], then["S_final"], rtol=1e-12, atol=1e-14)
    assert np.allclose(now["S0"], then["S0"], rtol=1e-12, atol=1e-14)
    for t in then["sample_steps"]:
        assert np.allclose(now["out_first8"][str(t)], then["out_first8"][str(t)], rtol=1e-12, atol=1e-15)


@pytest.mark.gpu
def test_hip_path_matches_the_golden_file():
    from paper_2602_16839_amd import inputs as I
    from tests import helpers as H
    g = _load()
    wl = I.WORKLOADS[g["workload_base"]].replace(**g["case"])
    enc = I.encoder_params(wl)
    layer = H.make_layer(wl, enc)
    q, k, v = (x.cuda() for x in I.qkv_steps(wl, 0, wl.steps))
    out = layer.run(q, k, v)
    for t in g["sample_steps"]:
        H.assert_close(H.f64(out[t - 1])[:, :, :8], np.array(g["out_first8"][str(t)]), H.BF16_ABS, H.BF16_REL,
                       "golden out step %d" % t)
    ln, base = layer.counters()
    assert ln.tolist() == g["len"] and base.tolist() == g["base"]
    H.assert_close(layer.get_state(), np.array(g["S_final"]), H.S_ABS, H.S_REL, "golden S")
    H.assert_close(layer.encoder_state()[1], np.array(g["S0"]), H.S_ABS, H.S_REL, "golden S0")
