"""The stored oracle outputs (tests/golden/oracle_small_case.json and scored_small_case.json, written by
make_oracle_golden.py from the oracles alone): the oracles still reproduce them, and the HIP path
matches them."""
import importlib.util
import json
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
GOLDEN = os.path.join(HERE, "golden", "oracle_small_case.json")


SCORED = os.path.join(HERE, "golden", "scored_small_case.json")


def _load(path=GOLDEN):
    with open(path) as f:
        return json.load(f)


def _maker():
    spec = importlib.util.spec_from_file_location("make_oracle_golden", os.path.join(HERE, "golden", "make_oracle_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_reproduces_its_golden_file():
    now, then = _maker().compute(), _load()
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


def test_scored_oracle_reproduces_its_golden_file():
    now, then = _maker().compute_scored(), _load(SCORED)
    assert now["victims"] == then["victims"] and len(then["victims"]) == 3        # ceil((170 - 96) / 32) evictions
    assert now["positions"] == then["positions"] and now["len"] == then["len"] and now["base"] == then["base"] == [96, 96]
    assert then["min_margin"] > 2e-2                                              # no selection was close to a tie
    assert np.allclose(now["scores"], then["scores"], rtol=1e-12, atol=1e-14)
    assert np.allclose(now["S_final"], then["S_final"], rtol=1e-12, atol=1e-14)
    # the policy did not simply slide: what is left is not a run of consecutive positions
    assert any(p != list(range(p[0], p[0] + len(p))) for p in then["positions"])


@pytest.mark.gpu
def test_hip_scored_policy_matches_the_golden_file():
    from paper_2602_16839_amd import inputs as I
    from paper_2602_16839_amd import ptenc
    from tests import helpers as H
    g = _load(SCORED)
    wl = I.WORKLOADS[g["workload_base"]].replace(**g["case"])
    enc = I.encoder_params(wl)
    layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk, dtype=wl.torch_dtype,
                        n_global=wl.n_global, rank=wl.rank, poison_cache=True)
    layer.set_option(ptenc.OPT_RECENT, g["n_recent"])
    layer.set_option(ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED)
    dev = {k: v.cuda() for k, v in enc.items()}
    layer.set_encoder(dev["q_g"], dev["WaQ"], dev["WaK"], dev["WaV"], dev["k_g"], dev["v_g"])
    layer.reset()
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    q = (q.float() * g["q_gain"]).to(q.dtype)
    q, k, v = q.cuda(), k.cuda(), v.cuda()
    seen, last = [], None
    for t in range(wl.steps):
        layer.step(q[t], k[t], v[t])
        vic = layer.victims().tolist()
        if vic[0][0] >= 0 and vic != last:             # a new selection was made
            seen.append(vic)
            last = vic
    assert seen == g["victims"]
    ln, base = layer.counters()
    assert ln.tolist() == g["len"] and base.tolist() == g["base"]
    sc, ps = layer.scores()
    for b in range(wl.batch):
        n = len(g["positions"][b])
        assert ps[b, :n].tolist() == g["positions"][b]
        ref = np.array(g["scores"][b])
        assert (np.abs(sc[b, :n] - ref) <= 1e-4 + 1e-3 * np.abs(ref)).all()
    H.assert_close(layer.get_state(), np.array(g["S_final"]), H.S_ABS, H.S_REL, "golden S (scored)")
