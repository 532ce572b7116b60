"""The multi-layer driver: L layers stepped through ptenc_stack_decode_step and through the recorded
HIP graph, against L independent oracle layers fed the same per-layer seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2602_16839_amd import inputs as I
from paper_2602_16839_amd import ptenc
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _layer_workloads(wl, L):
    # a layer's parameters and inputs are those of the same workload under another seed
    return [wl.replace(seed=wl.seed + 7919 * l) for l in range(L)]


def _make_stack(wl, L, encs):
    st = ptenc.Stack(L, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                     dtype=wl.torch_dtype, n_global=wl.n_global, rank=wl.rank, poison_cache=True, n_sink=wl.n_sink)
    for l, enc in enumerate(encs):
        dev = {k: v.cuda() for k, v in enc.items()}
        st.layers[l].set_encoder(dev["q_g"], dev["WaQ"], dev["WaK"], dev["WaV"], dev["k_g"], dev["v_g"])
    st.reset()
    return st


@pytest.mark.parametrize("kind", ["mfma", "mfma_inline", "f32"])
def test_stack_steps_and_graph_replays_match_per_layer_oracles(kind):
    L = 3
    inline = kind == "mfma_inline"
    if inline:
        kind = "mfma"
    if kind == "mfma":
        wl = I.WORKLOADS["qwen7b"].replace(batch=3, n_q_heads=14, n_kv_heads=2, window=96, chunk=32, steps=150)
    else:
        wl = I.WORKLOADS["tiny_f32"].replace(batch=3, window=24, chunk=8, steps=60)
    wls = _layer_workloads(wl, L)
    encs = [I.encoder_params(w) for w in wls]
    orcs = [H.make_oracle(w, e) for w, e in zip(wls, encs)]
    st = _make_stack(wl, L, encs)
    assert [layer.plan()[0] for layer in st.layers] == [1 if kind == "mfma" else 0] * L
    if kind == "mfma":
        # two encoding workgroups per rollout: their shares of S' meet in the scratch buffer the layers share
        for layer in st.layers:
            if inline:
                # ... or the rollouts' own workgroups fold their next chunk ahead of time: the pending block and its
                # group count are updated in place by replays and eager steps alike
                layer.set_option(ptenc.OPT_ENCODE_INLINE, 1)
            else:
                layer.set_option(ptenc.OPT_ENCODE_PARTS, 2)
    T = wl.steps
    qkv = [I.qkv_steps(w, 0, T) for w in wls]
    dev = [tuple(x.cuda() for x in t) for t in qkv]
    host = [tuple(H.f64(x) for x in t) for t in qkv]
    abs_tol, rel_tol = H.tolerances(wl)
    # static buffers of the recorded step
    qs = [torch.empty_like(d[0][0]) for d in dev]
    ks = [torch.empty_like(d[1][0]) for d in dev]
    vs = [torch.empty_like(d[2][0]) for d in dev]
    outs = [torch.empty_like(d[0][0]) for d in dev]
    with pytest.raises(ptenc.PtencError) as ei:
        st.graph_launch()                                    # nothing recorded yet
    assert ei.value.status == ptenc.ERR_STATE
    st.graph_capture(qs, ks, vs, outs)
    for t in range(T):
        refs = [orcs[l].step(host[l][0][t], host[l][1][t], host[l][2][t], None) for l in range(L)]
        if t % 3 == 0:                                       # eager launches and replays interleave freely
            got = st.step([d[0][t] for d in dev], [d[1][t] for d in dev], [d[2][t] for d in dev])
        else:
            for l in range(L):
                qs[l].copy_(dev[l][0][t]); ks[l].copy_(dev[l][1][t]); vs[l].copy_(dev[l][2][t])
            st.graph_launch()
            got = outs
            if t % 7 == 0:
                torch.cuda.synchronize()
                _ = (dev[0][0][t].float() * 2).sum().item()  # unrelated eager work between replays
        for l in range(L):
            H.assert_close(H.f64(got[l]), refs[l], abs_tol, rel_tol, "layer %d out at step %d" % (l, t))
    for l in range(L):
        ln, base = st.layers[l].counters()
        oln, obase = orcs[l].counters()
        assert np.array_equal(ln, oln) and np.array_equal(base, obase)
        H.assert_close(st.layers[l].get_state(), orcs[l].state(), H.S_ABS, H.S_REL, "layer %d state" % l)
        assert st.layers[l].poll_error() == 0
    # the layers really are distinct contexts: their states differ
    assert not np.array_equal(st.layers[0].get_state(), st.layers[1].get_state())


def test_stack_equals_separate_layers_bitwise():
    # same kernels, same plan: a stack's outputs are those of L stand-alone contexts, bit for bit
    L = 2
    wl = I.WORKLOADS["qwen7b"].replace(batch=4, n_q_heads=14, n_kv_heads=2, window=128, chunk=48, steps=200)
    wls = _layer_workloads(wl, L)
    encs = [I.encoder_params(w) for w in wls]
    st = _make_stack(wl, L, encs)
    singles = [H.make_layer(w, e) for w, e in zip(wls, encs)]
    dev = [tuple(x.cuda() for x in I.qkv_steps(w, 0, wl.steps)) for w in wls]
    for t in range(wl.steps):
        got = st.step([d[0][t] for d in dev], [d[1][t] for d in dev], [d[2][t] for d in dev])
        for l in range(L):
            ref = singles[l].step(dev[l][0][t], dev[l][1][t], dev[l][2][t])
            assert torch.equal(got[l], ref), "layer %d step %d" % (l, t)
    for l in range(L):
        assert np.array_equal(st.layers[l].get_state(), singles[l].get_state())
        K0, V0 = st.layers[l].gather_window()
        K1, V1 = singles[l].gather_window()
        ln, base = singles[l].counters()
        n = int(ln[0] - base[0])
        assert torch.equal(K0[:, :, :n], K1[:, :, :n]) and torch.equal(V0[:, :, :n], V1[:, :, :n])


def test_stack_layers_under_the_scored_policy():
    # every layer of a stack is an ordinary context: the importance-based policy is set per layer, and
    # the recorded graph replays its steps (selection included) like eager launches
    from oracle import scored_oracle as so
    L, n_recent = 2, 24
    wl = I.WORKLOADS["qwen7b"].replace(batch=3, n_q_heads=14, n_kv_heads=2, window=96, chunk=32, steps=200)
    wls = _layer_workloads(wl, L)
    encs = [I.encoder_params(w) for w in wls]
    orcs = []
    for w, enc in zip(wls, encs):
        e = {k: H.f64(v) for k, v in enc.items()}
        orcs.append(so.ScoredOracleLayer(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.window, w.chunk, n_recent,
                                         e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"]))
    st = ptenc.Stack(L, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                     dtype=wl.torch_dtype, poison_cache=True)
    for l, enc in enumerate(encs):
        st.layers[l].set_option(ptenc.OPT_RECENT, n_recent)
        st.layers[l].set_option(ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED)
        dev = {k: v.cuda() for k, v in enc.items()}
        st.layers[l].set_encoder(dev["q_g"], dev["WaQ"], dev["WaK"], dev["WaV"], dev["k_g"], dev["v_g"])
    st.reset()
    qkv = []
    for w in wls:
        q, k, v = I.qkv_steps(w, 0, wl.steps)
        qkv.append(((q.float() * 48.0).to(q.dtype), k, v))
    dev = [tuple(x.cuda() for x in t) for t in qkv]
    host = [tuple(H.f64(x) for x in t) for t in qkv]
    qs = [torch.empty_like(d[0][0]) for d in dev]
    ks = [torch.empty_like(d[1][0]) for d in dev]
    vs = [torch.empty_like(d[2][0]) for d in dev]
    outs = [torch.empty_like(d[0][0]) for d in dev]
    st.graph_capture(qs, ks, vs, outs)
    for t in range(wl.steps):
        refs = [orcs[l].step(host[l][0][t], host[l][1][t], host[l][2][t]) for l in range(L)]
        if t % 2 == 0:
            got = st.step([d[0][t] for d in dev], [d[1][t] for d in dev], [d[2][t] for d in dev])
        else:
            for l in range(L):
                qs[l].copy_(dev[l][0][t]); ks[l].copy_(dev[l][1][t]); vs[l].copy_(dev[l][2][t])
            st.graph_launch()
            got = outs
        for l in range(L):
            H.assert_close(H.f64(got[l]), refs[l], H.BF16_ABS, H.BF16_REL, "layer %d out at step %d" % (l, t))
    for l in range(L):
        assert orcs[l].min_margin >= 1e-2, "inputs leave a selection too close to call: pick others"
        assert all(np.array_equal(a, b) for a, b in zip(st.layers[l].counters(), orcs[l].counters()))
        vic = st.layers[l].victims()
        for b in range(wl.batch):
            assert vic[b].tolist() == orcs[l].last_victims[b]
        H.assert_close(st.layers[l].get_state(), orcs[l].state(), H.S_ABS, H.S_REL, "layer %d state" % l)


def test_a_layer_stepped_on_its_own_is_noticed_by_the_recorded_step():
    # the recorded step exists once for either role assignment of the layers' two counter buffers; a
    # layer that is stepped alone leaves the assignment the others have, and the stack says so
    L = 2
    wl = I.WORKLOADS["qwen7b"].replace(batch=2, n_q_heads=14, n_kv_heads=2, window=64, chunk=16, steps=8)
    wls = _layer_workloads(wl, L)
    st = _make_stack(wl, L, [I.encoder_params(w) for w in wls])
    dev = [tuple(x.cuda() for x in I.qkv_steps(w, 0, 4)) for w in wls]
    qs, ks, vs = ([d[i][0].clone() for d in dev] for i in range(3))
    outs = [torch.empty_like(x) for x in qs]
    st.graph_capture(qs, ks, vs, outs)
    st.graph_launch()
    st.graph_launch()
    st.step([d[0][1] for d in dev], [d[1][1] for d in dev], [d[2][1] for d in dev])
    st.graph_launch()                                        # any mix of replays and eager steps is fine
    st.layers[1].step(dev[1][0][2], dev[1][1][2], dev[1][2][2])
    with pytest.raises(ptenc.PtencError) as ei:
        st.graph_launch()
    assert ei.value.status == ptenc.ERR_STATE
    st.layers[0].step(dev[0][0][2], dev[0][1][2], dev[0][2][2])   # the other layer catches up
    st.graph_launch()
    torch.cuda.synchronize()
    for layer in st.layers:
        ln, base = layer.counters()
        assert (ln == 6).all() and (base == 0).all()
        assert layer.poll_error() == 0
