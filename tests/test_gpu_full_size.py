"""Parity at the benchmark's full sizes, in the launch configuration bench.py times
(ptenc_decode_run over step-major buffers, default plan): the whole run is decoded on the GPU
and sampled outputs, ring contents and states are recomputed one by one by the CPU oracle from
the stateless input generator.  Counters are checked in full against the closed forms."""
import numpy as np
import pytest
import torch

from oracle import pte_oracle as po
from oracle.ring_model import evicted_closed_form
from paper_2602_16839_amd import inputs as I
from paper_2602_16839_amd import ptenc
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _run_full(wl, sample_steps, seg_steps, options=None):
    """Decode the whole workload in segments; returns (layer, lengths, {t: out[t-1] on the host})."""
    dev = torch.device("cuda:0")
    enc = I.encoder_params(wl, device=dev)
    layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                        dtype=wl.torch_dtype, n_global=wl.n_global, rank=wl.rank, poison_cache=True, n_sink=wl.n_sink)
    for opt, val in (options or {}).items():
        layer.set_option(opt, val)
    layer.set_encoder(enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    layer.reset()
    if wl.n_sink:
        pk, pv = I.prompt_kv(wl, device=dev)
        layer.prefill(pk, pv, I.prompt_lengths(wl))
    lengths = I.rollout_lengths(wl)
    T = int(lengths.max())
    len_dev = torch.from_numpy(lengths).to(dev).view(1, -1)
    kept = {}
    for t0 in range(0, T, seg_steps):
        t1 = min(T, t0 + seg_steps)
        q, k, v = I.qkv_steps(wl, t0, t1, device=dev)
        active = None
        if wl.ragged:
            tt = torch.arange(t0, t1, device=dev).view(-1, 1)
            active = (tt < len_dev).to(torch.uint8).contiguous()
        out = layer.run(q, k, v, active=active)
        for t in sample_steps:
            if t0 < t <= t1:
                kept[t] = out[t - 1 - t0].cpu()
        del q, k, v, out
    torch.cuda.synchronize()
    return layer, lengths, kept, T


def _oracle_window(wl, b, t, L):
    """(queries, keys, values) rollout b attends with at decode step t (1-based), from regenerated inputs."""
    E = evicted_closed_form(t, wl.window - wl.n_sink, wl.chunk)
    q, k, v = I.qkv_steps(wl, E, t, b0=b, b1=b + 1)
    keys, values = list(H.f64(k[:, 0])), list(H.f64(v[:, 0]))
    if wl.n_sink:                                   # question tokens come first and never leave
        P = int(I.prompt_lengths(wl)[b])
        pk, pv = I.prompt_kv(wl)
        keys, values = list(H.f64(pk[b, :P])) + keys, list(H.f64(pv[b, :P])) + values
    return H.f64(q[-1, 0]), keys, values


def _oracle_out(wl, b, t, L):
    """Attention output of rollout b at decode step t (1-based)."""
    if t > L:
        return np.zeros((wl.n_q_heads, wl.head_dim))
    q, keys, values = _oracle_window(wl, b, t, L)
    return po.attend(q, keys, values)


def _strawmen_fail(wl, b, t, L, ref, what):
    """The comparison at (b, t) must have the power to reject wrong softmax weights: the plain mean of the
    live values (uniform weights, queries ignored) and a softmax that forgot the 1/sqrt(d) scale have to
    miss BOTH contract bars by a factor of ten.  Computed on the CPU from the oracle's own inputs."""
    q, keys, values = _oracle_window(wl, b, t, L)
    V = np.stack(values)                                                  # [n, H_kv, d]
    g = wl.n_q_heads // wl.n_kv_heads
    mean_v = np.repeat(V.mean(axis=0), g, axis=0)                         # [H_q, d]
    unscaled = po.attend(q, keys, values, scale=1.0)
    for name, wrong in (("mean of V", mean_v), ("softmax without 1/sqrt(d)", unscaled)):
        a, r = H.row_errors(wrong, ref)
        assert a >= 10 * H.BF16_ABS and r >= 10 * H.BF16_REL, (
            "%s: the strawman '%s' is only %.2e abs / %.2e row-rel away from the oracle: this case cannot tell it "
            "from the attention equation" % (what, name, a, r))


def _oracle_state(wl, b, L, enc):
    """S of rollout b after L decode steps: every eviction replayed from regenerated inputs."""
    e = {k: H.f64(v) for k, v in enc.items()}
    Q_a, S = po.init_state(e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"])
    E = evicted_closed_form(L, wl.window - wl.n_sink, wl.chunk)
    if E:
        _, k, v = I.qkv_steps(wl, 0, E, b0=b, b1=b + 1)
        k, v = H.f64(k[:, 0]).reshape(E, -1), H.f64(v[:, 0]).reshape(E, -1)
        for c0 in range(0, E, wl.chunk):
            S = po.normalize(S + po.encode_chunk(Q_a, k[c0:c0 + wl.chunk], v[c0:c0 + wl.chunk], e["WaK"], e["WaV"]))
    return S


def _check(wl, sample_b, sample_t, seg_steps, peaked=False, options=None):
    layer, lengths, kept, T = _run_full(wl, sample_t, seg_steps, options)
    assert layer.poll_error() == 0
    # counters, all rollouts, against the closed forms
    ln, base = layer.counters()
    assert np.array_equal(ln, lengths)
    assert np.array_equal(base, np.array([evicted_closed_form(int(L), wl.window - wl.n_sink, wl.chunk) for L in lengths]))
    # sampled outputs
    for t in sample_t:
        got = H.f64(kept[t])
        for b in sample_b:
            ref = _oracle_out(wl, b, t, int(lengths[b]))
            H.assert_close(got[b], ref, H.BF16_ABS, H.BF16_REL, "%s out b=%d t=%d" % (wl.name, b, t))
            if peaked and t > 64:
                _strawmen_fail(wl, b, t, int(lengths[b]), ref, "%s b=%d t=%d" % (wl.name, b, t))
    # sampled ring contents (bit exact) and states
    Kw, Vw = layer.gather_window()
    S = layer.get_state()
    enc = I.encoder_params(wl)
    for b in sample_b:
        L = int(lengths[b])
        E, n = int(base[b]), int(ln[b] - base[b])
        P = int(I.prompt_lengths(wl)[b])
        _, k, v = I.qkv_steps(wl, E, L, b0=b, b1=b + 1)
        assert torch.equal(Kw[b, :, P:P + n].cpu(), k[:, 0].transpose(0, 1)), "ring K of rollout %d" % b
        assert torch.equal(Vw[b, :, P:P + n].cpu(), v[:, 0].transpose(0, 1)), "ring V of rollout %d" % b
        H.assert_close(S[b], _oracle_state(wl, b, L, enc), H.S_ABS, H.S_REL, "%s S b=%d" % (wl.name, b))
    return layer


def test_qwen3b_full_run_sampled():
    wl = I.WORKLOADS["qwen3b"]
    W, C, T = wl.window, wl.chunk, wl.steps
    layer = _check(wl, [0, 37, 63], [1, 33, W, W + 1, W + C // 2, T - 1, T], seg_steps=1024)
    assert layer.plan()[0] == 1


def test_qwen7b_full_run_sampled():
    # the configuration the benchmark is quoted on
    wl = I.WORKLOADS["qwen7b"]
    W, C, T = wl.window, wl.chunk, wl.steps
    layer = _check(wl, [0, 77, 127], [1, 31, 1000, W, W + 1, W + C, 6001, T], seg_steps=1024)
    assert layer.plan() == (1, 1, 1)


def test_qwen7b_with_question_tokens_full_run_sampled():
    # 512 reserved slots (ragged question lengths 128..512) in front of the same 4096-token window
    wl = I.WORKLOADS["qwen7b_sink"]
    R, C, T = wl.window - wl.n_sink, wl.chunk, wl.steps
    pl = I.prompt_lengths(wl)
    assert pl.min() >= 128 and pl.max() <= 512 and len(set(pl.tolist())) > 32
    _check(wl, [0, 64, 127], [1, R, R + 1, T], seg_steps=1024)


def test_qwen7b_quarter_window_chunks_full_run_sampled():
    # the paper's own eviction ratio (a quarter of the window leaves on saturation), with a chunk
    # that is not a whole number of 32-slot groups
    wl = I.WORKLOADS["qwen7b"].replace(chunk=1000)
    W, C, T = wl.window, wl.chunk, wl.steps
    _check(wl, [5, 126], [W, W + 1, W + C + 1, T], seg_steps=1024)


def test_llama8b_full_run_sampled():
    wl = I.WORKLOADS["llama8b"]
    W, C, T = wl.window, wl.chunk, wl.steps
    _check(wl, [3, 255], [W, W + 1, T], seg_steps=512)


# The benchmark's input scale leaves the softmax weights uniform to within a per cent, so the cases above check
# which keys are live and the value sum, but could not tell the attention equation from a plain mean of V.
# The peaked twins (values of std 0.25, queries 64 times larger: scores about N(0, 4^2)) run the same shapes,
# plans and kernels -- the non-temporal instantiation, the walk that requests two groups ahead of the counters,
# the 8-wavefront workgroups of the 3B shape -- with a few keys carrying the attention and the running maximum
# moving throughout the walk; each sampled comparison also proves its own power (_strawmen_fail).
def test_qwen7b_peaked_full_run_sampled():
    wl = I.WORKLOADS["qwen7b_peaked"]
    W, C, T = wl.window, wl.chunk, wl.steps
    layer = _check(wl, [0, 77, 127], [W, W + 1, W + C, T], seg_steps=1024, peaked=True)
    assert layer.plan() == (1, 1, 1)


def test_llama8b_peaked_full_run_sampled():
    wl = I.WORKLOADS["llama8b_peaked"]
    W, C, T = wl.window, wl.chunk, wl.steps
    _check(wl, [3, 255], [W, W + 1, W + C, T], seg_steps=512, peaked=True)


def test_qwen3b_peaked_full_run_sampled():
    # one workgroup per CU at most: the plan takes 8 wavefronts per workgroup here
    wl = I.WORKLOADS["qwen3b_peaked"]
    W, C, T = wl.window, wl.chunk, wl.steps
    layer = _check(wl, [0, 37, 63], [33, W, W + 1, W + C, T], seg_steps=1024, peaked=True)
    assert layer.plan()[0] == 1


@pytest.mark.parametrize("waves,splits", [(4, 1), (8, 3)])
def test_forced_nontemporal_variant_peaked(waves, splits):
    # The kernel instantiation with non-temporal loads is otherwise chosen only for caches beyond the
    # memory-side cache; forced here on a cache of a few MB, with peaked attention.  4 wavefronts and one
    # split over 64 groups is also the walk that requests two groups ahead of the counters.
    wl = I.WORKLOADS["qwen7b_peaked"].replace(name="nt_peaked", batch=3, n_q_heads=16, n_kv_heads=2, window=2048,
                                              chunk=100, steps=2048 + 2 * 100 + 17)
    W, C, T = wl.window, wl.chunk, wl.steps
    layer = _check(wl, [0, 1, 2], [33, 1000, W, W + 1, W + C + 1, T], seg_steps=1024, peaked=True,
                   options={ptenc.OPT_NONTEMPORAL: 1, ptenc.OPT_WAVES: waves, ptenc.OPT_SPLITS: splits})
    assert layer.plan()[:2] == (1, splits)


def test_ragged_full_run_sampled():
    wl = I.WORKLOADS["ragged"]
    lengths = I.rollout_lengths(wl)
    order = np.argsort(lengths)
    b_short, b_med, b_long = int(order[0]), int(order[len(order) // 2]), int(order[-1])
    never_full = [int(b) for b in np.where(lengths < wl.window)[0][:1]]
    sample_b = sorted(set([b_short, b_med, b_long] + never_full))
    Lm = int(lengths[b_med])
    sample_t = sorted(set([1, int(lengths[b_short]), wl.window + 1, Lm, Lm + 1, int(lengths[b_long])]))
    _check(wl, sample_b, sample_t, seg_steps=1024)


def test_qwen7b_rollouts_that_start_at_different_steps_full_size():
    # a running batch: rollout b joins at step start_b, so the rollouts' evictions fall in different steps
    # (every step of the steady state has an evicting rollout whose chunk is encoded beside everybody's
    # attention).  Masked full-batch steps at the benchmark's shape; sampled outputs, rings, states.
    wl = I.WORKLOADS["qwen7b"]
    B, W, C = wl.batch, wl.window, wl.chunk
    T = W + 3 * C + 57
    starts = (np.arange(B) * C) // B + (np.arange(B) % 3)             # 0 .. C + 1, spread
    dev = torch.device("cuda:0")
    enc = I.encoder_params(wl, device=dev)
    layer = ptenc.Layer(B, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, W, C, dtype=wl.torch_dtype,
                        n_global=wl.n_global, rank=wl.rank, poison_cache=True)
    layer.set_encoder(enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    layer.reset()
    sample_t = [1, 60, W, W + 1, W + C, W + 2 * C + 31, T]
    start_dev = torch.from_numpy(starts).to(dev).view(1, -1)
    kept = {}
    for t0 in range(0, T, 1024):
        t1 = min(T, t0 + 1024)
        q, k, v = I.qkv_steps(wl, t0, t1, device=dev)
        tt = torch.arange(t0, t1, device=dev).view(-1, 1)
        active = (tt >= start_dev).to(torch.uint8).contiguous()
        out = layer.run(q, k, v, active=active)
        for t in sample_t:
            if t0 < t <= t1:
                kept[t] = out[t - 1 - t0].cpu()
        del q, k, v, out
    assert layer.poll_error() == 0
    ln, base = layer.counters()
    Wr = W
    assert np.array_equal(ln, T - starts)
    assert np.array_equal(base, np.array([evicted_closed_form(int(T - s), Wr, C) for s in starts]))
    assert len(set(base.tolist())) > 1                                 # they did not evict in step
    e64 = {kk: H.f64(vv) for kk, vv in I.encoder_params(wl).items()}
    Kw, Vw = layer.gather_window()
    S = layer.get_state()
    for b in (0, 41, 127):
        s = int(starts[b])
        for t in sample_t:
            tl = t - s                                                # the rollout's own step count
            if tl <= 0:
                assert not kept[t][b].any()
                continue
            E = evicted_closed_form(tl, Wr, C)
            q, k, v = I.qkv_steps(wl, s + E, t, b0=b, b1=b + 1)
            ref = po.attend(H.f64(q[-1, 0]), list(H.f64(k[:, 0])), list(H.f64(v[:, 0])))
            H.assert_close(H.f64(kept[t][b]), ref, H.BF16_ABS, H.BF16_REL, "out b=%d t=%d" % (b, t))
        E, n = int(base[b]), int(ln[b] - base[b])
        _, k, v = I.qkv_steps(wl, s + E, T, b0=b, b1=b + 1)
        assert torch.equal(Kw[b, :, :n].cpu(), k[:, 0].transpose(0, 1)) and torch.equal(Vw[b, :, :n].cpu(), v[:, 0].transpose(0, 1))
        Q_a, Sr = po.init_state(e64["q_g"], e64["WaQ"], e64["WaK"], e64["WaV"], e64["k_g"], e64["v_g"])
        if E:
            _, k, v = I.qkv_steps(wl, s, s + E, b0=b, b1=b + 1)
            k, v = H.f64(k[:, 0]).reshape(E, -1), H.f64(v[:, 0]).reshape(E, -1)
            for c0 in range(0, E, C):
                Sr = po.normalize(Sr + po.encode_chunk(Q_a, k[c0:c0 + C], v[c0:c0 + C], e64["WaK"], e64["WaV"]))
        H.assert_close(S[b], Sr, H.S_ABS, H.S_REL, "S b=%d" % b)
