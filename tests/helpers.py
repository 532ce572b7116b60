"""Shared plumbing for the GPU parity tests: build the oracle and the HIP layer from one workload
description, feed both the same seeded inputs, and compare with the stated tolerances."""
import numpy as np
import torch

from oracle import pte_oracle as po
from paper_2602_16839_amd import inputs as I

# bf16 inputs, fp32 accumulation, bf16 outputs: the bar the task states
BF16_ABS, BF16_REL = 1e-2, 2e-2
# fp32 end to end (different summation order and exp2 vs exp only)
F32_ABS, F32_REL = 2e-6, 2e-5
# the state S is fp32 on the device for either input type
S_ABS, S_REL = 1e-4, 1e-4


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def row_errors(got: np.ndarray, ref: np.ndarray):
    """(max abs error, max over rows of ||g - r||_inf / max(||r||_inf, 1e-30)); rows = last axis."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref)
    if diff.size == 0:
        return 0.0, 0.0
    row_err = diff.reshape(-1, ref.shape[-1]).max(axis=1)
    row_ref = np.abs(ref).reshape(-1, ref.shape[-1]).max(axis=1)
    return float(diff.max()), float((row_err / np.maximum(row_ref, 1e-30)).max())


# Errors observed on MI355X are far below the contract bars above (which stay the contract).  A regression
# guard of about four times the observed maximum, where one is on record for the case, catches a kernel
# that drifts towards the bar long before it crosses it.  Keys: the `what` prefix a full-size test uses.
# (max abs, max row-relative); measured values are listed in the design notes.
GUARDS = {
    # full-size cases (tests/test_gpu_full_size.py): observed maxima are listed in the design notes.  Output
    # errors are dominated by the bf16 rounding of the output itself (half an ulp = 2^-9 of the value) and of
    # the probabilities, so the observed row-relative error sits at 4-5e-3 whatever the shape: its guard is
    # 3 x that (4 x would be the contract bar); the absolute guards are 4 x the observed maxima.
    "qwen3b out": (1.0e-3, 1.5e-2), "qwen7b out": (1.1e-3, 1.5e-2), "llama8b out": (4.0e-5, 1.5e-2),
    "ragged out": (3.0e-4, 1.5e-2), "qwen7b_sink out": (3.0e-4, 1.5e-2),
    "qwen3b_peaked out": (8.0e-3, 1.5e-2), "qwen7b_peaked out": (8.0e-3, 1.5e-2),
    "llama8b_peaked out": (8.0e-3, 1.5e-2), "nt_peaked out": (8.0e-3, 1.5e-2),
    # the state: fp32 accumulation of exactly representable products, observed <= 1.1e-7 abs / 1.6e-6 row-rel
    "qwen3b S": (4e-7, 6e-6), "qwen7b S": (4e-7, 6e-6), "llama8b S": (4e-7, 6e-6), "ragged S": (4e-7, 6e-6),
    "qwen7b_sink S": (4e-7, 6e-6), "qwen3b_peaked S": (4e-7, 6e-6), "qwen7b_peaked S": (4e-7, 6e-6),
    "llama8b_peaked S": (4e-7, 6e-6), "nt_peaked S": (4e-7, 6e-6),
}

# every comparison made through assert_close, for the record of observed errors: {what: (abs, rel)} maxima
OBSERVED = {}


def _record(what, a, r):
    key = what.split(" b=")[0].split(" at step")[0]
    pa, pr = OBSERVED.get(key, (0.0, 0.0))
    OBSERVED[key] = (max(pa, a), max(pr, r))


def assert_close(got, ref, abs_tol, rel_tol, what="", guard=None):
    """The contract bars abs_tol / rel_tol must hold; `guard` = (abs, rel), or the GUARDS entry whose key
    starts `what`, is the tighter regression bar."""
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), "%s: non-finite output" % what
    a, r = row_errors(got, ref)
    _record(what, a, r)
    assert a <= abs_tol and r <= rel_tol, "%s: max abs %.3e (tol %.1e), max row-rel %.3e (tol %.1e)" % (
        what, a, abs_tol, r, rel_tol)
    if guard is None:
        for key, g in GUARDS.items():
            if what.startswith(key):
                guard = g
                break
    if guard is not None:
        assert a <= guard[0] and r <= guard[1], (
            "%s: within the contract but beyond the regression guard: max abs %.3e (guard %.1e), max row-rel %.3e "
            "(guard %.1e)" % (what, a, guard[0], r, guard[1]))


def tolerances(wl):
    return (F32_ABS, F32_REL) if wl.dtype == "f32" else (BF16_ABS, BF16_REL)


def make_oracle(wl, enc, norm_mode=po.NORM_FROBENIUS, keep_chunks=False, softmax_scale=None):
    e = {k: f64(v) for k, v in enc.items()}
    return po.OracleLayer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                          e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e.get("k_g"), e.get("v_g"),
                          norm_mode=norm_mode, keep_chunks=keep_chunks, softmax_scale=softmax_scale,
                          n_sink=wl.n_sink)


def make_layer(wl, enc, norm_mode=0, splits=0, force_generic=False, poison=True, softmax_scale=0.0, waves=0,
               enc_parts=0, enc_inline=-1):
    from paper_2602_16839_amd import ptenc
    layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                        dtype=wl.torch_dtype, n_global=wl.n_global, rank=wl.rank, norm_mode=norm_mode,
                        softmax_scale=softmax_scale, poison_cache=poison, n_sink=wl.n_sink)
    if force_generic:
        layer.set_option(ptenc.OPT_FORCE_GENERIC, 1)
    if splits:
        layer.set_option(ptenc.OPT_SPLITS, splits)
    if waves:
        layer.set_option(ptenc.OPT_WAVES, waves)
    if enc_parts:
        layer.set_option(ptenc.OPT_ENCODE_PARTS, enc_parts)
    if enc_inline >= 0:
        layer.set_option(ptenc.OPT_ENCODE_INLINE, enc_inline)
    dev = {k: v.to("cuda:0") for k, v in enc.items()}
    layer.set_encoder(dev["q_g"], dev["WaQ"], dev["WaK"], dev["WaV"], dev.get("k_g"), dev.get("v_g"))
    layer.reset()
    return layer


def prefill_both(wl, orc, layer, prompt_len=None):
    """Question tokens into both sides; returns the lengths used."""
    pl = I.prompt_lengths(wl) if prompt_len is None else np.asarray(prompt_len, dtype=np.int32)
    pk, pv = I.prompt_kv(wl)
    for b in range(wl.batch):
        orc.prefill(b, f64(pk[b, :pl[b]]), f64(pv[b, :pl[b]]))
    layer.prefill(pk.cuda(), pv.cuda(), pl)
    assert np.array_equal(layer.prompt_len(), pl)
    return pl


def run_both(wl, T, norm_mode=0, splits=0, force_generic=False, lengths=None, with_global_kv=True,
             q_gain=1.0, check_every=1, prompt_len=None, waves=0, enc_parts=0, enc_inline=-1):
    """Decode T steps on the oracle and on the HIP layer; compare outputs every `check_every` steps,
    counters every step, and the state at the end.  Returns (layer, oracle)."""
    enc = I.encoder_params(wl, with_global_kv=with_global_kv)
    orc = make_oracle(wl, enc, norm_mode=norm_mode)
    layer = make_layer(wl, enc, norm_mode=norm_mode, splits=splits, force_generic=force_generic, waves=waves,
                       enc_parts=enc_parts, enc_inline=enc_inline)
    if wl.n_sink:
        prefill_both(wl, orc, layer, prompt_len)
    q, k, v = I.qkv_steps(wl, 0, T)
    if q_gain != 1.0:
        q = (q.float() * q_gain).to(q.dtype)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    act_all = None
    if lengths is not None:
        act_all = np.stack([I.active_mask(lengths, t) for t in range(T)])
        act_dev = torch.from_numpy(act_all).cuda()
    abs_tol, rel_tol = tolerances(wl)
    qn, kn, vn = f64(q), f64(k), f64(v)
    for t in range(T):
        act = None if act_all is None else act_all[t]
        ref = orc.step(qn[t], kn[t], vn[t], act)
        out = layer.step(qd[t], kd[t], vd[t], active=None if act_all is None else act_dev[t])
        ln, base = layer.counters()
        oln, obase = orc.counters()
        assert np.array_equal(ln, oln) and np.array_equal(base, obase), "counters differ at step %d" % t
        if t % check_every == 0 or t == T - 1:
            assert_close(f64(out), ref, abs_tol, rel_tol, "out at step %d" % t)
    assert_close(layer.get_state(), orc.state(), S_ABS, S_REL, "state S")
    assert layer.poll_error() == 0
    return layer, orc
