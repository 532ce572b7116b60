"""Seeded random small configurations through the whole decode path against the oracle: shapes, window
/ chunk / reserved-slot sizes, window splits, workgroup sizes, encoding workgroups per chunk, masks and
compact id lists are drawn together, so that combinations nobody wrote a dedicated test for get
exercised too."""
import numpy as np
import pytest
import torch

from paper_2602_16839_amd import inputs as I
from paper_2602_16839_amd import ptenc
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _draw(rng, kind):
    if kind == "mfma":
        n_kv = int(rng.choice([1, 2, 3]))
        group = int(rng.choice([1, 2, 4, 7, 8, 16]))
        n_sink = int(rng.choice([0, 0, 32, 64]))
        ring = 32 * int(rng.integers(1, 6))
        W = n_sink + ring
        base = "qwen7b"
        d = 128
    else:
        n_kv = int(rng.choice([1, 2]))
        group = int(rng.choice([1, 2, 3]))
        n_sink = int(rng.choice([0, 0, 5, 16]))
        ring = int(rng.integers(3, 70))
        W = n_sink + ring
        base = "tiny_f32" if kind == "f32" else "qwen3b"
        d = int(rng.choice([16, 64, 96]))
    C = int(rng.integers(1, ring + 1))
    B = int(rng.integers(1, 6))
    T = ring + int(rng.integers(1, 3 * C + 20))
    wl = I.WORKLOADS[base].replace(batch=B, n_q_heads=n_kv * group, n_kv_heads=n_kv, head_dim=d, window=W, chunk=C,
                                   n_sink=n_sink, steps=T, n_global=int(rng.choice([4, 32])), rank=int(rng.choice([8, 32])),
                                   seed=int(rng.integers(1, 1 << 20)))
    splits = int(rng.choice([0, 1, 2, 3, 5]))
    waves = int(rng.choice([0, 4, 8])) if kind == "mfma" and group <= 8 else 0
    mode = str(rng.choice(["full", "masked", "ids"]))
    return wl, splits, waves, mode


@pytest.mark.parametrize("kind,seed", [(k, s) for k in ("mfma", "f32", "generic_bf16") for s in range(20)])
def test_random_configuration(kind, seed):
    rng = np.random.default_rng(1000 * ("mfma", "f32", "generic_bf16").index(kind) + seed)
    wl, splits, waves, mode = _draw(rng, kind)
    enc = I.encoder_params(wl)
    orc = H.make_oracle(wl, enc)
    # (a generator of its own, so that the cases drawn before this option existed stay what they were)
    parts = int(np.random.default_rng(5000 + seed).choice([0, 1, 2, 3, 5, 8])) if kind == "mfma" else 0
    # who encodes evicted chunks (again a generator of its own): the launch's own choice, encoding workgroups,
    # or the rollouts' own workgroups ahead of time
    inline = int(np.random.default_rng(7000 + seed).choice([-1, 0, 1, 1])) if kind == "mfma" else -1
    layer = H.make_layer(wl, enc, splits=splits, waves=waves, enc_parts=parts, enc_inline=inline)
    assert layer.plan()[0] == (1 if kind == "mfma" else 0), (kind, wl)
    prompt_len = None
    if wl.n_sink:
        prompt_len = rng.integers(0, wl.n_sink + 1, wl.batch)
        H.prefill_both(wl, orc, layer, prompt_len)
    T = wl.steps
    lengths = np.full(wl.batch, T) if mode == "full" else rng.integers(1, T + 1, wl.batch)
    lengths[int(rng.integers(0, wl.batch))] = T
    q, k, v = I.qkv_steps(wl, 0, T)
    if kind == "mfma" and seed % 2:
        q = (q.float() * 32.0).to(q.dtype)          # peaked attention: the online rescale gets work
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    abs_tol, rel_tol = H.tolerances(wl)
    what = "%s seed %d: %s splits %d waves %d parts %d %s" % (kind, seed, wl, splits, waves, parts, mode)
    for t in range(T):
        act = I.active_mask(lengths, t)
        ref = orc.step(qn[t], kn[t], vn[t], None if mode == "full" else act)
        if mode == "ids":
            ids = np.nonzero(act)[0].astype(np.int32)
            idt = torch.from_numpy(ids).cuda()
            out = layer.step_ids(qd[t][idt.long()].contiguous(), kd[t][idt.long()].contiguous(),
                                 vd[t][idt.long()].contiguous(), idt)
            H.assert_close(H.f64(out), ref[ids], abs_tol, rel_tol, what + " out at step %d" % t)
        else:
            out = layer.step(qd[t], kd[t], vd[t], active=None if mode == "full" else torch.from_numpy(act).cuda())
            H.assert_close(H.f64(out), ref, abs_tol, rel_tol, what + " out at step %d" % t)
    ln, base = layer.counters()
    oln, obase = orc.counters()
    assert np.array_equal(ln, oln) and np.array_equal(base, obase), what
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, what + " state")
    Kw, Vw = layer.gather_window()
    for b in range(wl.batch):
        ko, vo = orc.window_kv(b)
        n = len(ko)
        assert torch.equal(Kw[b, :, :n].cpu().to(torch.float64), torch.from_numpy(ko).transpose(0, 1)), what + " window K"
        assert torch.equal(Vw[b, :, :n].cpu().to(torch.float64), torch.from_numpy(vo).transpose(0, 1)), what + " window V"
    assert layer.poll_error() == 0, what
