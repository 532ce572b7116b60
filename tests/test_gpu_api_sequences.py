"""Seeded random sequences of valid API calls against the oracle: fused steps (full batch, masked,
compact id lists in random order), the three separate entry points, attention without a step, finished
rollouts recycled (masked reset + new question tokens), and options changed in mid-run (window
splits, workgroup size, encoding workgroups per chunk, counters in place or alternating).  Every
call's outputs and the counters are compared at once, S and the cache contents at the end."""
import numpy as np
import pytest
import torch

from paper_2602_16839_amd import inputs as I
from paper_2602_16839_amd import ptenc
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _workload(rng, kind):
    if kind == "mfma":
        n_sink = int(rng.choice([0, 32]))
        ring = 32 * int(rng.integers(1, 5))
        wl = I.WORKLOADS["qwen7b"].replace(batch=5, n_q_heads=8, n_kv_heads=2, window=n_sink + ring, n_sink=n_sink,
                                           chunk=int(rng.integers(1, ring + 1)), steps=0)
    else:
        n_sink = int(rng.choice([0, 7]))
        ring = int(rng.integers(4, 40))
        wl = I.WORKLOADS["tiny_f32"].replace(batch=5, window=n_sink + ring, n_sink=n_sink,
                                             chunk=int(rng.integers(1, ring + 1)), steps=0)
    ticks = 3 * ring + 40
    return wl.replace(steps=ticks, seed=int(rng.integers(1, 1 << 20)))


@pytest.mark.parametrize("kind,seed", [(k, s) for k in ("mfma", "f32") for s in range(12)])
def test_random_call_sequence(kind, seed):
    rng = np.random.default_rng(31337 * (1 + ("mfma", "f32").index(kind)) + seed)
    wl = _workload(rng, kind)
    B, T = wl.batch, wl.steps
    enc = I.encoder_params(wl)
    orc = H.make_oracle(wl, enc)
    layer = H.make_layer(wl, enc)
    pl = None
    if wl.n_sink:
        pl = H.prefill_both(wl, orc, layer, rng.integers(0, wl.n_sink + 1, B))
    pk2, pv2 = I.prompt_kv(wl.replace(seed=wl.seed + 1)) if wl.n_sink else (None, None)
    q, k, v = I.qkv_steps(wl, 0, T)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    abs_tol, rel_tol = H.tolerances(wl)
    log = []

    def dev_mask(act):
        return torch.from_numpy(act.astype(np.uint8)).cuda()

    def check(out, ref, rows, what):
        if len(rows):
            H.assert_close(H.f64(out), ref, abs_tol, rel_tol, "%s; calls so far: %s" % (what, log[-12:]))

    for t in range(T):
        op = str(rng.choice(["step", "step", "masked", "ids", "trio", "attend", "recycle", "option"]))
        act = rng.random(B) < rng.choice([0.3, 0.7, 1.0])
        log.append((t, op))
        if op == "step":
            ref = orc.step(qn[t], kn[t], vn[t])
            check(layer.step(qd[t], kd[t], vd[t]), ref, range(B), "step %d" % t)
        elif op == "masked":
            ref = orc.step(qn[t], kn[t], vn[t], act)
            check(layer.step(qd[t], kd[t], vd[t], active=dev_mask(act)), ref, range(B), "masked step %d" % t)
        elif op == "ids":
            idx = rng.permutation(np.nonzero(act)[0])
            m = np.zeros(B, dtype=bool)
            m[idx] = True
            ref = orc.step(qn[t], kn[t], vn[t], m)
            it = torch.from_numpy(idx)
            out = layer.step_ids(qd[t][it.cuda()].contiguous(), kd[t][it.cuda()].contiguous(),
                                 vd[t][it.cuda()].contiguous(), it.to(torch.int32).cuda())
            check(out, ref[idx], idx, "compact step %d" % t)
        elif op == "trio":
            ref = np.zeros((B, wl.n_q_heads, wl.head_dim))
            for b in np.nonzero(act)[0]:
                orc.evict_encode(b)
                orc.append(b, kn[t][b], vn[t][b])
                ref[b] = orc.attend(b, qn[t][b])
            am = dev_mask(act)
            layer.evict_encode(am)
            layer.append(kd[t], vd[t], am)
            check(layer.attend(qd[t], active=am), ref, range(B), "separate calls at tick %d" % t)
        elif op == "attend":
            # attention alone changes nothing; rollouts with nothing to attend over sit it out
            ln, base = orc.counters()
            have = act & ((ln - base + orc.prompt_lengths()) > 0)
            ref = np.zeros((B, wl.n_q_heads, wl.head_dim))
            for b in np.nonzero(have)[0]:
                ref[b] = orc.attend(b, qn[t][b])
            check(layer.attend(qd[t], active=dev_mask(have)), ref, range(B), "attention alone at tick %d" % t)
        elif op == "recycle":
            ids = [int(b) for b in np.nonzero(rng.random(B) < 0.3)[0]]
            if not ids:
                continue
            mask = np.zeros(B, dtype=bool)
            mask[ids] = True
            layer.reset(dev_mask(mask))
            for b in ids:
                orc.reset_rollout(b)
            if wl.n_sink:
                lens = [int(x) for x in rng.integers(0, wl.n_sink + 1, len(ids))]
                layer.prefill_ids(pk2[ids].cuda().contiguous(), pv2[ids].cuda().contiguous(),
                                  torch.tensor(ids, dtype=torch.int32, device="cuda"), lens)
                for b, n in zip(ids, lens):
                    orc.prefill(b, H.f64(pk2[b, :n]), H.f64(pv2[b, :n]))
                    pl[b] = n
                assert np.array_equal(layer.prompt_len(), pl)
        else:
            which = str(rng.choice(["splits", "waves", "parts", "in_place"]))
            log[-1] = (t, which)
            if which == "splits":
                layer.set_option(ptenc.OPT_SPLITS, int(rng.choice([0, 1, 2, 3])))
            elif which == "waves" and kind == "mfma":
                layer.set_option(ptenc.OPT_WAVES, int(rng.choice([0, 4, 8])))
            elif which == "parts":
                layer.set_option(ptenc.OPT_ENCODE_PARTS, int(rng.choice([0, 1, 2, 5])))
            elif which == "in_place":
                layer.set_option(ptenc.OPT_COUNTERS_IN_PLACE, int(rng.integers(0, 2)))
        ln, base = layer.counters()
        oln, obase = orc.counters()
        assert np.array_equal(ln, oln) and np.array_equal(base, obase), "counters after tick %d; calls: %s" % (t, log[-12:])
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")
    Kw, Vw = layer.gather_window()
    for b in range(B):
        ko, vo = orc.window_kv(b)
        if len(ko):
            assert torch.equal(Kw[b, :, :len(ko)].cpu().to(torch.float64), torch.from_numpy(ko).transpose(0, 1)), b
            assert torch.equal(Vw[b, :, :len(vo)].cpu().to(torch.float64), torch.from_numpy(vo).transpose(0, 1)), b
    assert layer.poll_error() == 0
