"""Importance-based eviction on the GPU against the scored oracle.

The scores are floating point (compared with a tolerance); which tokens leave is an integer
decision taken on them.  Two kinds of test keep the two apart: selection on INJECTED scores (the
same float32 values on both sides, many ties) must agree bit for bit, and end-to-end runs use
inputs whose oracle-side margin between the last victim and the best survivor is far above the
score tolerance at every eviction (asserted), so both sides must pick the same tokens."""
import numpy as np
import pytest
import torch

from oracle import scored_oracle as so
from paper_2602_16839_amd import inputs as I
from paper_2602_16839_amd import ptenc
from tests import helpers as H

pytestmark = pytest.mark.gpu

SCORE_ABS, SCORE_REL = 1e-4, 1e-3      # fp32 exp2 / accumulation against fp64
MIN_MARGIN = 2e-2                      # relative gap the end-to-end inputs must keep at every selection


def small(**kw):
    base = dict(batch=3, n_q_heads=14, n_kv_heads=2, window=96, chunk=32, steps=200)
    base.update(kw)
    return I.WORKLOADS["qwen7b"].replace(**base)


def make_both(wl, n_recent, splits=0, waves=0):
    enc = I.encoder_params(wl)
    e = {k: H.f64(v) for k, v in enc.items()}
    orc = so.ScoredOracleLayer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk, n_recent,
                               e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"], n_sink=wl.n_sink)
    layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                        dtype=wl.torch_dtype, n_global=wl.n_global, rank=wl.rank, poison_cache=True, n_sink=wl.n_sink)
    layer.set_option(ptenc.OPT_RECENT, n_recent)
    layer.set_option(ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED)
    if splits:
        layer.set_option(ptenc.OPT_SPLITS, splits)
    if waves:
        layer.set_option(ptenc.OPT_WAVES, waves)
    dev = {k: v.cuda() for k, v in enc.items()}
    layer.set_encoder(dev["q_g"], dev["WaQ"], dev["WaK"], dev["WaV"], dev["k_g"], dev["v_g"])
    layer.reset()
    return orc, layer


def check_scores(wl, orc, layer, what):
    sc, ps = layer.scores()
    for b in range(wl.batch):
        n = len(orc.win[b])
        assert (ps[b, n:] == -1).all() and (sc[b, n:] == 0).all()
        got_p, got_s, ref_p, ref = ps[b, :n], sc[b, :n], orc.positions(b), orc.scores(b)
        if n == wl.window - wl.n_sink:
            # a full ring: the library has already brought the next victims to the front (the oracle does
            # it when they leave), so only the tokens and their scores are comparable, not the order
            og, orf = np.argsort(got_p), np.argsort(ref_p)
            got_p, got_s, ref_p, ref = got_p[og], got_s[og], ref_p[orf], ref[orf]
        assert np.array_equal(got_p, ref_p), "%s: ring positions of rollout %d" % (what, b)
        err = np.abs(got_s - ref)
        assert (err <= SCORE_ABS + SCORE_REL * np.abs(ref)).all(), "%s: scores of rollout %d off by %.3e" % (what, b, err.max())


def run_both(wl, T, n_recent, q_gain, splits=0, lengths=None, prompt_len=None, score_every=17, waves=0):
    orc, layer = make_both(wl, n_recent, splits, waves)
    if wl.n_sink:
        pl = np.asarray(prompt_len, dtype=np.int32)
        pk, pv = I.prompt_kv(wl)
        for b in range(wl.batch):
            orc.prefill(b, H.f64(pk[b, :pl[b]]), H.f64(pv[b, :pl[b]]))
        layer.prefill(pk.cuda(), pv.cuda(), pl)
    q, k, v = I.qkv_steps(wl, 0, T)
    q = (q.float() * q_gain).to(q.dtype)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    n_evictions = 0
    for t in range(T):
        act = None if lengths is None else I.active_mask(lengths, t)
        before = list(orc.evicted)
        ref = orc.step(qn[t], kn[t], vn[t], act)
        out = layer.step(qd[t], kd[t], vd[t], active=None if act is None else torch.from_numpy(act).cuda())
        H.assert_close(H.f64(out), ref, H.BF16_ABS, H.BF16_REL, "out at step %d" % t)
        if list(orc.evicted) != before:
            n_evictions += 1
            vic = layer.victims()
            for b in range(wl.batch):
                if orc.evicted[b] != before[b]:
                    assert vic[b].tolist() == orc.last_victims[b], "victims of rollout %d at step %d" % (b, t)
        ln, base = layer.counters()
        oln, obase = orc.counters()
        assert np.array_equal(ln, oln) and np.array_equal(base, obase), "counters differ at step %d" % t
        if t % score_every == 0 or t == T - 1:
            check_scores(wl, orc, layer, "step %d" % t)
    assert orc.min_margin >= MIN_MARGIN, "inputs leave a selection too close to call (%.2e): pick others" % orc.min_margin
    assert n_evictions >= 3
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")
    assert layer.poll_error() == 0
    return orc, layer


@pytest.mark.parametrize("splits,waves", [(1, 4), (3, 4), (1, 8), (2, 8)])
def test_scored_run_matches_oracle(splits, waves):
    wl = small()
    orc, layer = run_both(wl, wl.steps, n_recent=24, q_gain=48.0, splits=splits, waves=waves)
    # the policy did something other than slide: some evicted chunk was not the oldest one
    assert any(list(orc.positions(b)) != list(range(orc.evicted[b], orc.appended[b])) for b in range(wl.batch))


def test_scored_run_with_a_long_window():
    # 66 groups walked by one workgroup of 4 wavefronts (17 groups' scores folded per wavefront and
    # step), one rollout so that the oracle stays cheap
    # (80 eligible entries and a seed whose margins are wide: with thousands eligible the chunk's
    # boundary would fall between scores too close to call)
    wl = small(batch=1, n_q_heads=2, n_kv_heads=1, window=2112, chunk=64, steps=2112 + 3 * 64 + 5, seed=5)
    orc, layer = run_both(wl, wl.steps, n_recent=2032, q_gain=48.0, splits=1, waves=4, score_every=257)
    assert layer.plan()[1] == 1


def test_scored_run_with_question_tokens_and_ragged_lengths():
    wl = small(batch=4, window=160, n_sink=64, chunk=40, steps=260, seed=2006)    # a seed with wide margins
    lengths = np.array([260, 90, 200, 131])
    run_both(wl, wl.steps, n_recent=16, q_gain=48.0, lengths=lengths, prompt_len=[64, 1, 37, 0])


def test_with_only_the_oldest_chunk_eligible_outputs_equal_the_sliding_window_bitwise():
    wl = small(batch=2, window=128, chunk=32, steps=300)
    enc = I.encoder_params(wl)
    plain = H.make_layer(wl, enc)
    _, scored = make_both(wl, n_recent=wl.window - wl.chunk)
    q, k, v = (x.cuda() for x in I.qkv_steps(wl, 0, wl.steps))
    for t in range(wl.steps):
        assert torch.equal(scored.step(q[t], k[t], v[t]), plain.step(q[t], k[t], v[t])), "step %d" % t
    assert all(np.array_equal(a, b) for a, b in zip(scored.counters(), plain.counters()))
    # the two encoders (plain ALU here, MFMA there) agree to fp32 rounding
    H.assert_close(scored.get_state(), plain.get_state(), 1e-5, 1e-4, "state")
    Ks, Vs = scored.gather_window()
    Kp, Vp = plain.gather_window()
    n = int(plain.counters()[0][0] - plain.counters()[1][0])
    assert torch.equal(Ks[:, :, :n], Kp[:, :, :n]) and torch.equal(Vs[:, :, :n], Vp[:, :, :n])


def _random_selection_cases(n):
    rng = np.random.default_rng(424242)
    cases = []
    for _ in range(n):
        n_sink = int(rng.choice([0, 32, 64]))
        ring = 32 * int(rng.integers(1, 7))
        C = int(rng.integers(1, ring + 1))
        n_recent = int(rng.integers(0, ring - C + 1))
        cases.append((n_sink + ring, C, n_recent, n_sink))
    return cases


@pytest.mark.parametrize("W,C,n_recent,n_sink", [(96, 32, 24, 0), (160, 40, 0, 32), (128, 7, 100, 0), (64, 64, 0, 0),
                                                   (608, 520, 50, 0),     # (a chunk long enough for several encoding workgroups)
                                                   (64, 1, 20, 0), (96, 1, 10, 32)]    # (a step that evicts also refills the ring)
                         + _random_selection_cases(12))
def test_selection_on_injected_scores_is_bit_exact(W, C, n_recent, n_sink):
    # scores with few distinct values (plenty of ties), the same float32 numbers on both sides
    # (ends one short of a full ring.  With C = 1 a step that evicts refills the ring and chooses again, from
    # scores nobody planted: such a run ends with its first eviction)
    wl = small(batch=3, window=W, chunk=C, n_sink=n_sink, steps=W - n_sink + (6 * C - 1 if C > 1 else 1))
    orc, layer = make_both(wl, n_recent)
    Wr = W - n_sink
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    rng = np.random.default_rng(7)
    n_checked = 0
    for t in range(wl.steps):
        if len(orc.win[0]) == Wr - 1:                  # the next step fills the ring, the one after evicts: plant the scores
            sc = np.zeros((wl.batch, W), dtype=np.float32)
            levels = rng.integers(2, 9)
            sc[:, :Wr - 1] = (rng.integers(0, levels, (wl.batch, Wr - 1)) / np.float32(levels)).astype(np.float32)
            layer.set_scores(sc)
            for b in range(wl.batch):
                orc.set_scores(b, sc[b, :Wr - 1].astype(np.float64))
        before = list(orc.evicted)
        ref = orc.step(qn[t], kn[t], vn[t])
        out = layer.step(qd[t], kd[t], vd[t])
        H.assert_close(H.f64(out), ref, H.BF16_ABS, H.BF16_REL, "out at step %d" % t)
        if list(orc.evicted) != before:
            vic = layer.victims()
            _, ps = layer.scores()
            for b in range(wl.batch):
                # (with C = 1 the step has already chosen again: what left shows in the ring order below)
                if C > 1:
                    assert vic[b].tolist() == orc.last_victims[b], "victims of rollout %d at step %d" % (b, t)
                n = len(orc.win[b])
                if C > 1:
                    assert np.array_equal(ps[b, :n], orc.positions(b)), "ring order of rollout %d after step %d" % (b, t)
                else:     # ... and has brought its next victim to the front: the same tokens, the oracle's victim gone
                    assert sorted(ps[b, :n].tolist()) == sorted(orc.positions(b).tolist()), (b, t)
                    assert orc.last_victims[b][0] not in ps[b, :n]
            n_checked += 1
    assert n_checked >= (4 if C > 1 else 1)
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")
    # what the cache holds is what the oracle's ring holds, token for token
    Kw, Vw = layer.gather_window()
    _, ps = layer.scores()
    for b in range(wl.batch):
        by_pos = {e.pos: e for e in orc.win[b]}
        n = len(orc.win[b])
        ks = torch.stack([torch.from_numpy(by_pos[int(p)].k) for p in ps[b, :n]]).to(torch.bfloat16)     # [n, H_kv, d]
        vs = torch.stack([torch.from_numpy(by_pos[int(p)].v) for p in ps[b, :n]]).to(torch.bfloat16)
        assert torch.equal(Kw[b, :, :n].cpu(), ks.transpose(0, 1))
        assert torch.equal(Vw[b, :, :n].cpu(), vs.transpose(0, 1))
    assert layer.poll_error() == 0


def test_scored_compact_id_lists():
    # finished rollouts dropped from the batch: the selection and the scores follow the id list
    wl = small(batch=4, window=96, chunk=32, steps=180, seed=2006)
    lengths = np.array([180, 60, 150, 101])
    orc, layer = make_both(wl, n_recent=24)
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    q = (q.float() * 48.0).to(q.dtype)
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    for t in range(wl.steps):
        act = I.active_mask(lengths, t)
        ids = np.nonzero(act)[0].astype(np.int32)
        ref = orc.step(qn[t], kn[t], vn[t], act)
        idt = torch.from_numpy(ids).cuda()
        out = layer.step_ids(q[t][ids].cuda().contiguous(), k[t][ids].cuda().contiguous(), v[t][ids].cuda().contiguous(), idt)
        H.assert_close(H.f64(out), ref[ids], H.BF16_ABS, H.BF16_REL, "out at step %d" % t)
    assert orc.min_margin >= MIN_MARGIN
    check_scores(wl, orc, layer, "end")
    assert all(np.array_equal(a, b) for a, b in zip(layer.counters(), orc.counters()))
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")


def test_scored_steps_replayed_from_a_graph_equal_eager_steps():
    wl = small(batch=3, window=96, chunk=32, steps=230)
    _, eager = make_both(wl, 24)
    _, layer = make_both(wl, 24)
    layer.set_option(ptenc.OPT_COUNTERS_IN_PLACE, 1)
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    q = (q.float() * 48.0).to(q.dtype)
    q, k, v = q.cuda(), k.cuda(), v.cuda()
    ref = eager.run(q, k, v)
    qs, ks, vs, outs = torch.empty_like(q[0]), torch.empty_like(k[0]), torch.empty_like(v[0]), torch.empty_like(q[0])
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer.step(qs, ks, vs, outs)
    for t in range(wl.steps):
        qs.copy_(q[t]); ks.copy_(k[t]); vs.copy_(v[t])
        g.replay()
        if t % 11 == 0:
            torch.cuda.synchronize()
            _ = (q[t].float() * 2).sum().item()              # unrelated eager work between replays
        assert torch.equal(outs, ref[t]), "replay %d" % t
    assert all(np.array_equal(a, b) for a, b in zip(layer.counters(), eager.counters()))
    assert np.array_equal(layer.victims(), eager.victims()) and (layer.victims() >= 0).all()
    assert np.array_equal(layer.get_state(), eager.get_state())
    sg, pg = layer.scores()
    se, pe = eager.scores()
    assert np.array_equal(pg, pe) and np.array_equal(sg, se)


def test_scored_full_size_properties():
    # the benchmark's shape (B 128, 28 / 4 heads, window 4096, chunk 128) through three evictions, in the
    # launch configuration the benchmark times.  Which tokens leave is a floating-point decision the CPU
    # cannot replay at this size, so this checks what holds for any correct choice.
    from oracle.ring_model import evicted_closed_form
    wl = I.WORKLOADS["qwen7b"]
    W, C, Hq = wl.window, wl.chunk, wl.n_q_heads
    T = W + 2 * C + 5
    n_recent = W // 2
    dev = torch.device("cuda:0")
    enc = I.encoder_params(wl, device=dev)
    layer = ptenc.Layer(wl.batch, Hq, wl.n_kv_heads, wl.head_dim, W, C, dtype=wl.torch_dtype, poison_cache=True)
    layer.set_option(ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED)
    layer.set_encoder(enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    layer.reset()
    seen_victims = [set() for _ in range(wl.batch)]
    for t0 in range(0, T, 512):
        t1 = min(T, t0 + 512)
        q, k, v = I.qkv_steps(wl, t0, t1, device=dev)
        out = layer.run(q, k, v)
        assert torch.isfinite(out.float()).all()
        vic = layer.victims()
        for b in range(wl.batch):
            if vic[b, 0] >= 0:
                seen_victims[b].update(vic[b].tolist())
    assert layer.poll_error() == 0
    ln, base = layer.counters()
    E = evicted_closed_form(T, W, C)
    assert (ln == T).all() and (base == E).all() and E == 3 * C
    sc, ps = layer.scores()
    n = T - E
    for b in range(0, wl.batch, 9):
        live = ps[b, :n]
        assert (ps[b, n:] == -1).all()
        assert len(set(live.tolist())) == n and live.min() >= 0 and live.max() == T - 1    # distinct tokens of this rollout
        assert set(range(T - n_recent, T)) <= set(live.tolist())                           # the recent ones are protected
        assert not (set(live.tolist()) & seen_victims[b])                                  # what left stays out
        s_b = sc[b, :n]
        assert np.isfinite(s_b).all() and (s_b >= 0).all()
        # every step hands out H_q of probability; the folded scores of the survivors cannot exceed it
        assert 0.2 * Hq * (T - 1) < s_b.sum() <= Hq * (T - 1) * (1 + 1e-4)
    # the last eviction took C distinct tokens, none of them among the then most recent ones
    vic = layer.victims()
    t_ev = W + 2 * C                      # 0-based step of the third eviction: positions < t_ev existed
    for b in range(0, wl.batch, 9):
        assert len(set(vic[b].tolist())) == C and vic[b].max() < t_ev - n_recent


def test_scored_policy_argument_checks():
    wl = small()
    enc = I.encoder_params(wl)
    plain = H.make_layer(wl, enc)
    sc = torch.zeros((wl.batch, wl.window), dtype=torch.float32, device="cuda")
    with pytest.raises(ptenc.PtencError) as ei:
        ptenc.ptenc_get_scores(plain.ctx, sc, None)         # sliding policy keeps no scores
    assert ei.value.status == ptenc.ERR_STATE
    _, layer = make_both(wl, 24)
    q, k, v = (x.cuda() for x in I.qkv_steps(wl, 0, 4))
    layer.step(q[0], k[0], v[0])
    with pytest.raises(ptenc.PtencError) as ei:
        layer.set_counters(np.full(wl.batch, 5), np.full(wl.batch, 2))    # live tokens without scores
    assert ei.value.status == ptenc.ERR_UNSUPPORTED


def test_scored_run_is_invariant_to_where_the_counters_start():
    # counters that start far beyond 2^32, and ones that cross 2^32 during the run, shift positions and
    # victims by the start value and nothing else (margins are wide, so rounding order cannot change a choice)
    wl = small()
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    q = (q.float() * 48.0).to(q.dtype)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    runs = []
    for x in (0, 2**32 - 70, 2**40 + 5):
        _, layer = make_both(wl, 24)
        layer.set_counters(np.full(wl.batch, x), np.full(wl.batch, x))
        outs, vics = [], []
        for t in range(wl.steps):
            base_before = layer.counters()[1] if t >= wl.window else None
            outs.append(layer.step(qd[t], kd[t], vd[t]).cpu())
            if base_before is not None and (layer.counters()[1] != base_before).any():
                vics.append(layer.victims() - x)
        sc, ps = layer.scores()
        ln, base = layer.counters()
        n = int(ln[0] - base[0])
        order = np.argsort(ps[:, :n], axis=1)
        runs.append((torch.stack(outs), vics, np.take_along_axis(ps[:, :n], order, 1) - x,
                     np.take_along_axis(sc[:, :n], order, 1), ln - x, base - x, layer.get_state()))
        assert layer.poll_error() == 0
    assert len(runs[0][1]) >= 3
    for r in runs[1:]:
        assert len(r[1]) == len(runs[0][1]) and all(np.array_equal(a, b) for a, b in zip(r[1], runs[0][1]))
        assert np.array_equal(r[2], runs[0][2]) and np.array_equal(r[4], runs[0][4]) and np.array_equal(r[5], runs[0][5])
        assert np.allclose(r[3], runs[0][3], rtol=1e-4, atol=1e-5)
        H.assert_close(H.f64(r[0]), H.f64(runs[0][0]), 2e-3, 2e-2, "outputs from shifted counters")
        H.assert_close(r[6], runs[0][6], 1e-5, 1e-4, "state from shifted counters")


def test_rebasing_an_emptied_ring_forgets_the_old_choice_of_victims():
    # fill a ring by whole steps (its victims get chosen), empty it through ptenc_set_counters, fill it
    # again by bare appends: nothing has been attended, all scores are zero, so the tie rule decides
    # and the oldest chunk leaves; a choice kept from the first filling would name other places
    wl = small(batch=2, window=64, chunk=16, steps=64)
    _, layer = make_both(wl, n_recent=8)
    q, k, v = I.qkv_steps(wl, 0, 2 * wl.window)
    q = (q.float() * 48.0).to(q.dtype)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    for t in range(wl.window):
        layer.step(qd[t], kd[t], vd[t])
    first = layer.victims()
    assert any(first[b].tolist() != list(range(wl.chunk)) for b in range(wl.batch))   # the scores did decide
    x = 1000
    layer.set_counters(np.full(wl.batch, x), np.full(wl.batch, x))
    for t in range(wl.window, 2 * wl.window):
        layer.append(kd[t], vd[t])
    dkv = wl.n_kv_heads * wl.head_dim
    dbg = torch.zeros((wl.batch, 2, wl.chunk, dkv), dtype=torch.bfloat16, device="cuda")
    layer.evict_encode(dbg_chunk=dbg)
    vic = layer.victims()
    for b in range(wl.batch):
        assert vic[b].tolist() == list(range(x, x + wl.chunk))
        assert torch.equal(dbg[b, 0].cpu(), k[wl.window:wl.window + wl.chunk, b].reshape(wl.chunk, dkv))
        assert torch.equal(dbg[b, 1].cpu(), v[wl.window:wl.window + wl.chunk, b].reshape(wl.chunk, dkv))
    ln, base = layer.counters()
    assert (ln == x + wl.window).all() and (base == x + wl.chunk).all()
    assert layer.poll_error() == 0


@pytest.mark.parametrize("seed", range(10))
def test_random_call_sequences_with_planted_scores(seed):
    # full, masked and compact steps in random order, options changed in mid-run, rollouts that fill
    # their rings at different ticks; whenever a rollout is one token short of a full ring its scores
    # are planted (few distinct values, the same float32 numbers on both sides), so that every choice
    # of victims is an integer decision both sides must take alike, whatever rounding did to the
    # scores in between
    rng = np.random.default_rng(900 + seed)
    n_sink = int(rng.choice([0, 32]))
    ring = 32 * int(rng.integers(1, 5))
    C = int(rng.integers(2, ring + 1))
    n_recent = int(rng.integers(0, ring - C + 1))
    wl = small(batch=4, n_q_heads=8, window=n_sink + ring, n_sink=n_sink, chunk=C, steps=3 * ring + 3 * C,
               seed=int(rng.integers(1, 1 << 20)))
    B, T, W = wl.batch, wl.steps, wl.window
    orc, layer = make_both(wl, n_recent)
    q, k, v = I.qkv_steps(wl, 0, T)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    n_evictions = 0
    for t in range(T):
        plant = [b for b in range(B) if len(orc.win[b]) == ring - 1]
        if plant:
            sc, _ = layer.scores()                       # the library's own values go back to it unchanged
            sc = np.array(sc, dtype=np.float32)
            levels = int(rng.integers(2, 9))
            for b in range(B):
                if b in plant:
                    sc[b, :ring - 1] = (rng.integers(0, levels, ring - 1) / np.float32(levels)).astype(np.float32)
                    orc.set_scores(b, sc[b, :ring - 1].astype(np.float64))
                else:
                    orc.set_scores(b, orc.scores(b))     # its own values; the waiting probabilities are dropped, as on the GPU
            layer.set_scores(sc)
        op = str(rng.choice(["step", "masked", "ids", "option"]))
        before = list(orc.evicted)
        if op == "step":
            ref = orc.step(qn[t], kn[t], vn[t])
            H.assert_close(H.f64(layer.step(qd[t], kd[t], vd[t])), ref, H.BF16_ABS, H.BF16_REL, "step %d" % t)
        elif op == "masked":
            act = rng.random(B) < 0.6
            ref = orc.step(qn[t], kn[t], vn[t], act)
            out = layer.step(qd[t], kd[t], vd[t], active=torch.from_numpy(act.astype(np.uint8)).cuda())
            H.assert_close(H.f64(out), ref, H.BF16_ABS, H.BF16_REL, "masked step %d" % t)
        elif op == "ids":
            idx = rng.permutation(np.nonzero(rng.random(B) < 0.6)[0])
            m = np.zeros(B, dtype=bool)
            m[idx] = True
            ref = orc.step(qn[t], kn[t], vn[t], m)
            it = torch.from_numpy(idx).cuda()
            out = layer.step_ids(qd[t][it].contiguous(), kd[t][it].contiguous(), vd[t][it].contiguous(), it.to(torch.int32))
            if len(idx):
                H.assert_close(H.f64(out), ref[idx], H.BF16_ABS, H.BF16_REL, "compact step %d" % t)
        else:
            which = str(rng.choice(["splits", "waves", "parts"]))
            if which == "splits":
                layer.set_option(ptenc.OPT_SPLITS, int(rng.choice([0, 1, 2, 3])))
            elif which == "waves":
                layer.set_option(ptenc.OPT_WAVES, int(rng.choice([0, 4, 8])))
            else:
                layer.set_option(ptenc.OPT_ENCODE_PARTS, int(rng.choice([0, 1, 2, 5])))
        ln, base = layer.counters()
        oln, obase = orc.counters()
        assert np.array_equal(ln, oln) and np.array_equal(base, obase), "counters after tick %d" % t
        if list(orc.evicted) != before:
            _, ps = layer.scores()
            for b in range(B):
                if orc.evicted[b] != before[b]:
                    n = len(orc.win[b])
                    assert np.array_equal(ps[b, :n], orc.positions(b)), "ring order of rollout %d after tick %d" % (b, t)
                    n_evictions += 1
    assert n_evictions >= 2
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")
    assert layer.poll_error() == 0
