"""Parity of the HIP path (through the C ABI) with the CPU fp64 oracle, element by element, on
seeded inputs small enough for the oracle yet spanning several 32-slot groups, window splits,
ring wrap-around and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import pte_oracle as po
from oracle.ring_model import RingModel
from paper_2602_16839_amd import inputs as I
from tests import helpers as H

pytestmark = pytest.mark.gpu


def small(name, **kw):
    return I.WORKLOADS[name].replace(**kw)


def test_tiny_f32_config_in_full():
    # the small fp32 configuration, every rollout, every one of the 512 steps
    wl = I.WORKLOADS["tiny_f32"]
    layer, orc = H.run_both(wl, wl.steps)
    ln, base = layer.counters()
    assert (ln == 512).all() and (base == 256).all()
    assert layer.plan()[0] == 0


@pytest.mark.parametrize("splits", [1, 3])
def test_bf16_mfma_path_small_window(splits):
    # 5 groups of 32 slots, chunk 48 wraps and is not group aligned, 7 query heads per KV head
    wl = small("qwen7b", batch=3, n_q_heads=14, n_kv_heads=2, window=160, chunk=48, steps=420)
    layer, _ = H.run_both(wl, wl.steps, splits=splits)
    assert layer.plan()[:2] == (1, splits)


@pytest.mark.parametrize("splits", [5, 17, 32])
def test_many_window_splits_merge_in_kernel(splits):
    # 33 groups of 32 slots: every split count leaves some splits empty and some with one group
    wl = small("qwen7b", batch=2, n_q_heads=14, n_kv_heads=2, window=1056, chunk=96, steps=1200)
    layer, _ = H.run_both(wl, wl.steps, splits=splits, check_every=37)
    assert layer.plan()[:2] == (1, splits)


@pytest.mark.parametrize("splits", [1, 2])
def test_eight_wavefront_workgroups(splits):
    # the 512-thread variant (query groups of at most 8): evictions, question tokens, splits
    wl = small("qwen3b", batch=3, n_q_heads=16, n_kv_heads=2, window=352, n_sink=32, chunk=72, steps=800)
    layer, _ = H.run_both(wl, wl.steps, splits=splits, waves=8, check_every=23, prompt_len=[32, 0, 9])
    assert layer.plan()[:2] == (1, splits)
    # a query group of 14 does not fit 8 rows: the request falls back to 4 wavefronts and still works
    wl = small("qwen7b", batch=2, n_q_heads=28, n_kv_heads=2, window=96, chunk=32, steps=150)
    H.run_both(wl, wl.steps, waves=8, check_every=11)


@pytest.mark.parametrize("W,C,n_sink,waves,splits,parts", [(1056, 520, 0, 4, 1, 0), (1120, 800, 32, 8, 2, 3),
                                                          (2112, 2070, 0, 4, 3, 0), (1024, 1024, 0, 8, 1, 5),
                                                          (160, 48, 0, 4, 1, 8), (96, 33, 0, 4, 1, 2)])
def test_chunks_are_encoded_by_several_workgroups(W, C, n_sink, waves, splits, parts):
    # the encoding of a chunk is shared by up to 8 workgroups per rollout (by default one per 64 tokens),
    # each a contiguous range of the chunk's 32-token groups; here with chunks that are not whole groups
    # (so later evictions start inside a group), that wrap around the ring's end, that are the whole ring,
    # and with more workgroups than the chunk has groups (some get nothing)
    wl = small("qwen3b", batch=2, n_q_heads=4, n_kv_heads=2, window=W, n_sink=n_sink, chunk=C,
               steps=(W - n_sink) + 2 * C + 40)
    lengths = np.array([wl.steps, (W - n_sink) + C + 17])        # the second rollout stops before its third eviction
    layer, _ = H.run_both(wl, wl.steps, splits=splits, waves=waves, check_every=61, lengths=lengths,
                          prompt_len=[n_sink, 5] if n_sink else None, enc_parts=parts)
    assert layer.plan()[:2] == (1, splits)
    ln, base = layer.counters()
    Wr = W - n_sink
    assert [int(x) for x in base] == [-(-(int(T) - Wr) // C) * C for T in lengths]      # an eviction at steps Wr, Wr + C, ...


@pytest.mark.parametrize("W,C,n_sink,waves,splits", [(1056, 520, 0, 4, 1), (1120, 800, 32, 8, 2), (2112, 2070, 0, 4, 3),
                                                     (1024, 1024, 0, 8, 1), (160, 48, 0, 4, 1), (96, 33, 0, 4, 1),
                                                     (64, 1, 0, 4, 1), (128, 32, 0, 8, 2)])
def test_chunks_folded_ahead_of_time_by_the_rollouts_own_workgroups(W, C, n_sink, waves, splits):
    # the way launches that fill the chip encode (forced here at small sizes): the workgroup of KV head 0 folds the
    # next chunk's groups into the pending block one at a time while the ring refills, and the evicting step
    # adds what is pending.  Chunks that are not whole groups, that wrap, that are the whole ring, single tokens;
    # a rollout that stops between evictions with groups pending.
    wl = small("qwen3b", batch=2, n_q_heads=4, n_kv_heads=2, window=W, n_sink=n_sink, chunk=C,
               steps=(W - n_sink) + 2 * C + 40)
    lengths = np.array([wl.steps, (W - n_sink) + C + max(1, C // 2)])
    layer, _ = H.run_both(wl, wl.steps, splits=splits, waves=waves, check_every=61, lengths=lengths,
                          prompt_len=[n_sink, 5] if n_sink else None, enc_inline=1)
    assert layer.plan()[:2] == (1, splits)
    ln, base = layer.counters()
    Wr = W - n_sink
    assert [int(x) for x in base] == [-(-(int(T) - Wr) // C) * C for T in lengths]


@pytest.mark.parametrize("inline_a,inline_b", [(1, 0), (0, 1), (1, 1)])
def test_pending_groups_survive_changes_of_who_encodes_and_of_entry_point(inline_a, inline_b):
    # Groups folded ahead of time wait in the pending block until the eviction, whoever performs it: the mode
    # changes in mid-refill (a ragged batch shrinks from a launch that fills the chip to one that does not), steps
    # are taken through the separate entry points (which fold nothing ahead), counters are rewritten with the
    # same values by the host (which drops what is pending: the eviction then folds the whole chunk itself).
    from paper_2602_16839_amd import ptenc
    wl = small("qwen7b", batch=3, n_q_heads=4, n_kv_heads=2, window=192, chunk=96, steps=192 + 3 * 96 + 11)
    enc = I.encoder_params(wl)
    orc = H.make_oracle(wl, enc)
    layer = H.make_layer(wl, enc, enc_inline=inline_a)
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    for t in range(wl.steps):
        ref = orc.step(qn[t], kn[t], vn[t])
        if t == 192 + 40:                     # first refill under way: somebody else takes over
            layer.set_option(ptenc.OPT_ENCODE_INLINE, inline_b)
        if t == 192 + 96 + 30:                # second refill: the host rewrites the counters as they are
            ln, base = layer.counters()
            layer.set_counters(ln, base)
        if 192 + 2 * 96 + 20 <= t < 192 + 2 * 96 + 50:   # third refill: thirty steps through the separate calls
            layer.evict_encode()
            layer.append(kd[t], vd[t])
            out = layer.attend(qd[t])
        else:
            out = layer.step(qd[t], kd[t], vd[t])
        if t % 7 == 0 or t == wl.steps - 1:
            H.assert_close(H.f64(out), ref, H.BF16_ABS, H.BF16_REL, "out at step %d" % t)
        if t in (192, 192 + 96, 192 + 2 * 96, 192 + 3 * 96, wl.steps - 1):
            H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state after step %d" % t)
    ln, base = layer.counters()
    oln, obase = orc.counters()
    assert np.array_equal(ln, oln) and np.array_equal(base, obase) and layer.poll_error() == 0


def test_bf16_generic_path_small_window():
    wl = small("qwen3b", batch=2, n_q_heads=8, n_kv_heads=2, window=96, chunk=40, steps=250)
    layer, _ = H.run_both(wl, wl.steps, force_generic=True, splits=2)
    assert layer.plan()[0] == 0


def test_bf16_row_major_when_window_is_not_a_multiple_of_32():
    wl = small("qwen3b", batch=2, n_q_heads=4, n_kv_heads=2, window=50, chunk=7, steps=130)
    layer, _ = H.run_both(wl, wl.steps)
    assert layer.plan()[0] == 0


@pytest.mark.parametrize("W,C", [(32, 32), (64, 1), (128, 128), (96, 32)])
def test_degenerate_window_and_chunk_sizes(W, C):
    wl = small("qwen3b", batch=2, n_q_heads=8, n_kv_heads=1, window=W, chunk=C, steps=2 * W + 9)
    H.run_both(wl, wl.steps, splits=2 if W >= 64 else 1)


@pytest.mark.parametrize("name,d", [("tiny_f32", 256), ("tiny_f32", 8), ("tiny_f32", 37), ("qwen3b", 80), ("qwen3b", 256)])
def test_head_dims_other_than_128_take_the_plain_path(name, d):
    # the largest head_dim the library takes, the smallest, odd ones; bf16 and fp32
    wl = I.WORKLOADS[name].replace(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=d, window=40, chunk=12, steps=70)
    layer, _ = H.run_both(wl, wl.steps, check_every=3)
    assert layer.plan()[0] == 0


def test_empty_lists_zero_steps_and_all_inactive_steps_change_nothing():
    from paper_2602_16839_amd import ptenc
    for name in ("qwen7b", "tiny_f32"):
        wl = small(name, batch=3, window=64, chunk=16, steps=20) if name == "qwen7b" else small(name, batch=3, window=24, chunk=8, steps=20)
        enc = I.encoder_params(wl)
        layer = H.make_layer(wl, enc)
        q, k, v = (x.cuda() for x in I.qkv_steps(wl, 0, 6))
        layer.run(q[:5], k[:5], v[:5])
        before = (layer.counters(), layer.get_state().copy(), [t.clone() for t in layer.gather_window()])
        # a run of zero steps
        ptenc.ptenc_decode_run(layer.ctx, q[:0], k[:0], v[:0], q[:0].clone(), None, 0)
        # an empty rollout list: nothing is launched, pointers may be anything
        ids = torch.zeros(0, dtype=torch.int32, device="cuda")
        layer.step_ids(q[5][:0].contiguous(), k[5][:0].contiguous(), v[5][:0].contiguous(), ids)
        layer.run_ids(q[5][:0].contiguous(), k[5][:0].contiguous(), v[5][:0].contiguous(), ids, np.array([0, 0, 0]))
        # a step in which no rollout is active: zeros out, nothing moves
        off = torch.zeros(wl.batch, dtype=torch.uint8, device="cuda")
        out = layer.step(q[5], k[5], v[5], active=off)
        assert (out == 0).all()
        ln, base = layer.counters()
        assert np.array_equal(ln, before[0][0]) and np.array_equal(base, before[0][1])
        assert np.array_equal(layer.get_state(), before[1])
        Kw, Vw = layer.gather_window()
        assert torch.equal(Kw, before[2][0]) and torch.equal(Vw, before[2][1])
        assert layer.poll_error() == 0


@pytest.mark.parametrize("hq,hkv", [(16, 1), (4, 4), (32, 8)])
def test_group_sizes_1_4_16(hq, hkv):
    wl = small("llama8b", batch=2, n_q_heads=hq, n_kv_heads=hkv, window=64, chunk=16, steps=100)
    H.run_both(wl, wl.steps)


@pytest.mark.parametrize("norm", [po.NORM_FROBENIUS, po.NORM_ROW_L2, po.NORM_NONE])
def test_norm_modes_and_zero_initialised_state(norm):
    wl = small("qwen3b", batch=2, n_q_heads=4, n_kv_heads=2, window=64, chunk=32, steps=200,
               n_global=16, rank=24)
    H.run_both(wl, wl.steps, norm_mode=norm, with_global_kv=(norm != po.NORM_NONE), check_every=7)


@pytest.mark.parametrize("G,r", [(48, 64), (64, 16), (1, 1), (64, 64), (33, 17), (17, 50)])
def test_global_token_counts_and_latent_widths(G, r):
    # the global-token ablation sizes (16 / 32 / 48 / 64) and latent widths up to 64, on the MFMA encoder
    wl = small("qwen7b", batch=2, n_q_heads=14, n_kv_heads=2, window=64, chunk=40, steps=150, n_global=G, rank=r)
    layer, _ = H.run_both(wl, wl.steps, check_every=13)
    assert layer.plan() == (1, 4, 1) or layer.plan()[2] == 1


def test_peaky_softmax_exercises_the_online_rescale():
    # queries scaled x64: scores ~ 4 N(0,1), i.e. a range of ~30 base-2 units across the window, so
    # the running max keeps moving; values stay O(0.25) so that the absolute bar is not spent on
    # the bf16 rounding of the output itself
    wl = small("qwen3b", batch=2, n_q_heads=8, n_kv_heads=2, window=128, chunk=32, steps=300, scale=0.25)
    H.run_both(wl, wl.steps, q_gain=64.0, splits=2)


def test_ragged_rollouts_are_masked():
    wl = small("ragged", batch=6, window=64, chunk=16, steps=200)
    lengths = np.array([200, 1, 63, 64, 65, 130])
    layer, orc = H.run_both(wl, wl.steps, lengths=lengths)
    ln, base = layer.counters()
    assert ln.tolist() == lengths.tolist()


def _compact_run(wl, lengths, T, **layer_kw):
    """Decode with compact id lists (finished rollouts dropped from the batch) next to the oracle's masked run."""
    enc = I.encoder_params(wl)
    orc = H.make_oracle(wl, enc)
    layer = H.make_layer(wl, enc, **layer_kw)
    q, k, v = I.qkv_steps(wl, 0, T)
    rows_q, rows_k, rows_v, ids, offs, refs = [], [], [], [], [0], []
    for t in range(T):
        act = I.active_mask(lengths, t)
        ref = orc.step(H.f64(q[t]), H.f64(k[t]), H.f64(v[t]), act)
        idx = np.nonzero(act)[0]
        it = torch.from_numpy(idx)
        rows_q.append(q[t][it]); rows_k.append(k[t][it]); rows_v.append(v[t][it])
        ids.append(it.to(torch.int32)); offs.append(offs[-1] + len(idx)); refs.append(ref[idx])
    cq, ck, cv = (torch.cat(x).cuda() for x in (rows_q, rows_k, rows_v))
    cid = torch.cat(ids).cuda()
    return layer, orc, cq, ck, cv, cid, np.array(offs), np.concatenate(refs)


@pytest.mark.parametrize("kind", ["mfma", "generic_bf16", "f32"])
def test_compact_rollout_lists_equal_masked_decoding(kind):
    lengths = np.array([90, 1, 31, 32, 33, 70, 0, 90])
    if kind == "f32":
        wl = small("tiny_f32", batch=8, window=32, chunk=8, steps=90)
        kw = {}
    else:
        wl = small("ragged", batch=8, n_q_heads=8, n_kv_heads=2, window=32, chunk=8, steps=90)
        kw = dict(force_generic=(kind == "generic_bf16"))
    layer, orc, cq, ck, cv, cid, offs, ref = _compact_run(wl, lengths, wl.steps, **kw)
    out = layer.run_ids(cq, ck, cv, cid, offs)
    abs_tol, rel_tol = H.tolerances(wl)
    H.assert_close(H.f64(out), ref, abs_tol, rel_tol, "compact outputs")
    ln, base = layer.counters()
    oln, obase = orc.counters()
    assert np.array_equal(ln, oln) and np.array_equal(base, obase) and ln.tolist() == lengths.tolist()
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")
    assert layer.poll_error() == 0
    # step by step gives the same bits as the batched call; so does mixing in a full-batch masked step
    layer2 = H.make_layer(wl, I.encoder_params(wl), **kw)
    outs = []
    for t in range(wl.steps):
        r0, r1 = int(offs[t]), int(offs[t + 1])
        if r1 > r0:
            outs.append(layer2.step_ids(cq[r0:r1], ck[r0:r1], cv[r0:r1], cid[r0:r1]))
    assert torch.equal(torch.cat(outs), out) and np.array_equal(layer2.get_state(), layer.get_state())


@pytest.mark.parametrize("kind,in_place", [("mfma", 0), ("mfma", 1), ("generic_bf16", 0), ("f32", 0)])
def test_rollouts_pause_and_resume_in_compact_lists(kind, in_place):
    # every step lists a random subset in random order (some steps nobody, some everybody), and every
    # tenth step is a masked full-batch step: a rollout's counters must survive any number of steps it
    # sits out, whichever interface the steps in between went through
    from paper_2602_16839_amd import ptenc
    if kind == "f32":
        wl = small("tiny_f32", batch=7, window=32, chunk=8, steps=140)
        kw = {}
    else:
        wl = small("ragged", batch=7, n_q_heads=8, n_kv_heads=2, window=32, chunk=8, steps=140)
        kw = dict(force_generic=(kind == "generic_bf16"), enc_parts=2 if in_place else 0)
    enc = I.encoder_params(wl)
    orc = H.make_oracle(wl, enc)
    layer = H.make_layer(wl, enc, **kw)
    if in_place:
        layer.set_option(ptenc.OPT_COUNTERS_IN_PLACE, 1)
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    rng = np.random.default_rng(77)
    abs_tol, rel_tol = H.tolerances(wl)
    for t in range(wl.steps):
        p = rng.choice([0.0, 0.15, 0.5, 0.9, 1.0])
        act = rng.random(wl.batch) < p
        ref = orc.step(H.f64(q[t]), H.f64(k[t]), H.f64(v[t]), act)
        if t % 10 == 9:
            out = layer.step(q[t].cuda(), k[t].cuda(), v[t].cuda(), active=torch.from_numpy(act.astype(np.uint8)).cuda())
            got, want = H.f64(out), ref
        else:
            idx = rng.permutation(np.nonzero(act)[0])
            it = torch.from_numpy(idx)
            out = layer.step_ids(q[t][it].cuda(), k[t][it].cuda(), v[t][it].cuda(), it.to(torch.int32).cuda())
            got, want = H.f64(out), ref[idx]
        if got.size:
            H.assert_close(got, want, abs_tol, rel_tol, "outputs at step %d" % t)
        ln, base = layer.counters()
        oln, obase = orc.counters()
        assert np.array_equal(ln, oln) and np.array_equal(base, obase), "counters at step %d" % t
    assert (orc.counters()[1] > 0).any()          # some rollout did evict
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")
    assert layer.poll_error() == 0


def test_bad_rollout_id_is_flagged_and_skipped():
    from paper_2602_16839_amd import ptenc
    wl = small("ragged", batch=4, n_q_heads=8, n_kv_heads=2, window=32, chunk=8, steps=4)
    layer = H.make_layer(wl, I.encoder_params(wl))
    q, k, v = (x.cuda() for x in I.qkv_steps(wl, 0, 1))
    ids = torch.tensor([2, 9, 0], dtype=torch.int32, device="cuda")
    out = layer.step_ids(q[0][:3].contiguous(), k[0][:3].contiguous(), v[0][:3].contiguous(), ids)
    assert layer.poll_error() == ptenc.DEVERR_BAD_ID
    ln, _ = layer.counters()
    assert ln.tolist() == [1, 0, 1, 0]
    assert out[0].any() and out[2].any()


@pytest.mark.parametrize("name,d_in,d_out,G,r", [("qwen3b", 512, 384, 32, 32), ("qwen3b", 260, 77, 16, 24),
                                                 ("tiny_f32", 96, 130, 32, 32)])
def test_state_applied_as_weight_delta(name, d_in, d_out, G, r):
    wl = small(name, batch=5, window=32, chunk=8, steps=60, n_global=G, rank=r)
    if name != "tiny_f32":
        wl = wl.replace(n_q_heads=4, n_kv_heads=2)
    layer, orc = H.run_both(wl, wl.steps, check_every=20)          # leaves 4 evictions' worth of state in S
    ad = I.adapter_inputs(wl, d_in, d_out)
    x, y0, At, Bt = (H.f64(ad[k]) for k in ("x", "y", "At", "Bt"))
    S = orc.state()
    ref = np.stack([po.apply_delta(x[b], At.T, S[b], Bt.T, y0[b]) for b in range(wl.batch)])
    dev = {k: v.cuda() for k, v in ad.items()}
    y = dev["y"].clone()
    layer.apply_delta(dev["x"], dev["At"], dev["Bt"], y)
    abs_tol, rel_tol = H.tolerances(wl)
    H.assert_close(H.f64(y), ref, max(abs_tol, 2e-5), rel_tol, "y + x (A S B)")
    assert np.abs(ref - y0).max() > 0.02                           # the delta is not lost in the tolerance
    # masked rollouts keep their rows; a compact id list touches only the listed rows
    y = dev["y"].clone()
    mask = torch.tensor([1, 0, 1, 1, 0], dtype=torch.uint8, device="cuda")
    layer.apply_delta(dev["x"], dev["At"], dev["Bt"], y, active=mask)
    assert torch.equal(y[1], dev["y"][1]) and torch.equal(y[4], dev["y"][4])
    H.assert_close(H.f64(y[[0, 2, 3]]), ref[[0, 2, 3]], max(abs_tol, 2e-5), rel_tol, "masked")
    ids = torch.tensor([3, 0], dtype=torch.int32, device="cuda")
    yc = dev["y"][[3, 0]].contiguous()
    layer.apply_delta(dev["x"][[3, 0]].contiguous(), dev["At"], dev["Bt"], yc, ids=ids)
    H.assert_close(H.f64(yc), ref[[3, 0]], max(abs_tol, 2e-5), rel_tol, "compact")
    assert layer.poll_error() == 0


@pytest.mark.parametrize("kind", ["mfma", "f32"])
def test_a_captured_step_replays_like_eager_steps(kind):
    # one decode step captured into a HIP graph (counters updated in place) and replayed with refilled
    # inputs, with eager work and synchronisation between replays; every replay is checked
    from paper_2602_16839_amd import ptenc
    if kind == "mfma":
        wl = small("qwen7b", batch=3, n_q_heads=14, n_kv_heads=2, window=96, chunk=32, steps=150)
    else:
        wl = small("tiny_f32", batch=3, window=24, chunk=8, steps=60)
    enc = I.encoder_params(wl)
    q, k, v = (x.cuda() for x in I.qkv_steps(wl, 0, wl.steps))
    parts = 3 if kind == "mfma" else 0       # (three encoding workgroups per rollout for chunks of one or two groups)
    eager = H.make_layer(wl, enc, enc_parts=parts)
    ref = eager.run(q, k, v)
    layer = H.make_layer(wl, enc, enc_parts=parts)
    layer.set_option(ptenc.OPT_COUNTERS_IN_PLACE, 1)
    qs, ks, vs = torch.empty_like(q[0]), torch.empty_like(k[0]), torch.empty_like(v[0])
    outs = torch.empty_like(q[0])
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer.step(qs, ks, vs, outs)
    for t in range(wl.steps):
        qs.copy_(q[t]); ks.copy_(k[t]); vs.copy_(v[t])
        g.replay()
        if t % 7 == 0:
            torch.cuda.synchronize()
            _ = (q[t].float() * 2).sum().item()          # unrelated eager work between replays
        assert torch.equal(outs, ref[t]), "replay %d" % t
    ln, base = layer.counters()
    eln, ebase = eager.counters()
    assert np.array_equal(ln, eln) and np.array_equal(base, ebase)
    assert np.array_equal(layer.get_state(), eager.get_state())
    assert layer.poll_error() == 0


def test_init_state_matches_oracle():
    for name in ("tiny_f32", "qwen7b"):
        wl = I.WORKLOADS[name].replace(batch=2)
        enc = I.encoder_params(wl)
        layer = H.make_layer(wl, enc)
        e = {k: H.f64(v) for k, v in enc.items()}
        Qa_ref, S0_ref = po.init_state(e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"])
        Qa, S0 = layer.encoder_state()
        H.assert_close(Qa, Qa_ref, 1e-5, 1e-5, "Q_a")
        H.assert_close(S0, S0_ref, H.S_ABS, H.S_REL, "S_0")
        H.assert_close(layer.get_state(), np.stack([S0_ref] * 2), H.S_ABS, H.S_REL, "S after reset")


# ------------------------------------------------------------------------------------------------
# pinned question tokens in front of the sliding window
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("splits", [1, 3])
def test_question_tokens_mfma_path(splits):
    # 64 reserved slots + a ring of 96; question lengths: full, one token, mid-group, none
    wl = small("qwen7b", batch=4, n_q_heads=14, n_kv_heads=2, window=160, n_sink=64, chunk=40, steps=260)
    layer, orc = H.run_both(wl, wl.steps, splits=splits, prompt_len=[64, 1, 37, 0])
    assert layer.plan()[:2] == (1, splits)
    Kw, Vw = layer.gather_window()
    for b in range(wl.batch):
        Ko, Vo = orc.window_kv(b)
        n = Ko.shape[0]
        assert np.array_equal(H.f64(Kw[b, :, :n]), Ko.transpose(1, 0, 2)) and not Kw[b, :, n:].any()
        assert np.array_equal(H.f64(Vw[b, :, :n]), Vo.transpose(1, 0, 2)) and not Vw[b, :, n:].any()


def test_question_tokens_generic_paths():
    # fp32, and bf16 with reserved slots that are not whole groups (row-major layout)
    wl = small("tiny_f32", batch=3, window=40, n_sink=8, chunk=5, steps=100)
    layer, _ = H.run_both(wl, wl.steps, prompt_len=[8, 0, 3])
    assert layer.plan()[0] == 0
    wl = small("qwen3b", batch=2, n_q_heads=4, n_kv_heads=2, window=69, n_sink=5, chunk=16, steps=150)
    layer, _ = H.run_both(wl, wl.steps, splits=2, prompt_len=[5, 2])
    assert layer.plan()[0] == 0


@pytest.mark.parametrize("kind", ["mfma", "f32"])
def test_finished_rollouts_are_recycled_one_at_a_time(kind):
    # a rollout engine's loop: a rollout that has finished is reset and given a new question (its own
    # reserved slots only) while the others keep decoding; twice, different rollouts, different lengths
    from paper_2602_16839_amd import ptenc
    if kind == "mfma":
        wl = small("qwen7b", batch=4, n_q_heads=14, n_kv_heads=2, window=160, n_sink=64, chunk=40, steps=230)
    else:
        wl = small("tiny_f32", batch=4, window=40, n_sink=12, chunk=9, steps=120)
    enc = I.encoder_params(wl)
    orc = H.make_oracle(wl, enc)
    layer = H.make_layer(wl, enc)
    pl = H.prefill_both(wl, orc, layer, [wl.n_sink, 1, wl.n_sink // 2, 0])
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    qn, kn, vn = H.f64(q), H.f64(k), H.f64(v)
    abs_tol, rel_tol = H.tolerances(wl)
    # the new questions come from another seed of the same recipe
    pk2, pv2 = I.prompt_kv(wl.replace(seed=wl.seed + 1))
    recycle = {wl.steps // 3: ([2], [wl.n_sink // 3]), 2 * wl.steps // 3: ([3, 0], [wl.n_sink, 2])}
    for t in range(wl.steps):
        if t in recycle:
            ids, lens = recycle[t]
            mask = np.zeros(wl.batch, dtype=np.uint8)
            mask[ids] = 1
            layer.reset(torch.from_numpy(mask).cuda())
            layer.prefill_ids(pk2[ids].cuda().contiguous(), pv2[ids].cuda().contiguous(),
                              torch.tensor(ids, dtype=torch.int32, device="cuda"), lens)
            for b, n in zip(ids, lens):
                orc.reset_rollout(b)
                orc.prefill(b, H.f64(pk2[b, :n]), H.f64(pv2[b, :n]))
                pl[b] = n
            assert np.array_equal(layer.prompt_len(), pl)
        ref = orc.step(qn[t], kn[t], vn[t])
        out = layer.step(qd[t], kd[t], vd[t])
        H.assert_close(H.f64(out), ref, abs_tol, rel_tol, "out at step %d" % t)
        ln, base = layer.counters()
        oln, obase = orc.counters()
        assert np.array_equal(ln, oln) and np.array_equal(base, obase), "counters at step %d" % t
    H.assert_close(layer.get_state(), orc.state(), H.S_ABS, H.S_REL, "state S")
    Kw, Vw = layer.gather_window()
    for b in range(wl.batch):
        ko, vo = orc.window_kv(b)
        assert torch.equal(Kw[b, :, :len(ko)].cpu().to(torch.float64), torch.from_numpy(ko).transpose(0, 1))
        assert torch.equal(Vw[b, :, :len(vo)].cpu().to(torch.float64), torch.from_numpy(vo).transpose(0, 1))
    assert layer.poll_error() == 0
    # an id outside the batch is flagged and skipped; an empty list does nothing
    layer.prefill_ids(pk2[:1].cuda().contiguous(), pv2[:1].cuda().contiguous(), torch.tensor([wl.batch], dtype=torch.int32, device="cuda"), [1])
    assert layer.poll_error() == ptenc.DEVERR_BAD_ID
    layer.prefill_ids(pk2[:0].cuda().contiguous(), pv2[:0].cuda().contiguous(), torch.zeros(0, dtype=torch.int32, device="cuda"), [])
    assert np.array_equal(layer.prompt_len(), pl)


def test_question_tokens_only_no_thinking_tokens_yet():
    # attention right after prefill, before any append: softmax over the question tokens alone
    wl = small("qwen3b", batch=2, n_q_heads=8, n_kv_heads=2, window=96, n_sink=32, chunk=16, steps=4)
    enc = I.encoder_params(wl)
    orc, layer = H.make_oracle(wl, enc), H.make_layer(wl, enc)
    H.prefill_both(wl, orc, layer, [32, 7])
    q, _, _ = I.qkv_steps(wl, 0, 1)
    out = layer.attend(q[0].cuda())
    for b in range(2):
        H.assert_close(H.f64(out[b]), orc.attend(b, H.f64(q[0, b])), H.BF16_ABS, H.BF16_REL, "prompt-only b=%d" % b)
    assert layer.poll_error() == 0
    layer.reset()                                  # reset forgets the question tokens
    assert layer.prompt_len().tolist() == [0, 0]


# ------------------------------------------------------------------------------------------------
# integer / byte work: bit exact
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name,W,C,n_sink", [("tiny_f32", 24, 5, 0), ("qwen3b", 64, 24, 0), ("qwen3b", 40, 40, 0),
                                             ("qwen3b", 96, 24, 32), ("tiny_f32", 30, 4, 7)])
def test_ring_contents_and_eviction_order_are_bit_exact(name, W, C, n_sink):
    wl = small(name, batch=3, window=W, chunk=C, steps=3 * W + 5, n_sink=n_sink)
    if name != "tiny_f32":
        wl = wl.replace(n_q_heads=4, n_kv_heads=2)
    enc = I.encoder_params(wl)
    layer = H.make_layer(wl, enc)
    ring = RingModel(wl.batch, W, C, n_sink=n_sink)
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    kd, vd = k.cuda(), v.cuda()
    dkv = wl.d_kv
    pl = np.zeros(wl.batch, dtype=np.int64)
    if n_sink:
        pl = I.prompt_lengths(wl)
        pk, pv = I.prompt_kv(wl)
        layer.prefill(pk.cuda(), pv.cuda(), pl)
    for t in range(wl.steps):
        dbg = torch.zeros((wl.batch, 2, C, dkv), dtype=wl.torch_dtype, device="cuda")
        layer.evict_encode(dbg_chunk=dbg)
        evicted = ring.evict()
        for b in range(wl.batch):
            if evicted[b]:
                p0 = int(ring.base[b]) - C          # positions [p0, p0 + C) just left
                assert torch.equal(dbg[b, 0].cpu(), k[p0:p0 + C, b].reshape(C, dkv))
                assert torch.equal(dbg[b, 1].cpu(), v[p0:p0 + C, b].reshape(C, dkv))
            else:
                assert not dbg[b].any()
        layer.append(kd[t], vd[t])
        ring.append()
        ln, base = layer.counters()
        assert np.array_equal(ln, ring.len) and np.array_equal(base, ring.base)
        if t % 9 == 0 or t == wl.steps - 1:
            Kw, Vw = layer.gather_window()
            raw = layer.cache_view().cpu()
            for b in range(wl.batch):
                n = int(ring.n_live()[b])
                p0 = int(ring.base[b])
                P = int(pl[b])
                if P:
                    assert torch.equal(Kw[b, :, :P].cpu(), pk[b, :P].transpose(0, 1))
                    assert torch.equal(Vw[b, :, :P].cpu(), pv[b, :P].transpose(0, 1))
                assert torch.equal(Kw[b, :, P:P + n].cpu(), k[p0:p0 + n, b].transpose(0, 1))
                assert torch.equal(Vw[b, :, P:P + n].cpu(), v[p0:p0 + n, b].transpose(0, 1))
                assert not Kw[b, :, P + n:].any() and not Vw[b, :, P + n:].any()
                # physical slots: slot s holds position slot_pos[b, s] (documented offset function)
                for s in (n_sink, n_sink + (W - n_sink) // 2, W - 1):
                    p = int(ring.slot_pos[b, s])
                    if p >= 0:
                        off = layer.cache_offset(b, 1 if wl.n_kv_heads > 1 else 0, s, 3, 0)
                        assert raw[off] == k[p, b, 1 if wl.n_kv_heads > 1 else 0, 3]
    assert layer.poll_error() == 0


@pytest.mark.parametrize("name,generic", [("qwen3b", False), ("qwen3b", True), ("tiny_f32", False)])
def test_rotation_invariance_of_the_ring(name, generic):
    # starting the counters at x shifts every slot by x mod W; outputs, windows and S are bit-identical.
    # The offsets include counters that cross 2^31 and 2^32 during the run and ones far beyond
    # (the ring index is taken in 32 bits only while the counters fit).
    wl = small(name, batch=2, n_q_heads=8, n_kv_heads=2, window=96, chunk=32, steps=230)
    enc = I.encoder_params(wl)
    q, k, v = (t.cuda() for t in I.qkv_steps(wl, 0, wl.steps))
    results = []
    for x in (0, 37, 96 * 1000003 + 95, 2**31 - 100, 2**32 - 50, 2**33 + 77, 2**62 + 12345):
        layer = H.make_layer(wl, enc, force_generic=generic)
        layer.set_counters(np.full(2, x), np.full(2, x))
        out = layer.run(q, k, v)
        Kw, Vw = layer.gather_window()
        ln, base = layer.counters()
        results.append((out.cpu(), Kw.cpu(), Vw.cpu(), layer.get_state(), ln - x, base - x))
    for r in results[1:]:
        assert torch.equal(r[1], results[0][1]) and torch.equal(r[2], results[0][2])
        assert np.array_equal(r[4], results[0][4]) and np.array_equal(r[5], results[0][5])
        if name == "qwen3b" and not generic:
            # the MFMA encoder contracts a chunk's tokens four at a time by their place in a 32-slot group,
            # so which tokens share a partial sum rotates with the ring: S agrees to rounding
            H.assert_close(r[3], results[0][3], 1e-6, 1e-5, "rotated state S")
        else:
            assert np.array_equal(r[3], results[0][3])
        # attention walks physical groups, so the summation order (not the set of keys) rotates too
        # (fp32 rounding order, hence now and then another bf16 rounding of the output's last bit)
        H.assert_close(H.f64(r[0]), H.f64(results[0][0]), 2e-3, 2e-2, "rotated outputs")


def test_decode_run_equals_repeated_decode_step():
    wl = small("qwen7b", batch=2, n_q_heads=14, n_kv_heads=2, window=64, chunk=16, steps=150)
    enc = I.encoder_params(wl)
    q, k, v = (t.cuda() for t in I.qkv_steps(wl, 0, wl.steps))
    a = H.make_layer(wl, enc)
    out_a = a.run(q, k, v)
    b = H.make_layer(wl, enc)
    out_b = torch.stack([b.step(q[t], k[t], v[t]) for t in range(wl.steps)])
    assert torch.equal(out_a, out_b)
    assert np.array_equal(a.get_state(), b.get_state())
    # and equals the three separate entry points
    c = H.make_layer(wl, enc)
    outs = []
    for t in range(wl.steps):
        c.evict_encode()
        c.append(k[t], v[t])
        outs.append(c.attend(q[t]))
    assert torch.equal(torch.stack(outs), out_a)


def test_snapshot_and_resume_is_bit_identical():
    wl = small("qwen3b", batch=2, n_q_heads=8, n_kv_heads=2, window=64, chunk=16, steps=160)
    enc = I.encoder_params(wl)
    q, k, v = (t.cuda() for t in I.qkv_steps(wl, 0, wl.steps))
    a = H.make_layer(wl, enc)
    a.run(q[:100], k[:100], v[:100])
    snap_cache, snap_S, (ln, base) = a.cache.clone(), a.get_state(), a.counters()
    ref = a.run(q[100:], k[100:], v[100:])
    b = H.make_layer(wl, enc)
    b.cache.copy_(snap_cache)
    b.set_state(snap_S)
    b.set_counters(ln, base)
    got = b.run(q[100:], k[100:], v[100:])
    assert torch.equal(got, ref) and np.array_equal(a.get_state(), b.get_state())


def test_device_side_misuse_sets_sticky_error_bits():
    from paper_2602_16839_amd import ptenc
    wl = small("qwen3b", batch=2, n_q_heads=4, n_kv_heads=2, window=32, chunk=8, steps=40)
    enc = I.encoder_params(wl)
    layer = H.make_layer(wl, enc)
    q, k, v = (t.cuda() for t in I.qkv_steps(wl, 0, 40))
    out = layer.attend(q[0])                       # empty window, active rollout
    assert not out.any()
    assert layer.poll_error() == ptenc.DEVERR_ATTEND_EMPTY
    layer.reset()
    assert layer.poll_error() == 0
    for t in range(32):
        layer.append(k[t], v[t])
    assert layer.poll_error() == 0
    before = layer.cache.clone()
    layer.append(k[32], v[32])                     # window full, no eviction requested
    assert layer.poll_error() == ptenc.DEVERR_APPEND_FULL
    assert torch.equal(before, layer.cache)
    ln, base = layer.counters()
    assert (ln == 32).all() and (base == 0).all()
    mask = torch.tensor([1, 0], dtype=torch.uint8, device="cuda")
    layer.reset(mask)                              # partial reset keeps the sticky word
    assert layer.poll_error() == ptenc.DEVERR_APPEND_FULL
    ln, base = layer.counters()
    assert ln.tolist() == [0, 32]


def test_nan_poisoned_dead_slots_never_reach_outputs():
    wl = small("qwen3b", batch=2, n_q_heads=8, n_kv_heads=2, window=96, chunk=40, steps=150)
    enc = I.encoder_params(wl)
    orc = H.make_oracle(wl, enc)
    layer = H.make_layer(wl, enc, splits=2)
    ring = RingModel(wl.batch, wl.window, wl.chunk)
    q, k, v = I.qkv_steps(wl, 0, wl.steps)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    raw = layer.cache_view()
    for t in range(wl.steps):
        ref = orc.step(H.f64(q[t]), H.f64(k[t]), H.f64(v[t]))
        layer.evict_encode()
        layer.append(kd[t], vd[t])
        ring.step()
        # poison every dead slot of rollout 0 / head 1 before attending
        dead = sorted(set(range(wl.window)) - set(ring.live_slots(0).tolist()))
        for s in dead[:: max(1, len(dead) // 6)]:
            for which in (0, 1):
                raw[layer.cache_offset(0, 1, s, 5, which)] = float("nan")
        out = layer.attend(qd[t])
        H.assert_close(H.f64(out), ref, H.BF16_ABS, H.BF16_REL, "step %d" % t)


def test_two_contexts_on_two_streams_do_not_disturb_each_other():
    # every context owns its cache, state and scratch, and every call takes its stream: two layers decoding
    # at the same time on different streams give the bits they give alone
    wls = [small("qwen7b", batch=3, n_q_heads=14, n_kv_heads=2, window=160, chunk=48, steps=260),
           small("qwen3b", batch=5, n_q_heads=8, n_kv_heads=2, window=96, chunk=32, steps=260, seed=9)]
    encs = [I.encoder_params(w) for w in wls]
    ins = [tuple(t.cuda() for t in I.qkv_steps(w, 0, w.steps)) for w in wls]
    alone = []
    for w, e, (q, k, v) in zip(wls, encs, ins):
        layer = H.make_layer(w, e, splits=2)
        alone.append((layer.run(q, k, v).clone(), layer.get_state()))
    torch.cuda.synchronize()
    layers = [H.make_layer(w, e, splits=2) for w, e in zip(wls, encs)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.empty_like(ins[0][0]), torch.empty_like(ins[1][0])]
    torch.cuda.synchronize()
    for t0 in range(0, 260, 20):                       # interleave the two runs in slices of 20 steps
        for i in (0, 1):
            q, k, v = ins[i]
            with torch.cuda.stream(streams[i]):
                layers[i].run(q[t0:t0 + 20], k[t0:t0 + 20], v[t0:t0 + 20], out=outs[i][t0:t0 + 20])
    torch.cuda.synchronize()
    for i in (0, 1):
        assert torch.equal(outs[i], alone[i][0])
        assert np.array_equal(layers[i].get_state(), alone[i][1])
        assert layers[i].poll_error() == 0
