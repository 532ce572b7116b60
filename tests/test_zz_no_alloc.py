"""ptenc_decode_step_noalloc, the decode step for callers that cannot allocate, against ptenc_decode_step on the
same inputs: two contexts decode the same steps, one through the caller's scratch block, one through the
library's built-in block.  The plans are chosen so that the block is really used (several window splits
hand partial results over; several encoding workgroups share a chunk).  Two runs in a row, the second with a
smaller configuration, so the second finds the first one's leftovers in the block."""
import numpy as np
import pytest
import torch

from paper_2602_16839_amd import inputs as I
from paper_2602_16839_amd import ptenc
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _pair(wl, splits, enc_parts, force_generic=False):
    enc = I.encoder_params(wl)
    waves = 4 if wl.dtype == "bf16" else 0      # 4-wavefront workgroups: every split of these small windows gets groups
    a = H.make_layer(wl, enc, splits=splits, enc_parts=enc_parts, force_generic=force_generic, waves=waves)
    b = H.make_layer(wl, enc, splits=splits, enc_parts=enc_parts, force_generic=force_generic, waves=waves)
    return a, b


def _run_pair(wl, splits, enc_parts, masked=False, force_generic=False):
    ref_layer, na_layer = _pair(wl, splits, enc_parts, force_generic)
    assert ref_layer.plan() == na_layer.plan() and ref_layer.plan()[1] == splits
    # the no-alloc context's own scratch block must stay untouched: fill it with a pattern
    na_layer.scratch.fill_(0x5A)
    T = wl.steps
    q, k, v = I.qkv_steps(wl, 0, T)
    q = (q.float() * 16.0).to(q.dtype)                       # peaked enough for the splits' rescaling to matter
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    lengths = np.full(wl.batch, T)
    if masked:
        lengths = np.array([T - 3 * b for b in range(wl.batch)])
    abs_tol, rel_tol = H.tolerances(wl)
    out_na = torch.empty_like(qd[0])
    for t in range(T):
        act = torch.from_numpy(I.active_mask(lengths, t)).cuda() if masked else None
        ref = ref_layer.step(qd[t], kd[t], vd[t], active=act)
        got = na_layer.step_noalloc(qd[t], kd[t], vd[t], out_na, active=act)
        H.assert_close(H.f64(got), H.f64(ref), abs_tol, rel_tol, "no-alloc out at step %d" % t)
        # same kernels, same order of summation: the two outputs are the same bits
        assert torch.equal(got, ref), "step %d" % t
    la, ba = ref_layer.counters()
    lb, bb = na_layer.counters()
    assert np.array_equal(la, lb) and np.array_equal(ba, bb) and (ba > 0).any()
    H.assert_close(na_layer.get_state(), ref_layer.get_state(), H.S_ABS, H.S_REL, "no-alloc state")
    assert np.array_equal(na_layer.get_state(), ref_layer.get_state())
    assert ref_layer.poll_error() == 0 and na_layer.poll_error() == 0
    assert bool((na_layer.scratch == 0x5A).all()), "the caller's scratch block was written by the no-alloc step"
    return na_layer


def test_noalloc_step_equals_decode_step_twice_in_a_row_second_smaller():
    # MFMA path: 3 window splits (partials through the block), 2 encoding workgroups per chunk (shares of S')
    big = I.WORKLOADS["qwen7b"].replace(batch=5, n_q_heads=8, n_kv_heads=2, window=512, chunk=128, steps=512 + 128 + 9)
    _run_pair(big, splits=3, enc_parts=2)
    small = I.WORKLOADS["qwen7b"].replace(batch=2, n_q_heads=4, n_kv_heads=1, window=256, chunk=64, steps=256 + 64 + 5,
                                          seed=77)
    _run_pair(small, splits=2, enc_parts=2, masked=True)


def test_noalloc_step_plain_path():
    # fp32 plain path: the window splits' partials go through the block as well (separate combine launch)
    wl = I.WORKLOADS["tiny_f32"].replace(batch=3, window=48, chunk=16, steps=48 + 16 + 3)
    _run_pair(wl, splits=3, enc_parts=0)
    wl = I.WORKLOADS["tiny_f32"].replace(batch=1, window=32, chunk=8, steps=45, seed=5)
    _run_pair(wl, splits=2, enc_parts=0)


def test_noalloc_step_rejects_what_does_not_fit():
    # 32 splits of a 7B-shaped batch need 59 MiB of partial results: more than the built-in block
    wl = I.WORKLOADS["qwen7b"]
    layer = ptenc.Layer(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk)
    enc = I.encoder_params(wl, device="cuda:0")
    layer.set_encoder(enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    layer.reset()
    q, k, v = I.qkv_steps(wl, 0, 1, device="cuda:0")
    out = torch.empty_like(q[0])
    layer.step_noalloc(q[0], k[0], v[0], out)                   # the default plan (one split) fits
    layer.set_option(ptenc.OPT_SPLITS, 32)
    need = wl.batch * wl.n_q_heads * 32 * (wl.head_dim + 2) * 4
    assert need > ptenc.NOALLOC_SCRATCH_BYTES
    with pytest.raises(ptenc.PtencError) as ei:
        layer.step_noalloc(q[0], k[0], v[0], out)
    assert ei.value.status == ptenc.ERR_TOO_LARGE and "built-in" in str(ei.value)
    ln, _ = layer.counters()
    assert (ln == 1).all()                                      # the rejected call did nothing
    assert layer.poll_error() == 0
