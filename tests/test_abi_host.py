"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
rejects bad configurations, and its documented cache layout is a bijection.  No kernel runs."""
import ctypes as C
import os
import re

import pytest

from paper_2602_16839_amd import ptenc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ptenc.h")).read()
    declared = set(re.findall(r"\b(ptenc_[a-z_]+)\s*\(", header))
    assert declared == set(ptenc.EXPORTS)
    L = ptenc.lib()
    for name in declared:
        assert hasattr(L, name), name


def cfg(**kw):
    base = dict(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=128, window=64, chunk=16, n_sink=0,
                n_global=32, rank=32, dtype=ptenc.BF16, norm_mode=0, norm_eps=0.0, softmax_scale=0.0)
    base.update(kw)
    return ptenc.Config(**base)


def test_query_sizes():
    cb, sb, xb = ptenc.ptenc_query_sizes(cfg())
    assert cb == 2 * 2 * 2 * 64 * 128 * 2
    assert sb % 256 == 0 and sb >= 2 * 32 * 32 * 4 + 2 * 32 * 32 * 4 + 2 * 2 * 8 + 4
    assert xb >= 2 * 4 * ptenc.MAX_SPLITS * 130 * 4
    cb32, _, _ = ptenc.ptenc_query_sizes(cfg(dtype=ptenc.F32, head_dim=64))
    assert cb32 == 2 * 2 * 2 * 64 * 64 * 4


@pytest.mark.parametrize("bad,status", [
    (dict(batch=0), ptenc.ERR_INVALID_ARG),
    (dict(n_q_heads=5), ptenc.ERR_INVALID_ARG),
    (dict(chunk=0), ptenc.ERR_INVALID_ARG),
    (dict(chunk=65), ptenc.ERR_INVALID_ARG),
    (dict(dtype=7), ptenc.ERR_INVALID_ARG),
    (dict(norm_mode=3), ptenc.ERR_INVALID_ARG),
    (dict(softmax_scale=-1.0), ptenc.ERR_INVALID_ARG),
    (dict(n_sink=64), ptenc.ERR_INVALID_ARG),
    (dict(n_sink=-1), ptenc.ERR_INVALID_ARG),
    (dict(n_sink=56, chunk=16), ptenc.ERR_INVALID_ARG),
    (dict(head_dim=512), ptenc.ERR_UNSUPPORTED),
    (dict(rank=65), ptenc.ERR_UNSUPPORTED),
    (dict(n_global=128), ptenc.ERR_UNSUPPORTED),
])
def test_bad_configs_are_rejected(bad, status):
    with pytest.raises(ptenc.PtencError) as e:
        ptenc.ptenc_query_sizes(cfg(**bad))
    assert e.value.status == status


def _host_ctx(c):
    """A context over fake (never dereferenced) aligned addresses: create touches no device memory."""
    h = C.c_void_p()
    st = ptenc.lib().ptenc_create(C.byref(c), C.c_void_p(0x10000), C.c_void_p(0x20000), C.c_void_p(0x30000), C.byref(h))
    return st, h


def test_create_checks_pointers_and_order_of_calls():
    L = ptenc.lib()
    h = C.c_void_p()
    assert L.ptenc_create(C.byref(cfg()), None, C.c_void_p(256), C.c_void_p(256), C.byref(h)) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_create(C.byref(cfg()), C.c_void_p(0x10010), C.c_void_p(256), C.c_void_p(256), C.byref(h)) == ptenc.ERR_INVALID_ARG
    st, h = _host_ctx(cfg())
    assert st == ptenc.OK
    # nothing may be decoded before the encoder is set
    assert L.ptenc_reset(h, None, None) == ptenc.ERR_STATE
    assert L.ptenc_cache_append(h, C.c_void_p(256), C.c_void_p(256), None, None) == ptenc.ERR_STATE
    assert L.ptenc_decode_attn(h, None, C.c_void_p(256), None, None) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_set_option(h, ptenc.OPT_SPLITS, ptenc.MAX_SPLITS + 1) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_set_option(h, 99, 0) == ptenc.ERR_INVALID_ARG
    for v, st in ((-1, ptenc.ERR_INVALID_ARG), (9, ptenc.ERR_INVALID_ARG), (8, ptenc.OK), (0, ptenc.OK)):
        assert L.ptenc_set_option(h, ptenc.OPT_ENCODE_PARTS, v) == st
    assert L.ptenc_set_option(h, ptenc.OPT_SPLITS, 3) == ptenc.OK
    assert ptenc.ptenc_get_plan(h) == (1, 3, 1)
    assert L.ptenc_destroy(h) == ptenc.OK
    assert L.ptenc_destroy(None) == ptenc.ERR_INVALID_ARG
    assert ptenc.status_string(ptenc.ERR_UNSUPPORTED) == "unsupported configuration"


def test_scored_policy_options_are_checked_on_the_host():
    L = ptenc.lib()
    _, h = _host_ctx(cfg())                                # bf16, head_dim 128: the MFMA path
    W, Ck = cfg().window, cfg().chunk
    assert L.ptenc_set_option(h, ptenc.OPT_RECENT, W - Ck + 1) == ptenc.ERR_INVALID_ARG     # fewer than a chunk eligible
    assert L.ptenc_set_option(h, ptenc.OPT_RECENT, -2) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_set_option(h, ptenc.OPT_RECENT, W - Ck) == ptenc.OK
    assert L.ptenc_set_option(h, ptenc.OPT_EVICT_POLICY, 2) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_get_scores(h, C.c_void_p(256), None, None) == ptenc.ERR_STATE           # sliding policy keeps none
    assert L.ptenc_set_option(h, ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED) == ptenc.OK
    assert L.ptenc_set_option(h, ptenc.OPT_FORCE_GENERIC, 1) == ptenc.ERR_UNSUPPORTED      # the scores come from the MFMA kernel
    assert L.ptenc_get_scores(h, None, None, None) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_destroy(h) == ptenc.OK
    for bad in (cfg(dtype=ptenc.F32, head_dim=64), cfg(window=40, chunk=8), cfg(n_q_heads=36, n_kv_heads=2)):
        _, h = _host_ctx(bad)                               # fp32, untiled window, 18 query heads per KV head
        assert L.ptenc_set_option(h, ptenc.OPT_EVICT_POLICY, ptenc.POLICY_SCORED) == ptenc.ERR_UNSUPPORTED
        assert L.ptenc_destroy(h) == ptenc.OK


def test_stack_sizes_and_argument_checks():
    L = ptenc.lib()
    c = cfg()
    one = ptenc.ptenc_query_sizes(c)
    cb, sb, xb = ptenc.ptenc_stack_query_sizes(c, 5)
    assert (cb, sb, xb) == (5 * one[0], 5 * one[1], one[2])        # scratch is shared by the layers
    a = C.c_size_t()
    for n in (0, -1, 1025):
        assert L.ptenc_stack_query_sizes(C.byref(c), n, C.byref(a), None, None) == ptenc.ERR_INVALID_ARG
    h = C.c_void_p()
    assert L.ptenc_stack_create(C.byref(c), 2, None, C.c_void_p(0x20000), C.c_void_p(0x30000), C.byref(h)) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_stack_create(C.byref(c), 2, C.c_void_p(0x1000000), C.c_void_p(0x2000000), C.c_void_p(0x3000000), C.byref(h)) == ptenc.OK
    x = C.c_void_p()
    assert L.ptenc_stack_layer(h, 2, C.byref(x)) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_stack_layer(h, 1, C.byref(x)) == ptenc.OK and x.value
    assert L.ptenc_stack_graph_launch(h, None) == ptenc.ERR_STATE   # nothing recorded
    assert L.ptenc_stack_decode_step(h, None, None, None, None, None, None) == ptenc.ERR_INVALID_ARG
    assert L.ptenc_stack_destroy(h) == ptenc.OK
    assert L.ptenc_stack_destroy(None) == ptenc.ERR_INVALID_ARG


@pytest.mark.parametrize("c", [cfg(), cfg(dtype=ptenc.F32, head_dim=64, window=48, chunk=5),
                               cfg(window=40)])   # window 40 is not a multiple of 32: row-major bf16
def test_cache_layout_is_a_bijection(c):
    st, h = _host_ctx(c)
    assert st == ptenc.OK
    seen = set()
    per_slab = 2 * c.window * c.head_dim
    for b in (0, c.batch - 1):
        for hh in range(c.n_kv_heads):
            for slot in range(c.window):
                for i in range(c.head_dim):
                    for which in (0, 1):
                        off = ptenc.ptenc_cache_offset(h, b, hh, slot, i, which)
                        slab = b * c.n_kv_heads + hh
                        assert slab * per_slab <= off < (slab + 1) * per_slab
                        seen.add(off)
    assert len(seen) == 2 * c.n_kv_heads * per_slab
    with pytest.raises(ptenc.PtencError):
        ptenc.ptenc_cache_offset(h, 0, 0, c.window, 0, 0)
    ptenc.ptenc_destroy(h)


def test_reserved_question_slots_choose_the_plan():
    # the MFMA path needs whole 32-slot groups on both sides of the boundary
    for n_sink, kernel in ((0, 1), (32, 1), (4, 0), (16, 0)):
        st, h = _host_ctx(cfg(window=96, n_sink=n_sink))
        assert st == ptenc.OK
        assert ptenc.ptenc_get_plan(h)[0] == kernel
        L = ptenc.lib()
        assert L.ptenc_prefill(h, C.c_void_p(256), C.c_void_p(256), None, 8, None) == ptenc.ERR_INVALID_ARG
        assert L.ptenc_prefill(h, C.c_void_p(256), C.c_void_p(256), C.c_void_p(256), 8, None) == ptenc.ERR_STATE
        ptenc.ptenc_destroy(h)


def test_tiled_layout_matches_its_documented_formula():
    # bf16, d = 128, W % 32 == 0: 16 KiB groups of 32 slots = [K tile 0 | K tile 1 | V^T]
    c = cfg(window=96)
    st, h = _host_ctx(c)
    for slot, i in [(0, 0), (5, 77), (17, 127), (31, 8), (32, 0), (70, 33), (95, 127)]:
        grp, tl = divmod(slot, 32)
        t, m = divmod(tl, 16)
        cc, kg, e = i // 32, (i % 32) // 8, i % 8
        assert ptenc.ptenc_cache_offset(h, 0, 0, slot, i, 0) == grp * 8192 + t * 2048 + ((cc * 4 + kg) * 16 + m) * 8 + e
        it, mm = divmod(i, 16)
        kgv, ev = (tl % 16) // 4, (tl // 16) * 4 + tl % 4
        assert ptenc.ptenc_cache_offset(h, 0, 0, slot, i, 1) == grp * 8192 + 4096 + ((it * 4 + kgv) * 16 + mm) * 8 + ev
    ptenc.ptenc_destroy(h)


def test_missing_library_fails_loudly(monkeypatch):
    # no CPU fallback: without the shared library the binding raises instead of computing anything
    monkeypatch.setattr(ptenc, "_LIB", None)
    monkeypatch.delenv("PTENC_LIB", raising=False)
    monkeypatch.setattr(ptenc, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libptenc.so"))
    with pytest.raises(FileNotFoundError):
        ptenc.lib()
    with pytest.raises(FileNotFoundError):
        ptenc.ptenc_query_sizes(cfg())


def test_oracle_and_product_do_not_import_each_other():
    pkg = os.path.join(ROOT, "paper_2602_16839_amd")
    for root, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(root, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|oracle[./]pte_oracle|oracle[./]ring_model", text, re.M), \
                    "%s reaches into the oracle" % f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2602_16839_amd" not in text and "ptenc" not in text and "import torch" not in text


@pytest.mark.parametrize("batch,hq,hkv,window,splits", [
    (128, 28, 4, 4096, 1),      # qwen7b: 512 (rollout, KV head) rows
    (64, 16, 2, 2048, 1),       # qwen3b: 128 rows, one split from 121 rows up
    (256, 32, 8, 8192, 1),      # llama8b
    (60, 16, 2, 2048, 1),       # 120 rows: two splits would leave a wavefront 4 groups: not worth the hand-over
    (56, 16, 2, 4096, 2),       # 112 rows at twice the window: 8 groups per wavefront under two splits
    (40, 16, 2, 2048, 3),       # 80 rows
    (30, 16, 2, 2048, 4),       # 60 rows
    (16, 16, 2, 2048, 4),       # 32 rows: about 128 workgroups
    (4, 16, 2, 2048, 8),        # 8 rows: capped by 256 tokens per split
    (4, 16, 2, 512, 2),         # a short window allows two splits only
    (1, 8, 1, 8192, 32),        # one row: the maximum
    (24, 16, 2, 1024, 4),       # 48 rows: 3 splits deal 32 groups unevenly to 24 wavefronts; 4 fit the chip
    (32, 16, 2, 1024, 2),       # 64 rows: 4 splits no longer fit, and 3 are no shorter than 2
    (32, 16, 2, 2048, 3),       # 64 groups: 3 at most under 3 splits against 4 under 2: stays
    (64, 16, 2, 4096, 2),       # 128 rows fill half the chip and every wavefront keeps 8 groups
])
def test_window_split_plan_for_known_shapes(batch, hq, hkv, window, splits):
    # the measured rule of the host's plan (documented with the heuristic): a change shows up here
    st, h = _host_ctx(cfg(batch=batch, n_q_heads=hq, n_kv_heads=hkv, window=window, chunk=64))
    assert st == ptenc.OK
    assert ptenc.ptenc_get_plan(h) == (1, splits, 1)
    ptenc.ptenc_destroy(h)


def test_shapes_beyond_the_step_kernels_packed_arguments_take_the_plain_path():
    # the MFMA step kernel receives KV heads (8 bits) and W / 32 (16 bits) in one preloaded argument
    for c, kernel in ((cfg(n_q_heads=255, n_kv_heads=255), 1), (cfg(n_q_heads=256, n_kv_heads=256), 0),
                      (cfg(batch=1, n_q_heads=1, n_kv_heads=1, window=32 * 0xffff, chunk=32), 1),
                      (cfg(batch=1, n_q_heads=1, n_kv_heads=1, window=32 * 0x10000, chunk=32), 0)):
        st, h = _host_ctx(c)
        assert st == ptenc.OK
        assert ptenc.ptenc_get_plan(h)[0] == kernel
        assert ptenc.lib().ptenc_destroy(h) == ptenc.OK
