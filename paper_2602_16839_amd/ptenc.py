"""Thin ctypes binding of libptenc (same names as the C ABI in include/ptenc.h).

Argument marshalling only: torch tensors give device pointers and the current HIP stream;
every step of the decode path runs in the library's kernels.  There is no CPU fallback: if the
shared library is missing the import of this module's ``lib()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libptenc.so")

OK, ERR_INVALID_ARG, ERR_STATE, ERR_UNSUPPORTED, ERR_HIP, ERR_NOMEM, ERR_TOO_LARGE = range(7)
NOALLOC_SCRATCH_BYTES = 16 << 20
F32, BF16 = 0, 1
NORM_FROBENIUS, NORM_ROW_L2, NORM_NONE = 0, 1, 2
DEVERR_APPEND_FULL, DEVERR_ATTEND_EMPTY, DEVERR_BAD_ID = 1, 2, 4
OPT_SPLITS, OPT_FORCE_GENERIC, OPT_NONTEMPORAL, OPT_WAVES, OPT_COUNTERS_IN_PLACE = 0, 1, 2, 3, 4
OPT_EVICT_POLICY, OPT_RECENT, OPT_ENCODE_PARTS, OPT_ENCODE_INLINE = 5, 6, 7, 8
POLICY_SLIDING, POLICY_SCORED = 0, 1
MAX_SPLITS = 32

EXPORTS = [
    "ptenc_query_sizes", "ptenc_create", "ptenc_destroy", "ptenc_set_option", "ptenc_set_encoder",
    "ptenc_reset", "ptenc_cache_append", "ptenc_decode_attn", "ptenc_evict_encode", "ptenc_decode_step",
    "ptenc_decode_run", "ptenc_get_counters", "ptenc_set_counters", "ptenc_get_state", "ptenc_set_state",
    "ptenc_get_encoder_state", "ptenc_gather_window", "ptenc_cache_offset", "ptenc_poll_error",
    "ptenc_get_plan", "ptenc_status_string", "ptenc_util_stream_read", "ptenc_util_stream_read_nt", "ptenc_util_copy",
    "ptenc_prefill", "ptenc_get_prompt_len", "ptenc_decode_step_ids", "ptenc_decode_run_ids",
    "ptenc_apply_delta",
    "ptenc_get_scores", "ptenc_set_scores", "ptenc_get_victims", "ptenc_prefill_ids",
    "ptenc_stack_query_sizes", "ptenc_stack_create", "ptenc_stack_destroy", "ptenc_stack_layer",
    "ptenc_stack_reset", "ptenc_stack_decode_step", "ptenc_stack_graph_capture", "ptenc_stack_graph_launch",
    "ptenc_decode_step_noalloc",
]


class Config(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("window", C.c_int32), ("chunk", C.c_int32),
                ("n_sink", C.c_int32), ("n_global", C.c_int32), ("rank", C.c_int32),
                ("dtype", C.c_int32), ("norm_mode", C.c_int32), ("norm_eps", C.c_float),
                ("softmax_scale", C.c_float)]


class PtencError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, status_string(status), status))


_LIB = None


def lib() -> C.CDLL:
    """Loads libptenc.so (built by ``paper_2602_16839_amd.build``); raises if it is not there.
    PTENC_LIB names another build of the same library (the host-sanitized one of the host-only tests)."""
    global _LIB
    if _LIB is None:
        path = os.environ.get("PTENC_LIB") or LIB_PATH
        if not os.path.exists(path):
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2602_16839_amd.build`; there is no fallback path"
                % path)
        L = C.CDLL(path)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        P = C.POINTER
        sig = {
            "ptenc_query_sizes": [P(Config), P(sz), P(sz), P(sz)],
            "ptenc_create": [P(Config), vp, vp, vp, P(vp)],
            "ptenc_destroy": [vp],
            "ptenc_set_option": [vp, i32, i32],
            "ptenc_set_encoder": [vp, vp, vp, vp, vp, vp, vp, vp],
            "ptenc_reset": [vp, vp, vp],
            "ptenc_cache_append": [vp, vp, vp, vp, vp],
            "ptenc_decode_attn": [vp, vp, vp, vp, vp],
            "ptenc_evict_encode": [vp, vp, vp, vp],
            "ptenc_decode_step": [vp, vp, vp, vp, vp, vp, vp],
            "ptenc_decode_step_noalloc": [vp, vp, vp, vp, vp, vp, vp],
            "ptenc_decode_run": [vp, vp, vp, vp, vp, vp, i64, vp],
            "ptenc_get_counters": [vp, vp, vp, vp],
            "ptenc_set_counters": [vp, vp, vp, vp],
            "ptenc_get_state": [vp, vp, vp],
            "ptenc_set_state": [vp, vp, vp],
            "ptenc_get_encoder_state": [vp, vp, vp, vp],
            "ptenc_gather_window": [vp, vp, vp, vp],
            "ptenc_cache_offset": [vp, i32, i32, i32, i32, i32, P(sz)],
            "ptenc_poll_error": [vp, P(i32), vp],
            "ptenc_get_plan": [vp, P(i32), P(i32), P(i32)],
            "ptenc_util_stream_read": [vp, sz, vp, i32, vp],
            "ptenc_util_stream_read_nt": [vp, sz, vp, i32, vp],
            "ptenc_util_copy": [vp, vp, sz, i32, vp],
            "ptenc_prefill": [vp, vp, vp, vp, i32, vp],
            "ptenc_get_prompt_len": [vp, vp, vp],
            "ptenc_prefill_ids": [vp, vp, vp, vp, vp, i32, i32, vp],
            "ptenc_decode_step_ids": [vp, vp, vp, vp, vp, vp, i32, vp],
            "ptenc_decode_run_ids": [vp, vp, vp, vp, vp, vp, vp, i64, vp],
            "ptenc_apply_delta": [vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, vp],
            "ptenc_get_scores": [vp, vp, vp, vp],
            "ptenc_set_scores": [vp, vp, vp],
            "ptenc_get_victims": [vp, vp, vp],
            "ptenc_stack_query_sizes": [P(Config), i32, P(sz), P(sz), P(sz)],
            "ptenc_stack_create": [P(Config), i32, vp, vp, vp, P(vp)],
            "ptenc_stack_destroy": [vp],
            "ptenc_stack_layer": [vp, i32, P(vp)],
            "ptenc_stack_reset": [vp, vp, vp],
            "ptenc_stack_decode_step": [vp, P(vp), P(vp), P(vp), P(vp), vp, vp],
            "ptenc_stack_graph_capture": [vp, P(vp), P(vp), P(vp), P(vp), vp],
            "ptenc_stack_graph_launch": [vp, vp],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int
        L.ptenc_status_string.argtypes = [C.c_int]
        L.ptenc_status_string.restype = C.c_char_p
        _LIB = L
    return _LIB


def status_string(status: int) -> str:
    return lib().ptenc_status_string(status).decode()


def _check(status: int, what: str) -> None:
    if status != OK:
        raise PtencError(status, what)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor expected"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


# ---- functions with the C ABI's names -------------------------------------------------------

def ptenc_query_sizes(cfg: Config):
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().ptenc_query_sizes(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c)), "ptenc_query_sizes")
    return a.value, b.value, c.value


def ptenc_create(cfg: Config, d_cache, d_state, d_scratch):
    h = C.c_void_p()
    _check(lib().ptenc_create(C.byref(cfg), _ptr(d_cache), _ptr(d_state), _ptr(d_scratch), C.byref(h)), "ptenc_create")
    return h


def ptenc_destroy(ctx):
    _check(lib().ptenc_destroy(ctx), "ptenc_destroy")


def ptenc_set_option(ctx, option: int, value: int):
    _check(lib().ptenc_set_option(ctx, option, value), "ptenc_set_option")


def ptenc_set_encoder(ctx, q_g, WaQ, WaK, WaV, k_g=None, v_g=None):
    _check(lib().ptenc_set_encoder(ctx, _ptr(q_g), _ptr(WaQ), _ptr(WaK), _ptr(WaV), _ptr(k_g), _ptr(v_g), _stream()),
           "ptenc_set_encoder")


def ptenc_reset(ctx, mask=None):
    _check(lib().ptenc_reset(ctx, _ptr(mask), _stream()), "ptenc_reset")


def ptenc_prefill(ctx, k, v, prompt_len):
    """k, v: [B, p_max, H_kv, d] device tensors; prompt_len: B host integers."""
    pl = np.ascontiguousarray(prompt_len, dtype=np.int32)
    _check(lib().ptenc_prefill(ctx, _ptr(k), _ptr(v), pl.ctypes.data_as(C.c_void_p), int(k.shape[1]), _stream()),
           "ptenc_prefill")


def ptenc_prefill_ids(ctx, k, v, ids, prompt_len):
    """k, v: [n, p_max, H_kv, d] device tensors; ids: int32 [n] device tensor; prompt_len: n host integers."""
    assert ids.dtype == torch.int32
    pl = np.ascontiguousarray(prompt_len, dtype=np.int32)
    assert len(pl) == ids.numel()
    _check(lib().ptenc_prefill_ids(ctx, _ptr(k), _ptr(v), _ptr(ids), pl.ctypes.data_as(C.c_void_p), int(ids.numel()),
                                   int(k.shape[1]) if k is not None and k.dim() > 1 else 1, _stream()), "ptenc_prefill_ids")


def ptenc_get_prompt_len(ctx, batch: int):
    pl = np.zeros(batch, dtype=np.int32)
    _check(lib().ptenc_get_prompt_len(ctx, pl.ctypes.data_as(C.c_void_p), _stream()), "ptenc_get_prompt_len")
    return pl


def ptenc_cache_append(ctx, k, v, active=None):
    _check(lib().ptenc_cache_append(ctx, _ptr(k), _ptr(v), _ptr(active), _stream()), "ptenc_cache_append")


def ptenc_decode_attn(ctx, q, out, active=None):
    _check(lib().ptenc_decode_attn(ctx, _ptr(q), _ptr(out), _ptr(active), _stream()), "ptenc_decode_attn")


def ptenc_evict_encode(ctx, active=None, dbg_chunk=None):
    _check(lib().ptenc_evict_encode(ctx, _ptr(active), _ptr(dbg_chunk), _stream()), "ptenc_evict_encode")


def ptenc_decode_step(ctx, q, k, v, out, active=None):
    _check(lib().ptenc_decode_step(ctx, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(active), _stream()),
           "ptenc_decode_step")


def ptenc_decode_step_noalloc(ctx, q, k, v, out, active=None):
    _check(lib().ptenc_decode_step_noalloc(ctx, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(active), _stream()),
           "ptenc_decode_step_noalloc")


def ptenc_decode_run(ctx, q, k, v, out, active, n_steps: int):
    _check(lib().ptenc_decode_run(ctx, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(active), n_steps, _stream()),
           "ptenc_decode_run")


def ptenc_decode_step_ids(ctx, q, k, v, out, ids):
    """q, out [n, H_q, d]; k, v [n, H_kv, d]; ids int32 [n] device tensor of distinct rollout indices."""
    assert ids.dtype == torch.int32
    _check(lib().ptenc_decode_step_ids(ctx, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(ids), int(ids.numel()), _stream()),
           "ptenc_decode_step_ids")


def ptenc_decode_run_ids(ctx, q, k, v, out, ids, row_offsets):
    """Concatenated compact buffers; row_offsets: host int64 [n_steps + 1]."""
    assert ids.dtype == torch.int32
    ro = np.ascontiguousarray(row_offsets, dtype=np.int64)
    _check(lib().ptenc_decode_run_ids(ctx, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(ids),
                                      ro.ctypes.data_as(C.c_void_p), len(ro) - 1, _stream()), "ptenc_decode_run_ids")


def ptenc_apply_delta(ctx, x, At, Bt, y, active=None, ids=None):
    """y += ((x A) S) B in place; At = A^T [G, d_in], Bt = B^T [d_out, r]."""
    n = 0 if ids is None else int(ids.numel())
    _check(lib().ptenc_apply_delta(ctx, _ptr(x), _ptr(At), _ptr(Bt), _ptr(y), int(x.shape[-1]), int(y.shape[-1]),
                                   _ptr(active), _ptr(ids), n, _stream()), "ptenc_apply_delta")


def ptenc_get_counters(ctx, batch: int):
    ln = np.zeros(batch, dtype=np.int64)
    base = np.zeros(batch, dtype=np.int64)
    _check(lib().ptenc_get_counters(ctx, ln.ctypes.data_as(C.c_void_p), base.ctypes.data_as(C.c_void_p), _stream()),
           "ptenc_get_counters")
    return ln, base


def ptenc_set_counters(ctx, ln, base):
    ln = np.ascontiguousarray(ln, dtype=np.int64)
    base = np.ascontiguousarray(base, dtype=np.int64)
    _check(lib().ptenc_set_counters(ctx, ln.ctypes.data_as(C.c_void_p), base.ctypes.data_as(C.c_void_p), _stream()),
           "ptenc_set_counters")


def ptenc_get_state(ctx, batch: int, G: int, r: int):
    S = np.zeros((batch, G, r), dtype=np.float32)
    _check(lib().ptenc_get_state(ctx, S.ctypes.data_as(C.c_void_p), _stream()), "ptenc_get_state")
    return S


def ptenc_set_state(ctx, S):
    S = np.ascontiguousarray(S, dtype=np.float32)
    _check(lib().ptenc_set_state(ctx, S.ctypes.data_as(C.c_void_p), _stream()), "ptenc_set_state")


def ptenc_get_encoder_state(ctx, G: int, r: int):
    Qa = np.zeros((G, r), dtype=np.float32)
    S0 = np.zeros((G, r), dtype=np.float32)
    _check(lib().ptenc_get_encoder_state(ctx, Qa.ctypes.data_as(C.c_void_p), S0.ctypes.data_as(C.c_void_p), _stream()),
           "ptenc_get_encoder_state")
    return Qa, S0


def ptenc_gather_window(ctx, K, V):
    _check(lib().ptenc_gather_window(ctx, _ptr(K), _ptr(V), _stream()), "ptenc_gather_window")


def ptenc_cache_offset(ctx, b: int, h: int, slot: int, i: int, which: int) -> int:
    off = C.c_size_t()
    _check(lib().ptenc_cache_offset(ctx, b, h, slot, i, which, C.byref(off)), "ptenc_cache_offset")
    return off.value


def ptenc_poll_error(ctx) -> int:
    f = C.c_int32()
    _check(lib().ptenc_poll_error(ctx, C.byref(f), _stream()), "ptenc_poll_error")
    return f.value


def ptenc_get_plan(ctx):
    a, s, e = C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().ptenc_get_plan(ctx, C.byref(a), C.byref(s), C.byref(e)), "ptenc_get_plan")
    return a.value, s.value, e.value


def ptenc_util_stream_read(src, nbytes: int, sink, n_blocks: int):
    _check(lib().ptenc_util_stream_read(_ptr(src), nbytes, _ptr(sink), n_blocks, _stream()), "ptenc_util_stream_read")


def ptenc_util_stream_read_nt(src, nbytes: int, sink, n_blocks: int):
    _check(lib().ptenc_util_stream_read_nt(_ptr(src), nbytes, _ptr(sink), n_blocks, _stream()), "ptenc_util_stream_read_nt")


def ptenc_util_copy(dst, src, nbytes: int, n_blocks: int):
    _check(lib().ptenc_util_copy(_ptr(dst), _ptr(src), nbytes, n_blocks, _stream()), "ptenc_util_copy")


def ptenc_get_scores(ctx, score, pos):
    """score float32 [B, W], pos int64 [B, W] device tensors (either may be None)."""
    _check(lib().ptenc_get_scores(ctx, _ptr(score), _ptr(pos), _stream()), "ptenc_get_scores")


def ptenc_set_scores(ctx, score):
    assert score.dtype == torch.float32
    _check(lib().ptenc_set_scores(ctx, _ptr(score), _stream()), "ptenc_set_scores")


def ptenc_get_victims(ctx, batch: int, chunk: int):
    pos = np.zeros((batch, chunk), dtype=np.int64)
    _check(lib().ptenc_get_victims(ctx, pos.ctypes.data_as(C.c_void_p), _stream()), "ptenc_get_victims")
    return pos


def ptenc_stack_query_sizes(cfg: Config, n_layers: int):
    a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().ptenc_stack_query_sizes(C.byref(cfg), n_layers, C.byref(a), C.byref(b), C.byref(c)),
           "ptenc_stack_query_sizes")
    return a.value, b.value, c.value


def ptenc_stack_create(cfg: Config, n_layers: int, d_cache, d_state, d_scratch):
    h = C.c_void_p()
    _check(lib().ptenc_stack_create(C.byref(cfg), n_layers, _ptr(d_cache), _ptr(d_state), _ptr(d_scratch), C.byref(h)),
           "ptenc_stack_create")
    return h


def ptenc_stack_destroy(stack):
    _check(lib().ptenc_stack_destroy(stack), "ptenc_stack_destroy")


def ptenc_stack_layer(stack, layer: int):
    h = C.c_void_p()
    _check(lib().ptenc_stack_layer(stack, layer, C.byref(h)), "ptenc_stack_layer")
    return h


def ptenc_stack_reset(stack, mask=None):
    _check(lib().ptenc_stack_reset(stack, _ptr(mask), _stream()), "ptenc_stack_reset")


def _ptr_array(tensors):
    """Host array of device pointers, one per layer."""
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t)
    return arr


def ptenc_stack_decode_step(stack, q, k, v, out, active=None):
    """q, k, v, out: sequences of L per-layer device tensors."""
    _check(lib().ptenc_stack_decode_step(stack, _ptr_array(q), _ptr_array(k), _ptr_array(v), _ptr_array(out),
                                         _ptr(active), _stream()), "ptenc_stack_decode_step")


def ptenc_stack_graph_capture(stack, q, k, v, out, active=None):
    _check(lib().ptenc_stack_graph_capture(stack, _ptr_array(q), _ptr_array(k), _ptr_array(v), _ptr_array(out),
                                           _ptr(active)), "ptenc_stack_graph_capture")


def ptenc_stack_graph_launch(stack):
    _check(lib().ptenc_stack_graph_launch(stack, _stream()), "ptenc_stack_graph_launch")


# ---- convenience owner of the device buffers (plumbing only) ---------------------------------

class Layer:
    """Allocates the cache / state / scratch tensors for one context and forwards to the C ABI."""

    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, window, chunk, dtype=torch.bfloat16,
                 n_global=32, rank=32, norm_mode=NORM_FROBENIUS, norm_eps=0.0, softmax_scale=0.0,
                 device="cuda:0", poison_cache=False, n_sink=0):
        self.cfg = Config(batch, n_q_heads, n_kv_heads, head_dim, window, chunk, n_sink, n_global, rank,
                          F32 if dtype == torch.float32 else BF16, norm_mode, norm_eps, softmax_scale)
        self.dtype, self.device = dtype, torch.device(device)
        cb, sb, xb = ptenc_query_sizes(self.cfg)
        self.cache = torch.empty(cb, dtype=torch.uint8, device=self.device)
        if poison_cache:
            self.cache.fill_(0xFF)      # every bf16 / fp32 element reads as NaN
        self.state = torch.zeros(sb, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(xb, dtype=torch.uint8, device=self.device)
        self.ctx = ptenc_create(self.cfg, self.cache, self.state, self.scratch)
        self._enc = None
        self._owns_ctx = True

    @classmethod
    def _borrowed(cls, cfg, dtype, device, ctx, keep_alive):
        """A layer of a Stack: same methods, context and buffers owned by the stack."""
        self = cls.__new__(cls)
        self.cfg, self.dtype, self.device, self.ctx = cfg, dtype, device, ctx
        self.cache = self.state = self.scratch = None
        self._enc, self._owns_ctx, self._stack = None, False, keep_alive
        return self

    def close(self):
        if self.ctx is not None and self._owns_ctx:
            ptenc_destroy(self.ctx)
        self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def B(self):
        return self.cfg.batch

    def set_encoder(self, q_g, WaQ, WaK, WaV, k_g=None, v_g=None):
        self._enc = (q_g, WaQ, WaK, WaV, k_g, v_g)       # keep the borrowed tensors alive
        ptenc_set_encoder(self.ctx, q_g, WaQ, WaK, WaV, k_g, v_g)

    def reset(self, mask=None):
        ptenc_reset(self.ctx, mask)

    def prefill(self, k, v, prompt_len):
        ptenc_prefill(self.ctx, k, v, prompt_len)

    def prefill_ids(self, k, v, ids, prompt_len):
        ptenc_prefill_ids(self.ctx, k, v, ids, prompt_len)

    def prompt_len(self):
        return ptenc_get_prompt_len(self.ctx, self.B)

    def append(self, k, v, active=None):
        ptenc_cache_append(self.ctx, k, v, active)

    def attend(self, q, out=None, active=None):
        if out is None:
            out = torch.empty_like(q)
        ptenc_decode_attn(self.ctx, q, out, active)
        return out

    def evict_encode(self, active=None, dbg_chunk=None):
        ptenc_evict_encode(self.ctx, active, dbg_chunk)

    def step(self, q, k, v, out=None, active=None):
        if out is None:
            out = torch.empty_like(q)
        ptenc_decode_step(self.ctx, q, k, v, out, active)
        return out

    def step_noalloc(self, q, k, v, out, active=None):
        """One decode step through the library's built-in scratch block; `out` is the caller's (nothing is allocated)."""
        ptenc_decode_step_noalloc(self.ctx, q, k, v, out, active)
        return out

    def step_ids(self, q, k, v, ids, out=None):
        if out is None:
            out = torch.empty_like(q)
        ptenc_decode_step_ids(self.ctx, q, k, v, out, ids)
        return out

    def run_ids(self, q, k, v, ids, row_offsets, out=None):
        if out is None:
            out = torch.empty_like(q)
        ptenc_decode_run_ids(self.ctx, q, k, v, out, ids, row_offsets)
        return out

    def apply_delta(self, x, At, Bt, y, active=None, ids=None):
        ptenc_apply_delta(self.ctx, x, At, Bt, y, active, ids)
        return y

    def run(self, q, k, v, out=None, active=None):
        if out is None:
            out = torch.empty_like(q)
        ptenc_decode_run(self.ctx, q, k, v, out, active, q.shape[0])
        return out

    def prepared_run(self, q, k, v, out, active=None):
        """The same call with its arguments marshalled now: returns a function that only makes the C call
        (on the stream that is current now), for callers that time the call."""
        args = (self.ctx, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(active), int(q.shape[0]), _stream())
        fn, keep = lib().ptenc_decode_run, (q, k, v, out, active)

        def go():
            _check(fn(*args), "ptenc_decode_run")
            return keep[3]
        return go

    def prepared_run_ids(self, q, k, v, ids, row_offsets, out):
        """ptenc_decode_run_ids with its arguments marshalled now (see prepared_run)."""
        assert ids.dtype == torch.int32
        ro = np.ascontiguousarray(row_offsets, dtype=np.int64)
        args = (self.ctx, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(ids), ro.ctypes.data_as(C.c_void_p), len(ro) - 1,
                _stream())
        fn, keep = lib().ptenc_decode_run_ids, (q, k, v, out, ids, ro)

        def go():
            _check(fn(*args), "ptenc_decode_run_ids")
            return keep[3]
        return go

    def counters(self):
        return ptenc_get_counters(self.ctx, self.B)

    def set_counters(self, ln, base):
        ptenc_set_counters(self.ctx, ln, base)

    def get_state(self):
        return ptenc_get_state(self.ctx, self.B, self.cfg.n_global, self.cfg.rank)

    def set_state(self, S):
        ptenc_set_state(self.ctx, S)

    def encoder_state(self):
        return ptenc_get_encoder_state(self.ctx, self.cfg.n_global, self.cfg.rank)

    def gather_window(self):
        shape = (self.B, self.cfg.n_kv_heads, self.cfg.window, self.cfg.head_dim)
        K = torch.empty(shape, dtype=self.dtype, device=self.device)
        V = torch.empty(shape, dtype=self.dtype, device=self.device)
        ptenc_gather_window(self.ctx, K, V)
        return K, V

    def cache_view(self):
        """The raw cache as a flat tensor of the element dtype (for poisoning tests)."""
        return self.cache.view(self.dtype)

    def cache_offset(self, b, h, slot, i, which):
        return ptenc_cache_offset(self.ctx, b, h, slot, i, which)

    def poll_error(self):
        return ptenc_poll_error(self.ctx)

    def plan(self):
        return ptenc_get_plan(self.ctx)

    def set_option(self, option, value):
        ptenc_set_option(self.ctx, option, value)

    def scores(self):
        """(scores float32 [B, W], positions int64 [B, W]) of the live ring entries, ring order, on the host."""
        sc = torch.empty((self.B, self.cfg.window), dtype=torch.float32, device=self.device)
        ps = torch.empty((self.B, self.cfg.window), dtype=torch.int64, device=self.device)
        ptenc_get_scores(self.ctx, sc, ps)
        return sc.cpu().numpy(), ps.cpu().numpy()

    def set_scores(self, scores):
        sc = torch.as_tensor(np.ascontiguousarray(scores, dtype=np.float32)).to(self.device)
        assert tuple(sc.shape) == (self.B, self.cfg.window)
        ptenc_set_scores(self.ctx, sc)
        torch.cuda.current_stream().synchronize()

    def victims(self):
        return ptenc_get_victims(self.ctx, self.B, self.cfg.chunk)


class Stack:
    """L layers over one cache / state allocation and one shared scratch buffer; forwards to the
    ptenc_stack_* calls.  ``layers[l]`` is a Layer view of layer l (encoder, prefill, read-back)."""

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, window, chunk, dtype=torch.bfloat16,
                 n_global=32, rank=32, norm_mode=NORM_FROBENIUS, norm_eps=0.0, softmax_scale=0.0,
                 device="cuda:0", poison_cache=False, n_sink=0):
        self.cfg = Config(batch, n_q_heads, n_kv_heads, head_dim, window, chunk, n_sink, n_global, rank,
                          F32 if dtype == torch.float32 else BF16, norm_mode, norm_eps, softmax_scale)
        self.dtype, self.device, self.n_layers = dtype, torch.device(device), n_layers
        cb, sb, xb = ptenc_stack_query_sizes(self.cfg, n_layers)
        self.cache = torch.empty(cb, dtype=torch.uint8, device=self.device)
        if poison_cache:
            self.cache.fill_(0xFF)
        self.state = torch.zeros(sb, dtype=torch.uint8, device=self.device)
        self.scratch = torch.empty(xb, dtype=torch.uint8, device=self.device)
        self.stack = ptenc_stack_create(self.cfg, n_layers, self.cache, self.state, self.scratch)
        self.layers = [Layer._borrowed(self.cfg, dtype, self.device, ptenc_stack_layer(self.stack, l), self)
                       for l in range(n_layers)]
        self._graph_bufs = None

    def close(self):
        if self.stack is not None:
            for layer in self.layers:
                layer.ctx = None
            ptenc_stack_destroy(self.stack)
            self.stack = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self, mask=None):
        ptenc_stack_reset(self.stack, mask)

    def step(self, q, k, v, out=None, active=None):
        if out is None:
            out = [torch.empty_like(x) for x in q]
        ptenc_stack_decode_step(self.stack, q, k, v, out, active)
        return out

    def graph_capture(self, q, k, v, out, active=None):
        self._graph_bufs = (list(q), list(k), list(v), list(out), active)    # frozen into the graph: keep alive
        ptenc_stack_graph_capture(self.stack, q, k, v, out, active)

    def graph_launch(self):
        ptenc_stack_graph_launch(self.stack)
