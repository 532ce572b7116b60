"""Seeded synthetic inputs for the bounded-cache rollout decode path.

This module holds *no* arithmetic of the method (no attention, no eviction, no
encoding): it only produces reproducible tensors and workload descriptions.  It
serves the HIP path, the CPU oracle's tests and the benchmark alike, so both
sides see bit-identical inputs.

Every value is a pure function of (seed, stream, t, b, head, i):

    value = scale * head_scale[head] * QTAB[ mix64(counter ^ mix64(stream_key)) & 0xFFFF ]

* ``counter`` is the row-major index of the element in a ``[T, B, H, d]`` tensor.
* ``mix64`` is the splitmix64 output mix (Steele, Lea & Flood 2014), a bijection
  on 64-bit integers built from xor-shifts and two odd multiplications.
* ``QTAB`` is a 65 536-entry fp32 table of standard-normal quantiles
  ``Phi^-1((n + 0.5) / 65536)`` built once on the host in fp64.
* The product is evaluated in fp32 and, for bf16 workloads, rounded to nearest
  even.

Only integer operations and one table lookup run on the device, so the CPU and
the GPU generator agree bit for bit, and any single rollout's history can be
rebuilt on the host without storing the whole run.

The workloads stand in for the paper's RL rollouts (Experimental Setup section:
real models on a public math training set, which are not available here): the
attention shapes are those of the paper's three model families, the values are
Gaussian with the scale of normalised activations.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Tuple

import numpy as np
import torch

MASK64 = (1 << 64) - 1
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_GOLDEN = 0x9E3779B97F4A7C15

STREAM_Q, STREAM_K, STREAM_V = 0, 1, 2
STREAM_QG, STREAM_KG, STREAM_VG = 3, 4, 5
STREAM_WAQ, STREAM_WAK, STREAM_WAV = 6, 7, 8
STREAM_HEAD_SCALE_Q, STREAM_HEAD_SCALE_K, STREAM_HEAD_SCALE_V = 9, 10, 11
STREAM_PROMPT_K, STREAM_PROMPT_V, STREAM_PROMPT_LEN = 12, 13, 14
STREAM_ADAPT_A, STREAM_ADAPT_B, STREAM_ADAPT_X, STREAM_ADAPT_Y = 15, 16, 17, 18


def _signed(x: int) -> int:
    x &= MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def mix64_int(x: int) -> int:
    """splitmix64 output mix on a Python integer (the definition the tensor version is tested against)."""
    x &= MASK64
    x ^= x >> 30
    x = (x * _C1) & MASK64
    x ^= x >> 27
    x = (x * _C2) & MASK64
    x ^= x >> 31
    return x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    # logical shift right of a two's-complement int64 tensor
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output mix on an int64 tensor (bit pattern = unsigned 64-bit value)."""
    x = x ^ _lsr(x, 30)
    x = x * _signed(_C1)
    x = x ^ _lsr(x, 27)
    x = x * _signed(_C2)
    x = x ^ _lsr(x, 31)
    return x


def stream_key(seed: int, stream: int) -> int:
    return mix64_int((seed * 16 + stream + 1) * _GOLDEN)


_QTAB_CACHE = {}


def normal_table(device="cpu") -> torch.Tensor:
    """fp32 table of 65 536 standard-normal quantiles, built in fp64 on the host."""
    key = str(device)
    if key not in _QTAB_CACHE:
        from scipy.special import ndtri

        n = np.arange(65536, dtype=np.float64)
        tab = ndtri((n + 0.5) / 65536.0).astype(np.float32)
        _QTAB_CACHE[key] = torch.from_numpy(tab).to(device)
    return _QTAB_CACHE[key]


def uniform01_int(seed: int, stream: int, index: int) -> float:
    """A uniform in [0,1) with 24 bits, from the same hash (host only)."""
    h = mix64_int(index ^ stream_key(seed, stream))
    return ((h >> 16) & 0xFFFFFF) / float(1 << 24)


def gaussian(seed: int, stream: int, t0: int, t1: int, B: int, H: int, d: int, scale: float,
             head_scale: Optional[torch.Tensor] = None, dtype=torch.float32, device="cpu",
             b0: int = 0, b1: Optional[int] = None, B_total: Optional[int] = None) -> torch.Tensor:
    """Elements [t0:t1, b0:b1, :, :] of the virtual ``[T, B_total, H, d]`` tensor of a stream.

    ``head_scale`` (fp32, ``[H]``) multiplies each head; ``scale`` multiplies everything.
    The result has shape ``[t1-t0, b1-b0, H, d]`` and dtype ``dtype``.
    """
    B_total = B if B_total is None else B_total
    b1 = B if b1 is None else b1
    dev = torch.device(device)
    t = torch.arange(t0, t1, dtype=torch.int64, device=dev).view(-1, 1, 1, 1)
    b = torch.arange(b0, b1, dtype=torch.int64, device=dev).view(1, -1, 1, 1)
    h = torch.arange(H, dtype=torch.int64, device=dev).view(1, 1, -1, 1)
    i = torch.arange(d, dtype=torch.int64, device=dev).view(1, 1, 1, -1)
    counter = ((t * B_total + b) * H + h) * d + i
    bits = mix64(counter ^ _signed(stream_key(seed, stream))) & 0xFFFF
    z = normal_table(dev)[bits]
    s = torch.full((1, 1, H, 1), float(np.float32(scale)), dtype=torch.float32, device=dev)
    if head_scale is not None:
        s = s * head_scale.to(device=dev, dtype=torch.float32).view(1, 1, H, 1)
    return (z * s).to(dtype)


def head_scales(seed: int, stream: int, H: int, lo: float, hi: float) -> torch.Tensor:
    """One fp32 scale per head, uniform in [lo, hi), drawn once per (seed, stream)."""
    u = [uniform01_int(seed, stream, h) for h in range(H)]
    return torch.tensor([lo + (hi - lo) * x for x in u], dtype=torch.float32)


@dataclasses.dataclass(frozen=True)
class Workload:
    """One decode workload: a single attention layer's shapes plus the run recipe."""

    name: str
    dtype: str            # "f32" | "bf16"
    batch: int            # B rollouts
    n_q_heads: int        # H_q
    n_kv_heads: int       # H_kv
    head_dim: int         # d
    window: int           # W ring slots
    chunk: int            # C tokens evicted at once
    steps: int            # T decode steps (for ragged runs: the cap on the per-rollout length)
    scale: float          # std of q/k/v before the per-head factor
    seed: int
    per_head_scale: bool = False   # per-head factor U(0.5, 1.5), independent for q, k and v heads
    ragged: bool = False           # per-rollout length lognormal(median 3000, sigma 0.8), capped at `steps`
    n_sink: int = 0                # cache slots reserved for question tokens (kept for good); part of `window`
    n_global: int = 32             # G global tokens (paper, Experimental Setup: 32 global tokens)
    rank: int = 32                 # r latent width (paper, Experimental Setup: LoRA rank 32)
    q_gain: float = 1.0            # extra factor on the queries only (a power of two keeps bf16 values exact):
                                   # > 1 spreads the scores so that a few keys carry most of the attention

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def d_q(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


WORKLOADS = {
    # the five benchmark configurations, in the order the baseline lists them
    "tiny_f32": Workload("tiny_f32", "f32", 4, 4, 1, 64, 256, 32, 512, 1.0 / 8.0, 1001),
    "qwen3b": Workload("qwen3b", "bf16", 64, 16, 2, 128, 2048, 64, 4096, 0.088, 1002),
    "qwen7b": Workload("qwen7b", "bf16", 128, 28, 4, 128, 4096, 128, 8192, 0.088, 1003, per_head_scale=True),
    "llama8b": Workload("llama8b", "bf16", 256, 32, 8, 128, 8192, 256, 16384, 0.088, 1004),
    "ragged": Workload("ragged", "bf16", 512, 16, 2, 128, 1024, 64, 16384, 0.088, 1005, ragged=True),
    # the qwen7b shape with 512 slots reserved for question tokens in front of the same 4096-token window
    "qwen7b_sink": Workload("qwen7b_sink", "bf16", 128, 28, 4, 128, 4096 + 512, 128, 8192, 0.088, 1006,
                            per_head_scale=True, n_sink=512),
}
# The benchmark's input scale (0.088) makes every score about N(0, 0.008^2): the softmax weights are
# uniform to within a per cent and the output is close to the plain mean of the values, whatever the
# queries are.  The "peaked" twins keep the shapes and take values of std 0.25 with queries 64 times
# larger, so the scores are about N(0, 4^2): a handful of keys carry the attention, the running
# maximum keeps moving, and an implementation that gets the scores, the exponentials or the rescaling
# wrong cannot hide behind the mean.  Used by the parity tests at full size.
for _name in ("qwen3b", "qwen7b", "llama8b"):
    _w = WORKLOADS[_name]
    WORKLOADS[_name + "_peaked"] = dataclasses.replace(_w, name=_name + "_peaked", scale=0.25, q_gain=64.0,
                                                       seed=_w.seed + 100)


def qkv_head_scales(wl: Workload) -> Tuple[Optional[torch.Tensor], Optional[torch.Tensor], Optional[torch.Tensor]]:
    if not wl.per_head_scale:
        return None, None, None
    return (head_scales(wl.seed, STREAM_HEAD_SCALE_Q, wl.n_q_heads, 0.5, 1.5),
            head_scales(wl.seed, STREAM_HEAD_SCALE_K, wl.n_kv_heads, 0.5, 1.5),
            head_scales(wl.seed, STREAM_HEAD_SCALE_V, wl.n_kv_heads, 0.5, 1.5))


def qkv_steps(wl: Workload, t0: int, t1: int, device="cpu", b0: int = 0, b1: Optional[int] = None):
    """q ``[t1-t0, b, H_q, d]``, k and v ``[t1-t0, b, H_kv, d]`` for decode steps t0..t1-1 (0-based)."""
    sq, sk, sv = qkv_head_scales(wl)
    kw = dict(dtype=wl.torch_dtype, device=device, b0=b0, b1=b1, B_total=wl.batch)
    q = gaussian(wl.seed, STREAM_Q, t0, t1, wl.batch, wl.n_q_heads, wl.head_dim, wl.scale * wl.q_gain, sq, **kw)
    k = gaussian(wl.seed, STREAM_K, t0, t1, wl.batch, wl.n_kv_heads, wl.head_dim, wl.scale, sk, **kw)
    v = gaussian(wl.seed, STREAM_V, t0, t1, wl.batch, wl.n_kv_heads, wl.head_dim, wl.scale, sv, **kw)
    return q, k, v


def encoder_params(wl: Workload, device="cpu", with_global_kv: bool = True):
    """Synthetic encoder parameters of the workload's dtype.

    Returns dict with q_g ``[G, d_q]``, WaQ ``[d_q, r]``, WaK ``[d_kv, r]``, WaV ``[d_kv, r]`` and,
    unless ``with_global_kv`` is false, k_g and v_g ``[G, d_kv]``.  Projections have std
    1/sqrt(fan_in); global tokens have the workload's activation scale.
    """
    G, r, dt = wl.n_global, wl.rank, wl.torch_dtype

    def g2(stream, rows, cols, scale):
        return gaussian(wl.seed, stream, 0, 1, 1, rows, cols, scale, dtype=dt, device=device).view(rows, cols)

    p = {
        "q_g": g2(STREAM_QG, G, wl.d_q, wl.scale),
        "WaQ": g2(STREAM_WAQ, wl.d_q, r, 1.0 / math.sqrt(wl.d_q)),
        "WaK": g2(STREAM_WAK, wl.d_kv, r, 1.0 / math.sqrt(wl.d_kv)),
        "WaV": g2(STREAM_WAV, wl.d_kv, r, 1.0 / math.sqrt(wl.d_kv)),
    }
    if with_global_kv:
        p["k_g"] = g2(STREAM_KG, G, wl.d_kv, wl.scale)
        p["v_g"] = g2(STREAM_VG, G, wl.d_kv, wl.scale)
    return p


def prompt_lengths(wl: Workload) -> np.ndarray:
    """Question length per rollout (int32 ``[B]``), uniform in [n_sink/4, n_sink], seeded; zeros without a sink."""
    if wl.n_sink == 0:
        return np.zeros(wl.batch, dtype=np.int32)
    lo = max(1, wl.n_sink // 4)
    u = np.array([uniform01_int(wl.seed, STREAM_PROMPT_LEN, b) for b in range(wl.batch)])
    return np.minimum(lo + np.floor(u * (wl.n_sink - lo + 1)), wl.n_sink).astype(np.int32)


def prompt_kv(wl: Workload, device="cpu"):
    """Question keys and values ``[B, n_sink, H_kv, d]`` (rows beyond a rollout's length are simply unused)."""
    sq, sk, sv = qkv_head_scales(wl)
    kw = dict(dtype=wl.torch_dtype, device=device)
    k = gaussian(wl.seed, STREAM_PROMPT_K, 0, wl.batch, wl.n_sink, wl.n_kv_heads, wl.head_dim, wl.scale, sk, **kw)
    v = gaussian(wl.seed, STREAM_PROMPT_V, 0, wl.batch, wl.n_sink, wl.n_kv_heads, wl.head_dim, wl.scale, sv, **kw)
    return k, v


def adapter_inputs(wl: Workload, d_in: int, d_out: int, device="cpu"):
    """Inputs of the weight-delta application: x [B, d_in], y [B, d_out] activations of unit scale, and the
    maps A^T [G, d_in], B^T [d_out, r] with std 1/sqrt(fan_in) (A maps d_in -> G, B maps r -> d_out)."""
    dt = wl.torch_dtype

    def g2(stream, rows, cols, scale):
        return gaussian(wl.seed, stream, 0, 1, 1, rows, cols, scale, dtype=dt, device=device).view(rows, cols)

    return {
        "x": g2(STREAM_ADAPT_X, wl.batch, d_in, 1.0), "y": g2(STREAM_ADAPT_Y, wl.batch, d_out, 1.0),
        "At": g2(STREAM_ADAPT_A, wl.n_global, d_in, 1.0 / math.sqrt(d_in)),
        "Bt": g2(STREAM_ADAPT_B, d_out, wl.rank, 1.0 / math.sqrt(wl.rank)),
    }


def rollout_lengths(wl: Workload) -> np.ndarray:
    """Per-rollout generation length (int64 ``[B]``).

    Fixed-length workloads return ``steps`` for every rollout.  Ragged ones draw
    ``min(round(exp(N(ln 3000, 0.8^2))), steps)`` (at least 1) from a seeded host generator.
    """
    if not wl.ragged:
        return np.full(wl.batch, wl.steps, dtype=np.int64)
    rng = np.random.default_rng(wl.seed)
    L = np.rint(np.exp(rng.normal(math.log(3000.0), 0.8, size=wl.batch))).astype(np.int64)
    return np.clip(L, 1, wl.steps)


def active_mask(lengths: np.ndarray, t: int) -> np.ndarray:
    """uint8 ``[B]``: rollout b takes decode step t (0-based) iff t < lengths[b]."""
    return (t < lengths).astype(np.uint8)
