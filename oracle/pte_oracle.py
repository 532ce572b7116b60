"""CPU fp64 oracle for the bounded-cache rollout decode step of Progressive Thought Encoding.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP library is checked
against.  It may be imported by the tests, by the smoke check and by the benchmark's
``cpu_baseline`` leg, and by nothing else; it shares no code with the HIP path and imports
nothing from it.  Everything is numpy float64; the window is a Python list in logical order
(oldest first) -- there is no ring buffer and no modulo anywhere in here.

What follows the paper, and where:

* ``attend``            -- o = softmax(q K^T / sqrt(d)) V over the cached keys, the query's own key
                           included (Notation and Preliminaries: the attention equation and the
                           decode-step equation that extends the cache by k_{t+1}, v_{t+1} first).
* ``encode_chunk``      -- S' = ((q_g W^a_Q)(K_e W^a_K)^T)(V_e W^a_V), linear (no softmax, no scale)
                           (Our Approach, the Delta-W equation: the under-braced term S_e).
* ``init_state``        -- S_0 = the same contraction with the global tokens' (k_g, v_g) as the chunk
                           (Our Approach, paragraph on bootstrapping with global tokens).
* ``normalize``         -- S <- Normalize(S + S') (Our Approach, the update rule).  The paper does not
                           define Normalize; the readings are listed below.  PARITY UNPINNED against
                           the authors' intent for the choice of norm.
* ``OracleLayer.step``  -- decode until the cache is full, then evict the oldest chunk (sliding window
                           over thinking tokens; Our Approach, first paragraph and "The selection of D
                           during training") and fold it into S before decoding continues.
* ``apply_delta``       -- the context state used as a weight delta: Delta-W = A S B, theta' = theta + Delta-W
                           (Our Approach, the Delta-W equation and the sentence after the update rule),
                           applied to one token's activations: y + ((x A) S) B.
* ``OracleLayer.prefill`` -- question tokens are kept in the cache permanently and only thinking tokens
                           slide ("The selection of D during training"; the response-length analysis
                           quotes a cache of 768 = 512 sink tokens + 256 in the sliding window).

Readings taken where the paper is silent or inconsistent (same list as the design notes):

1. The Delta-W equation prints W^a_K in front of V_e and the symbol list names W^a_Q twice; the
   initialisation formula uses W^a_V for v_g, so V_e is mapped by W^a_V and K_e by W^a_K.
2. Tokens are rows: q_g is G x d_q, K_e and V_e are C x d_kv, projections multiply on the right,
   S is G x r.
3. The encoding is taken literally: no softmax, no 1/sqrt(d).
4. Eviction is lazy: a chunk leaves at the start of the step whose append would overflow the window.
5. The query attends to its own key (append before attend).
6. With grouped-query attention, K_e / V_e rows are the concatenation of all KV heads of a token
   (the paper's k_i = W_K h_i is the whole projected vector); one S per rollout per layer.
7. Normalize(X) = X / max(||X||_F, eps) over the whole G x r state by default; per-row L2 and
   identity are selectable.
8. S_0 is not normalised; Normalize first applies at the first eviction.
13. Attention of an inactive rollout, or over an empty window, returns zeros.
14. Delta-W = A S B in the row convention of reading 2: a projection y = x W (x a row, W d_in x d_out)
    becomes y = x (W + A S B) with A d_in x G and B r x d_out.  Which projections receive it is not
    stated; the operation is the same for any.
15. Pinned question tokens: of the W cache slots, n_sink are reserved for a rollout's question
    tokens (at most n_sink of them, any number per rollout); the sliding window over thinking
    tokens holds W - n_sink.  Question tokens are attended to at every step, never evicted and
    never encoded; "full" means the sliding part is full.

End-to-end values are PARITY UNPINNED against the paper: it prints no number for any
intermediate or output of this path.  The pins in tests/ are closed forms, invariants, library
routines and brute force.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import numpy as np

NORM_FROBENIUS = 0
NORM_ROW_L2 = 1
NORM_NONE = 2


def attend(q: np.ndarray, keys: Sequence[np.ndarray], values: Sequence[np.ndarray],
           scale: Optional[float] = None) -> np.ndarray:
    """Grouped-query attention of one token's queries over a list of cached tokens.

    q: ``[H_q, d]``; keys[j], values[j]: ``[H_kv, d]`` for cached token j.  Query head h reads
    KV head ``h // (H_q // H_kv)``.  Returns ``[H_q, d]`` float64; zeros if the list is empty.
    """
    q = np.asarray(q, dtype=np.float64)
    H_q, d = q.shape
    out = np.zeros((H_q, d), dtype=np.float64)
    n = len(keys)
    if n == 0:
        return out
    K = np.stack([np.asarray(k, dtype=np.float64) for k in keys])      # [n, H_kv, d]
    V = np.stack([np.asarray(v, dtype=np.float64) for v in values])    # [n, H_kv, d]
    H_kv = K.shape[1]
    group = H_q // H_kv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    for h in range(H_q):
        kv = h // group
        scores = (K[:, kv, :] @ q[h]) * scale            # [n]
        e = np.exp(scores - scores.max())
        p = e / e.sum()
        out[h] = p @ V[:, kv, :]
    return out


def project_queries(q_g: np.ndarray, WaQ: np.ndarray) -> np.ndarray:
    """Q_a = q_g W^a_Q, ``[G, r]``."""
    return np.asarray(q_g, dtype=np.float64) @ np.asarray(WaQ, dtype=np.float64)


def encode_chunk(Q_a: np.ndarray, K_e: np.ndarray, V_e: np.ndarray,
                 WaK: np.ndarray, WaV: np.ndarray) -> np.ndarray:
    """S' = (Q_a (K_e W^a_K)^T)(V_e W^a_V), in exactly this association.

    Q_a ``[G, r]``; K_e, V_e ``[m, d_kv]`` (token rows, KV heads concatenated); WaK, WaV ``[d_kv, r]``.
    """
    K_a = np.asarray(K_e, dtype=np.float64) @ np.asarray(WaK, dtype=np.float64)   # [m, r]
    V_a = np.asarray(V_e, dtype=np.float64) @ np.asarray(WaV, dtype=np.float64)   # [m, r]
    return (np.asarray(Q_a, dtype=np.float64) @ K_a.T) @ V_a                      # [G, r]


def init_state(q_g, WaQ, WaK, WaV, k_g=None, v_g=None):
    """(Q_a, S_0): S_0 is the encoding of the global tokens' own keys and values, or zero without them."""
    Q_a = project_queries(q_g, WaQ)
    if k_g is None or v_g is None:
        return Q_a, np.zeros((Q_a.shape[0], np.asarray(WaV).shape[1]), dtype=np.float64)
    return Q_a, encode_chunk(Q_a, k_g, v_g, WaK, WaV)


def apply_delta(x: np.ndarray, A: np.ndarray, S: np.ndarray, B: np.ndarray, y: np.ndarray) -> np.ndarray:
    """y + x (A S B) for one rollout: x ``[d_in]``, A ``[d_in, G]``, S ``[G, r]``, B ``[r, d_out]``, y ``[d_out]``."""
    dW = np.asarray(A, dtype=np.float64) @ np.asarray(S, dtype=np.float64) @ np.asarray(B, dtype=np.float64)
    return np.asarray(y, dtype=np.float64) + np.asarray(x, dtype=np.float64) @ dW


def normalize(X: np.ndarray, mode: int = NORM_FROBENIUS, eps: float = 1e-12) -> np.ndarray:
    X = np.asarray(X, dtype=np.float64)
    if mode == NORM_NONE:
        return X.copy()
    if mode == NORM_FROBENIUS:
        return X / max(math.sqrt(float((X * X).sum())), eps)
    if mode == NORM_ROW_L2:
        n = np.sqrt((X * X).sum(axis=1, keepdims=True))
        return X / np.maximum(n, eps)
    raise ValueError("unknown norm mode %r" % (mode,))


class OracleRollout:
    """One rollout's bounded cache and context state."""

    def __init__(self, S0: np.ndarray):
        self.sink_k: List[np.ndarray] = []    # question tokens, kept for good; each [H_kv, d]
        self.sink_v: List[np.ndarray] = []
        self.win_k: List[np.ndarray] = []     # thinking tokens, logical order, oldest first
        self.win_v: List[np.ndarray] = []
        self.appended = 0                     # tokens appended so far
        self.evicted = 0                      # tokens evicted so far
        self.S = np.array(S0, dtype=np.float64)
        self.evicted_chunks: List[tuple] = [] # (K_e, V_e) of every eviction, for order checks


class OracleLayer:
    """Batched decode of B independent rollouts through one attention layer under a bounded window.

    ``window`` W is the cache capacity in tokens, ``chunk`` C the number of oldest tokens evicted
    at once when the window is full.  ``n_sink`` of the W slots are reserved for question tokens
    (see ``prefill``); the sliding window over thinking tokens then holds W - n_sink.
    """

    def __init__(self, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, window: int,
                 chunk: int, q_g, WaQ, WaK, WaV, k_g=None, v_g=None,
                 norm_mode: int = NORM_FROBENIUS, norm_eps: float = 1e-12,
                 softmax_scale: Optional[float] = None, keep_chunks: bool = False, n_sink: int = 0):
        assert n_q_heads % n_kv_heads == 0 and 0 <= n_sink < window and 1 <= chunk <= window - n_sink
        self.B, self.H_q, self.H_kv, self.d = batch, n_q_heads, n_kv_heads, head_dim
        self.W, self.C, self.n_sink = window, chunk, n_sink
        self.ring = window - n_sink           # capacity of the sliding part
        self.WaK = np.asarray(WaK, dtype=np.float64)
        self.WaV = np.asarray(WaV, dtype=np.float64)
        self.Q_a, self.S0 = init_state(q_g, WaQ, WaK, WaV, k_g, v_g)
        self.norm_mode, self.norm_eps = norm_mode, norm_eps
        self.scale = softmax_scale
        self.keep_chunks = keep_chunks
        self.rollouts = [OracleRollout(self.S0) for _ in range(batch)]

    # -- the three operations of a decode step, per rollout ---------------------------------
    def evict_encode(self, b: int) -> bool:
        """If rollout b's window is full: fold its C oldest tokens into S and drop them."""
        r = self.rollouts[b]
        if len(r.win_k) < self.ring:
            return False
        C = self.C
        K_e = np.stack([k.reshape(-1) for k in r.win_k[:C]])     # [C, d_kv], heads concatenated
        V_e = np.stack([v.reshape(-1) for v in r.win_v[:C]])
        S_new = encode_chunk(self.Q_a, K_e, V_e, self.WaK, self.WaV)
        r.S = normalize(r.S + S_new, self.norm_mode, self.norm_eps)
        del r.win_k[:C]
        del r.win_v[:C]
        r.evicted += C
        if self.keep_chunks:
            r.evicted_chunks.append((K_e, V_e))
        return True

    def append(self, b: int, k: np.ndarray, v: np.ndarray) -> None:
        r = self.rollouts[b]
        assert len(r.win_k) < self.ring, "append on a full window"
        r.win_k.append(np.array(k, dtype=np.float64))
        r.win_v.append(np.array(v, dtype=np.float64))
        r.appended += 1

    def attend(self, b: int, q: np.ndarray) -> np.ndarray:
        r = self.rollouts[b]
        return attend(q, r.sink_k + r.win_k, r.sink_v + r.win_v, self.scale)

    def prefill(self, b: int, K_p: np.ndarray, V_p: np.ndarray) -> None:
        """Question tokens of rollout b, ``[P, H_kv, d]`` each with P <= n_sink: kept permanently."""
        r = self.rollouts[b]
        assert len(K_p) == len(V_p) and len(r.sink_k) + len(K_p) <= self.n_sink, "more question tokens than n_sink"
        for kk, vv in zip(K_p, V_p):
            r.sink_k.append(np.array(kk, dtype=np.float64))
            r.sink_v.append(np.array(vv, dtype=np.float64))

    def reset_rollout(self, b: int) -> None:
        """Rollout b starts over: empty cache (question tokens included), S = S_0, counters at zero."""
        self.rollouts[b] = OracleRollout(self.S0)

    # -- one batched decode step ------------------------------------------------------------
    def step(self, q: np.ndarray, k: np.ndarray, v: np.ndarray,
             active: Optional[np.ndarray] = None) -> np.ndarray:
        """q ``[B, H_q, d]``, k and v ``[B, H_kv, d]``; returns out ``[B, H_q, d]`` (zeros where inactive)."""
        out = np.zeros((self.B, self.H_q, self.d), dtype=np.float64)
        for b in range(self.B):
            if active is not None and not active[b]:
                continue
            self.evict_encode(b)
            self.append(b, k[b], v[b])
            out[b] = self.attend(b, q[b])
        return out

    # -- views used by tests -----------------------------------------------------------------
    def state(self) -> np.ndarray:
        return np.stack([r.S for r in self.rollouts])

    def counters(self):
        return (np.array([r.appended for r in self.rollouts], dtype=np.int64),
                np.array([r.evicted for r in self.rollouts], dtype=np.int64))

    def window_kv(self, b: int):
        """Everything rollout b attends over: question tokens first, then the sliding window."""
        r = self.rollouts[b]
        ks, vs = r.sink_k + r.win_k, r.sink_v + r.win_v
        if not ks:
            z = np.zeros((0, self.H_kv, self.d))
            return z, z.copy()
        return np.stack(ks), np.stack(vs)

    def prompt_lengths(self) -> np.ndarray:
        return np.array([len(r.sink_k) for r in self.rollouts], dtype=np.int64)
