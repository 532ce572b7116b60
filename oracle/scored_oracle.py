"""CPU fp64 oracle for importance-based eviction on top of the bounded-cache decode step.

TEST INFRASTRUCTURE ONLY (same rules as ``pte_oracle``): imported by tests, the smoke check and
the benchmark's CPU leg; shares nothing with the HIP path and imports nothing from it.

The paper keeps the sliding window for training and reports, as an ablation, that dropping
tokens by importance instead of by age (H2O, PyramidKV, HeadKV) helps accuracy at a 37 % cost in
rollout time, leaving an efficient integration as future work (Ablation Study and Discussion, "Integration with
inference-time token dropping strategy").  It gives no algorithm of its own, so this file follows
the published heavy-hitter rule (H2O: keep the tokens with the largest accumulated attention
probability plus the most recent ones, drop the rest) with the readings below.  It is an
heuristic, not a quantity with a plain definition, so the oracle takes the steps in order.
PARITY UNPINNED against the paper: it prints the accuracy of such policies only.

Readings
  s1. A token's score is the attention probability it has received, summed over decode steps and
      over ALL query heads: the encoder folds whole tokens (all KV heads concatenated) into S, so
      a token leaves for every head at once and one score per token is what the selection needs.
  s2. One-step lag: the probabilities of a step are added to the scores during the NEXT step of
      that rollout (after its eviction and append), so a selection sees every step but the one
      just before it.  (The normaliser of a softmax is known only once the whole window has been
      read; folding a step's probabilities while the next step streams the same keys costs no
      extra pass over the cache.)  A token evicted in between simply loses that last increment.
  s3. Chunked: when the sliding part is full, C tokens leave at once (as in the sliding-window
      policy), chosen among all but the ``n_recent`` most recent ring entries as the C lowest
      scores, ties broken towards the older ring entry.  With n_recent = ring size - C only the
      oldest chunk is eligible and the policy IS the sliding window.
  s4. Ring order after an eviction: the ring stays a contiguous run.  The entries of the oldest
      chunk that survive are moved into the places of the victims outside that chunk (k-th
      survivor, oldest first, to the k-th such place, oldest first) and the oldest chunk's places
      are dropped.  Attention does not depend on the order of the cache (a key carries its own
      position), so this only decides which entries count as "recent" later on.
  s5. The victims are encoded as one chunk, S <- Normalize(S + S') as for the sliding window.  S' is
      a sum over tokens, so the order within the chunk matters to rounding only (here: ring order).
  s6. Question tokens are never scored, evicted or moved.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import numpy as np

from oracle import pte_oracle as po


def attention_probs(q: np.ndarray, keys: Sequence[np.ndarray], scale: Optional[float] = None) -> np.ndarray:
    """Softmax probabilities ``[H_q, n]`` of one token's queries over n cached tokens (keys[j] ``[H_kv, d]``)."""
    q = np.asarray(q, dtype=np.float64)
    H_q, d = q.shape
    n = len(keys)
    if n == 0:
        return np.zeros((H_q, 0), dtype=np.float64)
    K = np.stack([np.asarray(k, dtype=np.float64) for k in keys])      # [n, H_kv, d]
    group = H_q // K.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    P = np.zeros((H_q, n), dtype=np.float64)
    for h in range(H_q):
        s = (K[:, h // group, :] @ q[h]) * scale
        e = np.exp(s - s.max())
        P[h] = e / e.sum()
    return P


def select_victims(scores: Sequence[float], C: int, n_eligible: int) -> List[int]:
    """Ring indices (ascending) of the C lowest scores among indices [0, n_eligible); ties -> older."""
    assert 0 < C <= n_eligible <= len(scores)
    taken = [False] * n_eligible
    for _ in range(C):
        best = -1
        for i in range(n_eligible):
            if not taken[i] and (best < 0 or scores[i] < scores[best]):
                best = i                      # strict <: among equals the first (oldest) stays chosen
        taken[best] = True
    return [i for i in range(n_eligible) if taken[i]]


def ring_after_eviction(n: int, C: int, victims: Sequence[int]) -> List[int]:
    """New ring, as old ring indices: places C .. n-1 in order, a victim's place taken by a survivor
    of the oldest chunk (k-th survivor to the k-th victim place beyond the chunk)."""
    vset = set(victims)
    assert len(vset) == C and all(0 <= v < n for v in vset)
    survivors = [i for i in range(C) if i not in vset]
    places = [i for i in range(C, n) if i in vset]
    assert len(survivors) == len(places)
    move = dict(zip(places, survivors))
    return [move.get(i, i) for i in range(C, n)]


class _Entry:
    __slots__ = ("k", "v", "pos", "score", "pending")

    def __init__(self, k, v, pos):
        self.k, self.v, self.pos = k, v, pos
        self.score = 0.0      # accumulated attention probability, folded steps only
        self.pending = 0.0    # the latest step's probability, folded at the next step (reading s2)


class ScoredOracleLayer:
    """B independent rollouts through one attention layer whose bounded cache drops the
    lowest-scored tokens.  Same construction arguments as ``pte_oracle.OracleLayer`` plus
    ``n_recent``; the encoder, Normalize and attention are the functions of ``pte_oracle``."""

    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, window, chunk, n_recent,
                 q_g, WaQ, WaK, WaV, k_g=None, v_g=None, norm_mode=po.NORM_FROBENIUS, norm_eps=1e-12,
                 softmax_scale=None, n_sink: int = 0):
        self.B, self.H_q, self.H_kv, self.d = batch, n_q_heads, n_kv_heads, head_dim
        self.W, self.C, self.n_sink = window, chunk, n_sink
        self.ring = window - n_sink
        assert 0 <= n_recent and chunk <= self.ring - n_recent, "fewer eligible tokens than a chunk"
        self.n_recent = n_recent
        self.WaK = np.asarray(WaK, dtype=np.float64)
        self.WaV = np.asarray(WaV, dtype=np.float64)
        self.Q_a, self.S0 = po.init_state(q_g, WaQ, WaK, WaV, k_g, v_g)
        self.norm_mode, self.norm_eps, self.scale = norm_mode, norm_eps, softmax_scale
        self.sink_k: List[list] = [[] for _ in range(batch)]
        self.sink_v: List[list] = [[] for _ in range(batch)]
        self.win: List[List[_Entry]] = [[] for _ in range(batch)]
        self.S = [np.array(self.S0) for _ in range(batch)]
        self.appended = [0] * batch
        self.evicted = [0] * batch
        self.last_victims: List[Optional[List[int]]] = [None] * batch   # positions, ring order
        self.min_margin = math.inf     # smallest relative gap between the last victim and the best survivor

    def prefill(self, b: int, K_p, V_p) -> None:
        assert len(self.sink_k[b]) + len(K_p) <= self.n_sink
        for kk, vv in zip(K_p, V_p):
            self.sink_k[b].append(np.array(kk, dtype=np.float64))
            self.sink_v[b].append(np.array(vv, dtype=np.float64))

    # -- eviction (readings s3, s4, s5) ---------------------------------------------------------
    def evict_encode(self, b: int) -> bool:
        win = self.win[b]
        n = len(win)
        if n < self.ring:
            return False
        C, n_el = self.C, n - self.n_recent
        scores = [e.score for e in win]
        victims = select_victims(scores, C, n_el)
        vset = set(victims)
        rest = [scores[i] for i in range(n_el) if i not in vset]
        if rest:
            worst, best = max(scores[i] for i in victims), min(rest)
            self.min_margin = min(self.min_margin, (best - worst) / max(abs(best), 1e-300))
        K_e = np.stack([win[i].k.reshape(-1) for i in victims])
        V_e = np.stack([win[i].v.reshape(-1) for i in victims])
        S_new = po.encode_chunk(self.Q_a, K_e, V_e, self.WaK, self.WaV)
        self.S[b] = po.normalize(self.S[b] + S_new, self.norm_mode, self.norm_eps)
        self.last_victims[b] = [win[i].pos for i in victims]
        self.win[b] = [win[i] for i in ring_after_eviction(n, C, victims)]
        self.evicted[b] += C
        return True

    # -- one batched decode step ------------------------------------------------------------------
    def step(self, q, k, v, active=None) -> np.ndarray:
        out = np.zeros((self.B, self.H_q, self.d), dtype=np.float64)
        for b in range(self.B):
            if active is not None and not active[b]:
                continue
            self.evict_encode(b)
            win = self.win[b]
            assert len(win) < self.ring
            win.append(_Entry(np.array(k[b], dtype=np.float64), np.array(v[b], dtype=np.float64), self.appended[b]))
            self.appended[b] += 1
            for e in win:                       # the previous step's probabilities join the scores now
                e.score += e.pending
                e.pending = 0.0
            keys = self.sink_k[b] + [e.k for e in win]
            vals = self.sink_v[b] + [e.v for e in win]
            P = attention_probs(q[b], keys, self.scale)                       # [H_q, n]
            V = np.stack(vals)                                                # [n, H_kv, d]
            group = self.H_q // self.H_kv
            for h in range(self.H_q):
                out[b, h] = P[h] @ V[:, h // group, :]
            mass = P.sum(axis=0)[len(self.sink_k[b]):]
            for e, m in zip(win, mass):
                e.pending = float(m)
        return out

    # -- views used by tests ----------------------------------------------------------------------
    def state(self) -> np.ndarray:
        return np.stack(self.S)

    def counters(self):
        return np.array(self.appended, dtype=np.int64), np.array(self.evicted, dtype=np.int64)

    def scores(self, b: int) -> np.ndarray:
        """Folded scores of rollout b's ring entries, ring order (what a selection now would see)."""
        return np.array([e.score for e in self.win[b]], dtype=np.float64)

    def positions(self, b: int) -> np.ndarray:
        return np.array([e.pos for e in self.win[b]], dtype=np.int64)

    def set_scores(self, b: int, scores) -> None:
        assert len(scores) == len(self.win[b])
        for e, s in zip(self.win[b], scores):
            e.score, e.pending = float(s), 0.0
