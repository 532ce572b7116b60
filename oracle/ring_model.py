"""Integer model of the ring-buffer cache: which token position every slot holds, and which slots
an eviction takes.

TEST INFRASTRUCTURE ONLY (same rules as ``pte_oracle``): imported by tests, the smoke check and
the benchmark's CPU leg; shares nothing with the HIP path.

The model is independent of ``pte_oracle`` (which keeps a list and never computes a slot): a
token's *position* p is its 0-based append index within its rollout; it lives in slot
``n_sink + p mod (W - n_sink)`` while ``base <= p < len`` (slots ``0 .. n_sink-1`` are reserved for
question tokens, which never move: question token j sits in slot j).  The bounded cache of the
paper (Challenges for Efficient RL Training: the pruned context of the cache policy D; Our
Approach: sliding-window eviction of the earliest thinking tokens once the cache is full, question
tokens kept) is the question tokens plus the set of live positions.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np


class RingModel:
    def __init__(self, batch: int, window: int, chunk: int, start: int = 0, n_sink: int = 0):
        assert 0 <= n_sink < window and 1 <= chunk <= window - n_sink
        self.B, self.W, self.C, self.n_sink = batch, window, chunk, n_sink
        self.R = window - n_sink                            # ring capacity
        self.len = np.full(batch, start, dtype=np.int64)    # tokens appended (plus the start offset)
        self.base = np.full(batch, start, dtype=np.int64)   # tokens evicted (plus the start offset)
        # slot_pos[b][s] = position currently stored in slot s, or -1 if never written
        self.slot_pos = np.full((batch, window), -1, dtype=np.int64)
        self.evictions: List[List[np.ndarray]] = [[] for _ in range(batch)]   # slot lists, oldest first

    def n_live(self) -> np.ndarray:
        return self.len - self.base

    def evict(self, active: Optional[np.ndarray] = None) -> np.ndarray:
        """Evict the C oldest positions of every active rollout whose window is full.
        Returns uint8 [B]: which rollouts evicted."""
        did = np.zeros(self.B, dtype=np.uint8)
        for b in range(self.B):
            if active is not None and not active[b]:
                continue
            if self.len[b] - self.base[b] == self.R:
                pos = np.arange(self.base[b], self.base[b] + self.C, dtype=np.int64)
                self.evictions[b].append(self.n_sink + pos % self.R)
                self.base[b] += self.C
                did[b] = 1
        return did

    def append(self, active: Optional[np.ndarray] = None) -> np.ndarray:
        """Append one token per active rollout; returns the slot written (int64 [B], -1 if inactive)."""
        slots = np.full(self.B, -1, dtype=np.int64)
        for b in range(self.B):
            if active is not None and not active[b]:
                continue
            assert self.len[b] - self.base[b] < self.R, "append on a full window"
            s = self.n_sink + int(self.len[b] % self.R)
            self.slot_pos[b, s] = self.len[b]
            slots[b] = s
            self.len[b] += 1
        return slots

    def step(self, active: Optional[np.ndarray] = None) -> np.ndarray:
        self.evict(active)
        return self.append(active)

    def live_slots(self, b: int) -> np.ndarray:
        """Slots of rollout b's live positions in logical order (oldest first)."""
        return self.n_sink + np.arange(self.base[b], self.len[b], dtype=np.int64) % self.R


def n_live_closed_form(t: int, W: int, C: int) -> int:
    """Live tokens seen by the attention of decode step t (1-based) under lazy chunk eviction."""
    if t <= W:
        return t
    return W - C + ((t - W - 1) % C) + 1


def evicted_closed_form(t: int, W: int, C: int) -> int:
    """Tokens evicted by the end of decode step t (1-based): C * ceil((t - W) / C) for t > W."""
    if t <= W:
        return 0
    return C * (-((-(t - W)) // C))
