"""Pins for the importance-based eviction oracle (CPU only): every part is checked against
something other than itself -- closed forms, brute force written differently, the sliding-window
oracle it must reduce to, conservation of probability -- and planted mistakes must trip a pin."""
import math
from unittest import mock

import numpy as np
import pytest

from oracle import pte_oracle as po
from oracle import scored_oracle as so

RNG = np.random.default_rng(20260216)


def rand(*shape, scale=1.0):
    return RNG.standard_normal(shape) * scale


def _enc(G=3, r=4, d_q=8, d_kv=4):
    return dict(q_g=rand(G, d_q), WaQ=rand(d_q, r), WaK=rand(d_kv, r), WaV=rand(d_kv, r),
                k_g=rand(G, d_kv), v_g=rand(G, d_kv))


def _layer(B, H_q, H_kv, d, W, C, n_recent, n_sink=0, enc=None):
    e = enc or _enc(d_q=H_q * d, d_kv=H_kv * d)
    return so.ScoredOracleLayer(B, H_q, H_kv, d, W, C, n_recent, e["q_g"], e["WaQ"], e["WaK"], e["WaV"],
                                e["k_g"], e["v_g"], n_sink=n_sink), e


# ---- probabilities ---------------------------------------------------------------------------

def test_probabilities_sum_to_one_and_reproduce_the_attention_output():
    H_q, H_kv, d, n = 6, 2, 5, 9
    q, K, V = rand(H_q, d), rand(n, H_kv, d), rand(n, H_kv, d)
    P = so.attention_probs(q, list(K))
    assert P.shape == (H_q, n) and np.allclose(P.sum(axis=1), 1.0, atol=1e-14)
    ref = po.attend(q, list(K), list(V))
    got = np.stack([P[h] @ V[:, h // 3, :] for h in range(H_q)])
    assert np.allclose(got, ref, atol=1e-13)


def test_probabilities_closed_forms():
    # two keys: p_1 = sigmoid((q.k_1 - q.k_0) / sqrt(d)); one key: 1; zero query: uniform
    q = np.array([[1.0, 2.0, 0.0, -1.0]])
    k0, k1 = np.array([[0.5, 0.0, 1.0, 0.0]]), np.array([[0.0, 1.0, 0.0, 2.0]])
    P = so.attention_probs(q, [k0, k1])
    x = (q[0] @ k1[0] - q[0] @ k0[0]) / 2.0
    assert abs(P[0, 1] - 1.0 / (1.0 + math.exp(-x))) < 1e-15
    assert np.array_equal(so.attention_probs(q, [k0]), np.ones((1, 1)))
    assert np.allclose(so.attention_probs(np.zeros((2, 4)), [k0, k1, k0]), 1.0 / 3.0)
    assert so.attention_probs(q, []).shape == (1, 0)
    # custom scale and the GQA head map: head h reads KV head h // group
    K = rand(5, 2, 3)
    q2 = rand(4, 3)
    P2 = so.attention_probs(q2, list(K), scale=0.7)
    for h in range(4):
        e = np.exp(0.7 * (K[:, h // 2, :] @ q2[h]))
        assert np.allclose(P2[h], e / e.sum(), atol=1e-14)


# ---- selection -------------------------------------------------------------------------------

@pytest.mark.parametrize("n,n_el,C", [(12, 12, 4), (16, 9, 9), (20, 13, 1), (40, 31, 7)])
def test_selection_against_a_sort(n, n_el, C):
    for trial in range(20):
        # few distinct values: plenty of ties
        scores = RNG.integers(0, 5, n).astype(np.float64) / 4.0
        got = so.select_victims(list(scores), C, n_el)
        order = sorted(range(n_el), key=lambda i: (scores[i], i))       # by score, then older first
        assert got == sorted(order[:C])
        assert len(got) == C and all(0 <= i < n_el for i in got)
        rest = [scores[i] for i in range(n_el) if i not in got]
        assert not rest or max(scores[i] for i in got) <= min(rest)


def test_selection_prefers_the_older_entry_among_equals():
    assert so.select_victims([1.0, 0.5, 0.5, 0.5, 2.0], 2, 5) == [1, 2]
    assert so.select_victims([0.0, 0.0, 0.0, 0.0], 1, 3) == [0]
    # entries past n_eligible are never taken, however low their score
    assert so.select_victims([3.0, 2.0, 5.0, 0.0, 0.0], 2, 3) == [0, 1]


# ---- ring after an eviction --------------------------------------------------------------------

def _ring_by_copying(n, C, victims):
    """The same move written on an array of places, the way a cache would do it."""
    place = list(range(n))                       # place[i] = entry stored there
    holes = [i for i in sorted(victims) if i >= C]
    movers = [i for i in range(C) if i not in victims]
    for dst, src in zip(holes, movers):
        place[dst] = place[src]
    return place[C:]


@pytest.mark.parametrize("n,C", [(8, 3), (16, 4), (12, 12), (9, 1)])
def test_ring_after_eviction(n, C):
    # the oldest chunk itself: nothing moves
    assert so.ring_after_eviction(n, C, list(range(C))) == list(range(C, n))
    for trial in range(30):
        victims = sorted(RNG.choice(n, size=C, replace=False).tolist())
        new = so.ring_after_eviction(n, C, victims)
        assert new == _ring_by_copying(n, C, set(victims))
        assert sorted(new) == [i for i in range(n) if i not in victims]      # exactly the survivors
        for i in range(C, n):                                                # the others keep their place
            if i not in victims:
                assert new[i - C] == i
        moved = [x for x in new if x < C]
        assert moved == sorted(moved)                                        # survivors keep their order


def test_ring_after_eviction_hand_worked():
    # ring 0..7, chunk 3, victims 1, 4, 6: survivors 0 and 2 of the chunk go to places 4 and 6
    assert so.ring_after_eviction(8, 3, [1, 4, 6]) == [3, 0, 5, 2, 7]


# ---- the layer -----------------------------------------------------------------------------------

@pytest.mark.parametrize("n_sink,P", [(0, 0), (4, 3)])
def test_with_only_the_oldest_chunk_eligible_it_is_the_sliding_window(n_sink, P):
    B, H_q, H_kv, d, W, C, T = 2, 4, 2, 3, 10 + n_sink, 3, 40
    lay, e = _layer(B, H_q, H_kv, d, W, C, n_recent=W - n_sink - C, n_sink=n_sink)
    ref = po.OracleLayer(B, H_q, H_kv, d, W, C, e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"], n_sink=n_sink)
    if P:
        pk, pv = rand(B, P, H_kv, d), rand(B, P, H_kv, d)
        for b in range(B):
            lay.prefill(b, pk[b], pv[b])
            ref.prefill(b, pk[b], pv[b])
    for t in range(T):
        q, k, v = rand(B, H_q, d), rand(B, H_kv, d), rand(B, H_kv, d)
        act = np.array([1, t % 3 != 1], dtype=np.uint8)
        assert np.allclose(lay.step(q, k, v, act), ref.step(q, k, v, act), atol=1e-13)
    assert np.allclose(lay.state(), ref.state(), atol=1e-13)
    assert all(np.array_equal(a, b) for a, b in zip(lay.counters(), ref.counters()))
    for b in range(B):
        assert np.array_equal(lay.positions(b), np.arange(lay.evicted[b], lay.appended[b]))


def test_scores_without_eviction_are_lagged_column_sums_of_causal_attention():
    # W >= T: nothing leaves.  After T steps token j's folded score is the probability it received
    # from the queries of steps j .. T-2 (the last step is still pending), all heads summed.
    H_q, H_kv, d, T = 4, 2, 3, 9
    lay, _ = _layer(1, H_q, H_kv, d, 16, 4, n_recent=4)
    Q, K = rand(T, 1, H_q, d), rand(T, 1, H_kv, d)
    for t in range(T):
        lay.step(Q[t], K[t], rand(1, H_kv, d))
    full = np.zeros((T, T))                      # full[t, j] = sum over heads of p_t(j), causal
    for t in range(T):
        for h in range(H_q):
            s = np.array([K[j, 0, h // 2] @ Q[t, 0, h] for j in range(t + 1)]) / math.sqrt(d)
            w = np.exp(s)
            full[t, :t + 1] += w / w.sum()
    assert np.allclose(lay.scores(0), full[:T - 1].sum(axis=0), atol=1e-13)
    pending = np.array([e.pending for e in lay.win[0]])
    assert np.allclose(pending, full[T - 1], atol=1e-13)
    # every step hands out exactly H_q of probability
    assert abs(lay.scores(0).sum() + pending.sum() - H_q * T) < 1e-12


def test_a_heavy_hitter_stays_and_the_recent_tokens_are_protected():
    # token 2's key lines up with every later query: it collects the probability and is never chosen,
    # although it is among the oldest; victims never come from the n_recent newest ring entries
    H_q, H_kv, d, W, C, n_recent, T = 2, 1, 4, 12, 3, 4, 60
    lay, _ = _layer(1, H_q, H_kv, d, W, C, n_recent)
    u = np.array([1.0, 0.0, 0.0, 0.0])
    for t in range(T):
        k = rand(1, H_kv, d, scale=0.3)
        if t == 2:
            k[0, 0] = 6.0 * u
        before = lay.positions(0).tolist()
        lay.step(np.tile(3.0 * u, (1, H_q, 1)) + rand(1, H_q, d, scale=0.1), k, rand(1, H_kv, d))
        if lay.last_victims[0] is not None and lay.evicted[0] and len(before) == W:
            assert len(lay.last_victims[0]) == C and 2 not in lay.last_victims[0]
            assert set(lay.last_victims[0]) <= set(before[:W - n_recent])
    assert 2 in lay.positions(0).tolist()
    assert lay.evicted[0] == C * math.ceil((T - W) / C) and len(lay.win[0]) == T - lay.evicted[0]


def test_state_is_the_encoding_of_the_victims_in_ring_order():
    H_q, H_kv, d, W, C, n_recent = 2, 2, 2, 8, 3, 2
    lay, e = _layer(1, H_q, H_kv, d, W, C, n_recent)
    K, V = rand(W + 1, 1, H_kv, d), rand(W + 1, 1, H_kv, d)
    for t in range(W):
        lay.step(rand(1, H_q, d), K[t], V[t])
    lay.set_scores(0, [5, 1, 7, 0, 9, 2, 8, 8])          # eligible: the first 6; lowest three: 3, 1, 5
    lay.step(rand(1, H_q, d), K[W], V[W])
    assert lay.last_victims[0] == [1, 3, 5]
    Q_a, S0 = po.init_state(e["q_g"], e["WaQ"], e["WaK"], e["WaV"], e["k_g"], e["v_g"])
    S1 = sum(np.outer(Q_a @ (K[j, 0].reshape(-1) @ e["WaK"]), V[j, 0].reshape(-1) @ e["WaV"]) for j in (1, 3, 5))
    X = S0 + S1
    assert np.allclose(lay.state()[0], X / np.linalg.norm(X), atol=1e-13)
    # ring afterwards: places 3..7 with 0 -> place 3 and 2 -> place 5, then the new token
    assert lay.positions(0).tolist() == [0, 4, 2, 6, 7, 8]


# ---- planted mistakes ------------------------------------------------------------------------------

SCORED_PINS = [
    test_probabilities_sum_to_one_and_reproduce_the_attention_output,
    test_probabilities_closed_forms,
    lambda: test_selection_against_a_sort(16, 9, 4),
    test_selection_prefers_the_older_entry_among_equals,
    lambda: test_ring_after_eviction(16, 4),
    test_ring_after_eviction_hand_worked,
    lambda: test_with_only_the_oldest_chunk_eligible_it_is_the_sliding_window(4, 3),
    test_scores_without_eviction_are_lagged_column_sums_of_causal_attention,
    test_a_heavy_hitter_stays_and_the_recent_tokens_are_protected,
    test_state_is_the_encoding_of_the_victims_in_ring_order,
]


def _some_pin_fails():
    for pin in SCORED_PINS:
        try:
            with np.errstate(all="ignore"):
                pin()
        except (AssertionError, ValueError, IndexError, KeyError):
            return True
    return False


_probs, _select, _ring = so.attention_probs, so.select_victims, so.ring_after_eviction


def _probs_wrong_head(q, keys, scale=None):
    return _probs(np.asarray(q)[::-1], keys, scale)[::-1] if np.asarray(q).shape[0] > 1 else _probs(q, keys, 1.0)


def _select_highest(scores, C, n_el):
    return _select([-s for s in scores], C, n_el)


def _select_newer_among_equals(scores, C, n_el):
    return sorted(sorted(range(n_el), key=lambda i: (scores[i], -i))[:C])


def _select_ignores_recent(scores, C, n_el):
    return _select(scores, C, len(scores))


def _ring_reversed_matching(n, C, victims):
    vset = set(victims)
    surv = [i for i in range(C) if i not in vset][::-1]
    move = dict(zip([i for i in range(C, n) if i in vset], surv))
    return [move.get(i, i) for i in range(C, n)]


def _ring_drops_survivors(n, C, victims):
    return [i for i in range(C, n) if i not in set(victims)]


class _NoLag(so.ScoredOracleLayer):
    def step(self, q, k, v, active=None):
        out = super().step(q, k, v, active)
        for win in self.win:
            for e in win:
                e.score += e.pending
                e.pending = 0.0
        return out


@pytest.mark.parametrize("name,patch", [
    ("head map", ("attention_probs", _probs_wrong_head)),
    ("evicts the heaviest", ("select_victims", _select_highest)),
    ("ties towards newer", ("select_victims", _select_newer_among_equals)),
    ("recent tokens unprotected", ("select_victims", _select_ignores_recent)),
    ("survivors matched in reverse", ("ring_after_eviction", _ring_reversed_matching)),
    ("survivors of the oldest chunk lost", ("ring_after_eviction", _ring_drops_survivors)),
    ("no lag", ("ScoredOracleLayer", _NoLag)),
])
def test_planted_mistakes_trip_a_pin(name, patch):
    assert not _some_pin_fails()
    with mock.patch.object(so, patch[0], patch[1]):
        assert _some_pin_fails(), "no pin noticed: " + name
