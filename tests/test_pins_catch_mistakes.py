"""Planted mistakes, on the CPU, in the oracle: each plausible error (a dropped term, a wrong index,
a swapped operand, a step out of order) must trip at least one of the pins in test_oracle_pins."""
import math
from unittest import mock

import numpy as np
import pytest

from oracle import pte_oracle as po
from tests import test_oracle_pins as pins

PINS = [
    pins.test_two_keys_closed_form_with_scale,
    pins.test_single_key_weight_is_one,
    pins.test_zero_query_gives_mean_of_values,
    pins.test_gqa_head_mapping,
    lambda: pins.test_tiny_cases_against_naive_exponentials(5, 4),
    pins.test_peaky_scores_against_logsumexp,
    pins.test_encode_hand_worked_integers,
    pins.test_encode_uses_key_and_value_projections_separately,
    pins.test_encode_is_a_sum_of_per_token_outer_products,
    pins.test_encode_brute_force_loops,
    pins.test_init_state_is_encoding_of_global_tokens_unnormalised,
    pins.test_normalize_frobenius,
    pins.test_window_at_least_sequence_is_full_causal_attention,
    lambda: pins.test_bounded_window_is_attention_over_last_tokens_and_evicts_oldest_first(8, 3),
    pins.test_state_update_normalises_after_every_eviction_and_starts_from_S0,
    lambda: pins.test_question_tokens_stay_and_only_thinking_tokens_slide(12, 4, 3, (4, 2)),
    pins.test_apply_delta_hand_worked_and_structure,
]


def some_pin_fails():
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin()
        except AssertionError:
            return True
        except (ValueError, IndexError, FloatingPointError):
            return True          # the mistake broke shapes outright: caught as well
    return False


def test_the_unmodified_oracle_passes_every_pin():
    assert not some_pin_fails()


_attend = po.attend
_encode = po.encode_chunk
_normalize = po.normalize
_apply = po.apply_delta


def attend_without_scale(q, keys, values, scale=None):
    return _attend(q, keys, values, 1.0 if scale is None else scale)


def attend_wrong_head_map(q, keys, values, scale=None):
    H_q = np.asarray(q).shape[0]
    H_kv = np.asarray(keys[0]).shape[0] if len(keys) else 1
    perm = [(h % H_kv) * (H_q // H_kv) for h in range(H_q)]        # h % H_kv instead of h // group
    out = np.zeros_like(np.asarray(q, dtype=np.float64))
    for h in range(H_q):
        qq = np.zeros_like(np.asarray(q, dtype=np.float64))
        qq[perm[h]] = np.asarray(q)[h]
        out[h] = _attend(qq, keys, values, scale)[perm[h]]
    return out


def attend_no_max_subtraction(q, keys, values, scale=None):
    q = np.asarray(q, dtype=np.float64)
    if not len(keys):
        return np.zeros_like(q)
    K, V = np.stack(keys).astype(np.float64), np.stack(values).astype(np.float64)
    g = q.shape[0] // K.shape[1]
    sc = 1.0 / math.sqrt(q.shape[1]) if scale is None else scale
    out = np.zeros_like(q)
    for h in range(q.shape[0]):
        e = np.exp(np.minimum((K[:, h // g] @ q[h]) * sc, 60.0))    # "safe" clamp instead of the max trick
        out[h] = (e / e.sum()) @ V[:, h // g]
    return out


def attend_skips_newest_key(q, keys, values, scale=None):
    return _attend(q, keys[:-1], values[:-1], scale)


def encode_swapped_projections(Q_a, K_e, V_e, WaK, WaV):
    return _encode(Q_a, K_e, V_e, WaV, WaK)


def encode_with_attention_scale(Q_a, K_e, V_e, WaK, WaV):
    return _encode(Q_a, K_e, V_e, WaK, WaV) / math.sqrt(np.asarray(Q_a).shape[1])


def encode_keys_for_values(Q_a, K_e, V_e, WaK, WaV):
    return _encode(Q_a, K_e, K_e, WaK, WaV)


def encode_softmaxed(Q_a, K_e, V_e, WaK, WaV):
    K_a, V_a = np.asarray(K_e) @ WaK, np.asarray(V_e) @ WaV
    s = np.asarray(Q_a) @ K_a.T
    p = np.exp(s - s.max(axis=1, keepdims=True))
    return (p / p.sum(axis=1, keepdims=True)) @ V_a


def normalize_skipped(X, mode=po.NORM_FROBENIUS, eps=1e-12):
    return np.array(X, dtype=np.float64)


def normalize_by_max(X, mode=po.NORM_FROBENIUS, eps=1e-12):
    X = np.asarray(X, dtype=np.float64)
    return X / max(np.abs(X).max(), eps) if mode == po.NORM_FROBENIUS else _normalize(X, mode, eps)


def apply_delta_transposed_state(x, A, S, B, y):
    S = np.asarray(S)
    return _apply(x, A, S.T, B, y) if S.shape[0] == S.shape[1] else _apply(x, A, S, B, y) * 1.0 + 1.0


class EagerEvictionLayer(po.OracleLayer):
    def step(self, q, k, v, active=None):
        out = np.zeros((self.B, self.H_q, self.d))
        for b in range(self.B):
            if active is not None and not active[b]:
                continue
            self.append(b, k[b], v[b])
            out[b] = self.attend(b, q[b])
            self.evict_encode(b)                         # right after the window fills, not before the next append
        return out


class NewestChunkLayer(po.OracleLayer):
    def evict_encode(self, b):
        r = self.rollouts[b]
        if len(r.win_k) < self.ring:
            return False
        r.win_k[:], r.win_v[:] = r.win_k[::-1], r.win_v[::-1]       # the newest C tokens leave instead of the oldest
        done = super().evict_encode(b)
        r.win_k[:], r.win_v[:] = r.win_k[::-1], r.win_v[::-1]
        return done


class AttendBeforeAppendLayer(po.OracleLayer):
    def step(self, q, k, v, active=None):
        out = np.zeros((self.B, self.H_q, self.d))
        for b in range(self.B):
            if active is not None and not active[b]:
                continue
            self.evict_encode(b)
            out[b] = self.attend(b, q[b])
            self.append(b, k[b], v[b])
        return out


class SinkCountsAsWindowLayer(po.OracleLayer):
    def __init__(self, *a, **kw):
        super().__init__(*a, **kw)
        self.ring = self.W                                # question slots are not set aside


class NormalisedInitLayer(po.OracleLayer):
    def __init__(self, *a, **kw):
        super().__init__(*a, **kw)
        self.S0 = _normalize(self.S0)
        for r in self.rollouts:
            r.S = self.S0.copy()


FUNCTION_MISTAKES = {
    "no 1/sqrt(d) in the scores": ("attend", attend_without_scale),
    "query head h reads KV head h % H_kv": ("attend", attend_wrong_head_map),
    "clamp instead of max subtraction": ("attend", attend_no_max_subtraction),
    "query does not see its own key": ("attend", attend_skips_newest_key),
    "W^a_K and W^a_V swapped": ("encode_chunk", encode_swapped_projections),
    "1/sqrt(r) in the encoding": ("encode_chunk", encode_with_attention_scale),
    "K_e used for the values too (the equation's misprint taken literally)": ("encode_chunk", encode_keys_for_values),
    "softmax in the encoding": ("encode_chunk", encode_softmaxed),
    "Normalize dropped": ("normalize", normalize_skipped),
    "max-norm instead of Frobenius": ("normalize", normalize_by_max),
    "S transposed in the weight delta": ("apply_delta", apply_delta_transposed_state),
}

LAYER_MISTAKES = {
    "eager eviction": EagerEvictionLayer,
    "newest chunk evicted": NewestChunkLayer,
    "attend before append": AttendBeforeAppendLayer,
    "question slots not set aside": SinkCountsAsWindowLayer,
    "S_0 normalised": NormalisedInitLayer,
}


@pytest.mark.parametrize("what", sorted(FUNCTION_MISTAKES))
def test_function_level_mistake_is_caught(what):
    name, wrong = FUNCTION_MISTAKES[what]
    with mock.patch.object(po, name, wrong):
        assert some_pin_fails(), what


@pytest.mark.parametrize("what", sorted(LAYER_MISTAKES))
def test_layer_level_mistake_is_caught(what):
    with mock.patch.object(po, "OracleLayer", LAYER_MISTAKES[what]):
        assert some_pin_fails(), what
