"""Pins for the CPU oracle: closed forms, library routines, invariants and brute force.

The paper prints no numeric value for any quantity on this path, so nothing here is a stored
paper value; every expected number below is either derived by hand in the comment next to it,
or computed by an independent route (scipy / numpy library routine, pure-Python loops).
"""
import itertools
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import pte_oracle as po
from oracle.ring_model import RingModel, evicted_closed_form, n_live_closed_form

RNG = np.random.default_rng(7)


def rand(*shape, scale=1.0):
    return RNG.standard_normal(shape) * scale


# ---------------------------------------------------------------------------------------------
# attention (Notation and Preliminaries: o_t = softmax(q_t K_t^T / sqrt(d)) V_t)
# ---------------------------------------------------------------------------------------------

def direct_attention(q, K, V, group):
    """Independent route: library softmax, one head at a time. q [H_q,d], K,V [n,H_kv,d]."""
    H_q, d = q.shape
    out = np.zeros((H_q, d))
    for h in range(H_q):
        kv = h // group
        w = softmax(K[:, kv, :] @ q[h] / math.sqrt(d))
        out[h] = w @ V[:, kv, :]
    return out


def test_two_keys_closed_form_with_scale():
    # d = 4, q = (2,0,0,0), k1 = (1,0,0,0), k2 = (-1,0,0,0): scores = (2, -2)/sqrt(4) = (1, -1).
    # weights = (e, 1/e)/(e + 1/e); v1 = 1, v2 = 0 on every coordinate => out = e^2/(e^2+1).
    q = np.array([[2.0, 0, 0, 0]])
    k1 = np.array([[1.0, 0, 0, 0]])
    k2 = -k1
    v1 = np.ones((1, 4))
    v2 = np.zeros((1, 4))
    out = po.attend(q, [k1, k2], [v1, v2])
    expect = math.e ** 2 / (math.e ** 2 + 1.0)
    assert np.allclose(out, expect, rtol=0, atol=1e-15)
    # a dropped 1/sqrt(d) would give e^4/(e^4+1); make sure the two differ visibly
    assert abs(expect - math.e ** 4 / (math.e ** 4 + 1.0)) > 0.1


def test_single_key_weight_is_one():
    q = rand(4, 8)
    k = rand(2, 8)
    v = rand(2, 8)
    out = po.attend(q, [k], [v])
    assert np.array_equal(out[0], v[0]) and np.array_equal(out[1], v[0])
    assert np.array_equal(out[2], v[1]) and np.array_equal(out[3], v[1])


def test_zero_query_gives_mean_of_values():
    n, H_kv, d = 13, 2, 8
    K, V = rand(n, H_kv, d), rand(n, H_kv, d)
    out = po.attend(np.zeros((4, d)), list(K), list(V))
    assert np.allclose(out[0], V[:, 0].mean(axis=0), atol=1e-15)
    assert np.allclose(out[3], V[:, 1].mean(axis=0), atol=1e-15)


def test_shift_of_all_keys_leaves_output_unchanged():
    n, d = 17, 8
    q, K, V = rand(2, d), rand(n, 1, d), rand(n, 1, d)
    w = rand(1, d) * 3.0
    a = po.attend(q, list(K), list(V))
    b = po.attend(q, list(K + w), list(V))
    assert np.allclose(a, b, atol=1e-13)


def test_permutation_of_cached_tokens_leaves_output_unchanged():
    n, d = 29, 16
    q, K, V = rand(4, d), rand(n, 2, d), rand(n, 2, d)
    perm = RNG.permutation(n)
    a = po.attend(q, list(K), list(V))
    b = po.attend(q, list(K[perm]), list(V[perm]))
    assert np.allclose(a, b, atol=1e-14)


def test_gqa_head_mapping():
    # 6 query heads over 3 KV heads: head h must read KV head h // 2 and nothing else.
    n, d = 9, 4
    q, K, V = rand(6, d), rand(n, 3, d), rand(n, 3, d)
    base = po.attend(q, list(K), list(V))
    V2 = V.copy()
    V2[:, 1, :] += 1.0
    out = po.attend(q, list(K), list(V2))
    changed = [not np.allclose(out[h], base[h]) for h in range(6)]
    assert changed == [False, False, True, True, False, False]
    # softmax weights sum to one => adding 1 to every value of the head adds exactly 1
    assert np.allclose(out[2] - base[2], 1.0, atol=1e-14)


@pytest.mark.parametrize("n,d", [(1, 1), (2, 3), (5, 4), (8, 2)])
def test_tiny_cases_against_naive_exponentials(n, d):
    # brute force in pure Python, no max subtraction
    q, K, V = rand(1, d), rand(n, 1, d), rand(n, 1, d)
    out = po.attend(q, list(K), list(V))
    e = []
    for j in range(n):
        s = sum(q[0][i] * K[j][0][i] for i in range(d)) / math.sqrt(d)
        e.append(math.exp(s))
    Z = sum(e)
    for i in range(d):
        expect = sum(e[j] / Z * V[j][0][i] for j in range(n))
        assert abs(out[0][i] - expect) < 1e-14


def test_peaky_scores_against_logsumexp():
    # scores spread over hundreds of units: exercises the max-subtraction path
    n, d = 64, 16
    q, K, V = rand(2, d) * 32.0, rand(n, 1, d) * 4.0, rand(n, 1, d)
    out = po.attend(q, list(K), list(V))
    for h in range(2):
        s = K[:, 0, :] @ q[h] / math.sqrt(d)
        assert s.max() - s.min() > 100
        w = np.exp(s - logsumexp(s))
        assert np.allclose(out[h], w @ V[:, 0, :], rtol=1e-12, atol=1e-14)


def test_custom_softmax_scale():
    n, d = 6, 4
    q, K, V = rand(1, d), rand(n, 1, d), rand(n, 1, d)
    out = po.attend(q, list(K), list(V), scale=0.37)
    w = softmax(K[:, 0, :] @ q[0] * 0.37)
    assert np.allclose(out[0], w @ V[:, 0, :], atol=1e-15)


def test_empty_window_gives_zeros():
    assert np.array_equal(po.attend(rand(2, 4), [], []), np.zeros((2, 4)))


# ---------------------------------------------------------------------------------------------
# the encoding (Our Approach: S' = ((q_g W^a_Q)(K_e W^a_K)^T)(V_e W^a_V))
# ---------------------------------------------------------------------------------------------

def test_encode_hand_worked_integers():
    # Q_a = I_2, W^a_K = W^a_V = I_2, K_e = [[1,2],[3,4]], V_e = [[5,6],[7,8]].
    # Q_a K_e^T = [[1,3],[2,4]]; times V_e = [[1*5+3*7, 1*6+3*8], [2*5+4*7, 2*6+4*8]] = [[26,30],[38,44]].
    I = np.eye(2)
    K = np.array([[1.0, 2], [3, 4]])
    V = np.array([[5.0, 6], [7, 8]])
    S = po.encode_chunk(I, K, V, I, I)
    assert np.array_equal(S, np.array([[26.0, 30], [38, 44]]))
    # the transposed-operand mistake would give K_e V_e = [[19,22],[43,50]]
    assert not np.array_equal(S, K @ V)


def test_encode_uses_key_and_value_projections_separately():
    # W^a_K = diag(1,0) keeps only the first key coordinate, W^a_V = diag(0,1) only the second value
    # coordinate: S'[g, :] = (sum_j Q_a[g,0] K[j,0] V[j,1]) * e_2.
    Q = np.array([[2.0, 5.0]])
    K = np.array([[1.0, 9.0], [3.0, 9.0]])
    V = np.array([[7.0, 10.0], [7.0, 100.0]])
    S = po.encode_chunk(Q, K, V, np.diag([1.0, 0.0]), np.diag([0.0, 1.0]))
    assert np.array_equal(S, np.array([[0.0, 2 * 1 * 10 + 2 * 3 * 100]]))


def _rand_encoder(G=5, r=4, d_q=12, d_kv=6, m=7):
    return dict(q_g=rand(G, d_q), WaQ=rand(d_q, r), WaK=rand(d_kv, r), WaV=rand(d_kv, r),
                K=rand(m, d_kv), V=rand(m, d_kv))


def test_encode_is_a_sum_of_per_token_outer_products():
    p = _rand_encoder()
    Q_a = po.project_queries(p["q_g"], p["WaQ"])
    S = po.encode_chunk(Q_a, p["K"], p["V"], p["WaK"], p["WaV"])
    acc = np.zeros_like(S)
    for j in range(p["K"].shape[0]):
        k_a = p["K"][j] @ p["WaK"]
        v_a = p["V"][j] @ p["WaV"]
        acc += np.outer(Q_a @ k_a, v_a)                       # single-token closed form
        one = po.encode_chunk(Q_a, p["K"][j:j + 1], p["V"][j:j + 1], p["WaK"], p["WaV"])
        assert np.allclose(one, np.outer(Q_a @ k_a, v_a), atol=1e-13)
    assert np.allclose(S, acc, atol=1e-12)


def test_encode_permutation_invariance_and_reassociation():
    p = _rand_encoder(m=11)
    Q_a = po.project_queries(p["q_g"], p["WaQ"])
    S = po.encode_chunk(Q_a, p["K"], p["V"], p["WaK"], p["WaV"])
    perm = RNG.permutation(11)
    S2 = po.encode_chunk(Q_a, p["K"][perm], p["V"][perm], p["WaK"], p["WaV"])
    assert np.allclose(S, S2, atol=1e-12)
    K_a, V_a = p["K"] @ p["WaK"], p["V"] @ p["WaV"]
    assert np.allclose(S, Q_a @ (K_a.T @ V_a), atol=1e-12)
    assert np.allclose(S, np.einsum("gi,mi,mj->gj", Q_a, K_a, V_a), atol=1e-12)


def test_encode_brute_force_loops():
    G, r, d_q, d_kv, m = 2, 3, 4, 2, 3
    p = _rand_encoder(G, r, d_q, d_kv, m)
    Q_a = po.project_queries(p["q_g"], p["WaQ"])
    S = po.encode_chunk(Q_a, p["K"], p["V"], p["WaK"], p["WaV"])
    for g, c in itertools.product(range(G), range(r)):
        tot = 0.0
        for j in range(m):
            qa = [sum(p["q_g"][g][x] * p["WaQ"][x][a] for x in range(d_q)) for a in range(r)]
            ka = [sum(p["K"][j][x] * p["WaK"][x][a] for x in range(d_kv)) for a in range(r)]
            va = sum(p["V"][j][x] * p["WaV"][x][c] for x in range(d_kv))
            tot += sum(qa[a] * ka[a] for a in range(r)) * va
        assert abs(S[g][c] - tot) < 1e-12


def test_encode_zero_values_give_zero_state():
    p = _rand_encoder()
    Q_a = po.project_queries(p["q_g"], p["WaQ"])
    assert np.array_equal(po.encode_chunk(Q_a, p["K"], np.zeros_like(p["V"]), p["WaK"], p["WaV"]),
                          np.zeros((5, 4)))


def test_init_state_is_encoding_of_global_tokens_unnormalised():
    p = _rand_encoder()
    k_g, v_g = rand(5, 6), rand(5, 6)
    Q_a, S0 = po.init_state(p["q_g"], p["WaQ"], p["WaK"], p["WaV"], k_g, v_g)
    assert np.allclose(Q_a, p["q_g"] @ p["WaQ"], atol=0)
    expect = np.linalg.multi_dot([Q_a, (k_g @ p["WaK"]).T, v_g @ p["WaV"]])
    assert np.allclose(S0, expect, atol=1e-12)
    assert abs(np.linalg.norm(S0) - 1.0) > 1e-3          # not normalised
    _, Z = po.init_state(p["q_g"], p["WaQ"], p["WaK"], p["WaV"])
    assert Z.shape == (5, 4) and not Z.any()


# ---------------------------------------------------------------------------------------------
# the state as a weight delta (Our Approach: Delta-W = A S B, theta' = theta + Delta-W)
# ---------------------------------------------------------------------------------------------

def test_apply_delta_hand_worked_and_structure():
    # x = (1, 2), A = [[1, 0], [0, 1]], S = [[0, 1], [2, 0]], B = [[1, 1, 0], [0, 1, 1]], y = (10, 20, 30):
    # x A = (1, 2); (x A) S = (2*2, 1*1) = (4, 1); ((x A) S) B = (4, 4 + 1, 1) = (4, 5, 1) => y' = (14, 25, 31)
    x, A = np.array([1.0, 2.0]), np.eye(2)
    S, B = np.array([[0.0, 1.0], [2.0, 0.0]]), np.array([[1.0, 1.0, 0.0], [0.0, 1.0, 1.0]])
    y = np.array([10.0, 20.0, 30.0])
    assert np.array_equal(po.apply_delta(x, A, S, B, y), np.array([14.0, 25.0, 31.0]))
    # transposing S would give (x A) S^T = (2, 2) -> (2, 4, 2): visibly different
    assert not np.array_equal(po.apply_delta(x, A, S.T, B, y), np.array([14.0, 25.0, 31.0]))
    # random shapes: left-to-right evaluation, zero state, linearity in S, brute force
    d_in, G, r, d_out = 7, 3, 4, 5
    x, A, S, B, y = rand(d_in), rand(d_in, G), rand(G, r), rand(r, d_out), rand(d_out)
    out = po.apply_delta(x, A, S, B, y)
    assert np.allclose(out, y + ((x @ A) @ S) @ B, atol=1e-12)
    assert np.array_equal(po.apply_delta(x, A, np.zeros((G, r)), B, y), y)
    assert np.allclose(po.apply_delta(x, A, 3.0 * S, B, y) - y, 3.0 * (out - y), atol=1e-12)
    for j in range(d_out):
        tot = sum(x[i] * A[i][g] * S[g][c] * B[c][j] for i in range(d_in) for g in range(G) for c in range(r))
        assert abs(out[j] - y[j] - tot) < 1e-12


# ---------------------------------------------------------------------------------------------
# Normalize (Our Approach: S <- Normalize(S + S')) -- the choice of norm is parity-unpinned
# ---------------------------------------------------------------------------------------------

def test_normalize_frobenius():
    X = np.array([[3.0, 0.0], [0.0, 4.0]])
    assert np.allclose(po.normalize(X), X / 5.0, atol=1e-16)
    Y = rand(6, 5) * 37.0
    N = po.normalize(Y)
    assert abs(np.linalg.norm(N) - 1.0) < 1e-14
    assert np.allclose(po.normalize(N), N, atol=1e-15)                # idempotent
    assert np.allclose(po.normalize(Y * 12.5), N, atol=1e-14)         # scale invariant
    assert np.array_equal(po.normalize(np.zeros((2, 2))), np.zeros((2, 2)))   # eps guard


def test_normalize_row_and_none():
    X = np.array([[3.0, 4.0], [0.0, 2.0]])
    assert np.allclose(po.normalize(X, po.NORM_ROW_L2), [[0.6, 0.8], [0.0, 1.0]], atol=1e-16)
    assert np.array_equal(po.normalize(X, po.NORM_NONE), X)


# ---------------------------------------------------------------------------------------------
# the bounded-window layer: window >= sequence is full causal attention; otherwise it is
# attention over the last n_live tokens; eviction is oldest-first in chunks; the state streams.
# ---------------------------------------------------------------------------------------------

def _layer(B, H_q, H_kv, d, W, C, G=3, r=4, norm=po.NORM_FROBENIUS, with_global=True, keep=False):
    enc = dict(q_g=rand(G, H_q * d), WaQ=rand(H_q * d, r), WaK=rand(H_kv * d, r), WaV=rand(H_kv * d, r))
    if with_global:
        enc.update(k_g=rand(G, H_kv * d), v_g=rand(G, H_kv * d))
    return po.OracleLayer(B, H_q, H_kv, d, W, C, norm_mode=norm, keep_chunks=keep, **enc), enc


def test_window_at_least_sequence_is_full_causal_attention():
    B, H_q, H_kv, d, T = 2, 4, 2, 8, 20
    layer, _ = _layer(B, H_q, H_kv, d, W=T, C=5)
    q, k, v = rand(T, B, H_q, d), rand(T, B, H_kv, d), rand(T, B, H_kv, d)
    for t in range(T):
        out = layer.step(q[t], k[t], v[t])
        for b in range(B):
            expect = direct_attention(q[t, b], k[:t + 1, b], v[:t + 1, b], H_q // H_kv)
            assert np.allclose(out[b], expect, atol=1e-13)
    ln, base = layer.counters()
    assert (ln == T).all() and (base == 0).all()
    assert np.array_equal(layer.state(), np.stack([layer.S0] * B))      # nothing evicted, S untouched


@pytest.mark.parametrize("W,C", [(8, 2), (8, 3), (7, 7), (5, 1), (16, 4)])
def test_bounded_window_is_attention_over_last_tokens_and_evicts_oldest_first(W, C):
    B, H_q, H_kv, d, T = 2, 2, 1, 4, 3 * W + 5
    layer, enc = _layer(B, H_q, H_kv, d, W, C, norm=po.NORM_NONE, with_global=False, keep=True)
    ring = RingModel(B, W, C)
    q, k, v = rand(T, B, H_q, d), rand(T, B, H_kv, d), rand(T, B, H_kv, d)
    for t in range(1, T + 1):
        out = layer.step(q[t - 1], k[t - 1], v[t - 1])
        ring.step()
        n_live = n_live_closed_form(t, W, C)
        E = evicted_closed_form(t, W, C)
        ln, base = layer.counters()
        assert (ln == t).all() and (base == E).all() and n_live == t - E
        assert (ring.len == t).all() and (ring.base == E).all()
        for b in range(B):
            Kw, Vw = layer.window_kv(b)
            assert np.array_equal(Kw, k[E:t, b]) and np.array_equal(Vw, v[E:t, b])
            expect = direct_attention(q[t - 1, b], k[E:t, b], v[E:t, b], H_q // H_kv)
            assert np.allclose(out[b], expect, atol=1e-13)
            # the ring model's live slots hold exactly positions E..t-1
            assert np.array_equal(ring.slot_pos[b, ring.live_slots(b)], np.arange(E, t))
    # eviction order: the i-th chunk is positions [i*C, (i+1)*C), heads concatenated
    for b in range(B):
        chunks = layer.rollouts[b].evicted_chunks
        assert len(chunks) == E // C
        for i, (K_e, V_e) in enumerate(chunks):
            assert np.array_equal(K_e, k[i * C:(i + 1) * C, b].reshape(C, -1))
            assert np.array_equal(V_e, v[i * C:(i + 1) * C, b].reshape(C, -1))
            assert np.array_equal(ring.evictions[b][i], np.arange(i * C, (i + 1) * C) % W)
    # streaming state with no normalisation and S_0 = 0 is the one-shot linear-attention state of
    # everything evicted so far, independent of how it was chunked
    Q_a = enc["q_g"] @ enc["WaQ"]
    for b in range(B):
        K_all = k[:E, b].reshape(E, -1) @ enc["WaK"]
        V_all = v[:E, b].reshape(E, -1) @ enc["WaV"]
        assert np.allclose(layer.rollouts[b].S, Q_a @ (K_all.T @ V_all), rtol=1e-10, atol=1e-10)


def test_state_update_normalises_after_every_eviction_and_starts_from_S0():
    B, H_q, H_kv, d, W, C = 1, 2, 2, 4, 6, 2
    layer, enc = _layer(B, H_q, H_kv, d, W, C)
    T = 11
    q, k, v = rand(T, B, H_q, d), rand(T, B, H_kv, d), rand(T, B, H_kv, d)
    Q_a = enc["q_g"] @ enc["WaQ"]
    # the starting state, by an independent route: the global tokens' own encoding, NOT normalised
    S = np.linalg.multi_dot([Q_a, (enc["k_g"] @ enc["WaK"]).T, enc["v_g"] @ enc["WaV"]])
    assert np.allclose(layer.rollouts[0].S, S, atol=1e-13) and abs(np.linalg.norm(S) - 1.0) > 1e-3
    for t in range(T):
        before = layer.rollouts[0].evicted
        layer.step(q[t], k[t], v[t])
        after = layer.rollouts[0].evicted
        if after != before:
            K_e = k[before:after, 0].reshape(C, -1)
            V_e = v[before:after, 0].reshape(C, -1)
            S = S + np.linalg.multi_dot([Q_a, (K_e @ enc["WaK"]).T, V_e @ enc["WaV"]])
            S = S / np.linalg.norm(S)
            assert abs(np.linalg.norm(layer.rollouts[0].S) - 1.0) < 1e-14
        assert np.allclose(layer.rollouts[0].S, S, atol=1e-13)
    assert layer.rollouts[0].evicted == 6          # steps 7, 9, 11 each evicted 2


def test_inactive_rollouts_are_untouched_and_return_zeros():
    B, H_q, H_kv, d, W, C = 3, 2, 1, 4, 4, 2
    layer, _ = _layer(B, H_q, H_kv, d, W, C)
    T = 9
    q, k, v = rand(T, B, H_q, d), rand(T, B, H_kv, d), rand(T, B, H_kv, d)
    lengths = np.array([9, 3, 0])
    for t in range(T):
        act = (t < lengths).astype(np.uint8)
        out = layer.step(q[t], k[t], v[t], act)
        assert not out[2].any()
        if t >= 3:
            assert not out[1].any()
    ln, base = layer.counters()
    assert ln.tolist() == [9, 3, 0] and base.tolist() == [6, 0, 0]


# ---------------------------------------------------------------------------------------------
# pinned question tokens ("The selection of D during training": question tokens are kept for good,
# only thinking tokens slide; e.g. a cache of 768 = 512 sink tokens + 256 in the sliding window)
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("W,n_sink,C,P", [(12, 4, 3, (4, 2)), (10, 6, 4, (0, 6)), (9, 1, 8, (1, 1))])
def test_question_tokens_stay_and_only_thinking_tokens_slide(W, n_sink, C, P):
    B, H_q, H_kv, d = 2, 4, 2, 4
    R = W - n_sink
    T = 3 * R + 4
    enc = dict(q_g=rand(3, H_q * d), WaQ=rand(H_q * d, 5), WaK=rand(H_kv * d, 5), WaV=rand(H_kv * d, 5),
               k_g=rand(3, H_kv * d), v_g=rand(3, H_kv * d))
    layer = po.OracleLayer(B, H_q, H_kv, d, W, C, n_sink=n_sink, keep_chunks=True, **enc)
    plain = po.OracleLayer(B, H_q, H_kv, d, R, C, keep_chunks=True, **enc)     # no question tokens, window R
    pk = [rand(P[b], H_kv, d) for b in range(B)]
    pv = [rand(P[b], H_kv, d) for b in range(B)]
    for b in range(B):
        layer.prefill(b, pk[b], pv[b])
    assert layer.prompt_lengths().tolist() == list(P)
    q, k, v = rand(T, B, H_q, d), rand(T, B, H_kv, d), rand(T, B, H_kv, d)
    for t in range(1, T + 1):
        out = layer.step(q[t - 1], k[t - 1], v[t - 1])
        plain.step(q[t - 1], k[t - 1], v[t - 1])
        E = evicted_closed_form(t, R, C)
        assert n_live_closed_form(t, R, C) == t - E
        for b in range(B):
            Kall = np.concatenate([pk[b], k[E:t, b]])
            Vall = np.concatenate([pv[b], v[E:t, b]])
            assert np.allclose(out[b], direct_attention(q[t - 1, b], Kall, Vall, H_q // H_kv), atol=1e-13)
            Kw, Vw = layer.window_kv(b)
            assert np.array_equal(Kw, Kall) and np.array_equal(Vw, Vall)
    # eviction schedule, evicted chunks and the state are those of the plain window of R thinking tokens
    assert np.array_equal(layer.counters()[0], plain.counters()[0])
    assert np.array_equal(layer.counters()[1], plain.counters()[1])
    assert np.array_equal(layer.state(), plain.state())
    for b in range(B):
        for (Ka, Va), (Kb, Vb) in zip(layer.rollouts[b].evicted_chunks, plain.rollouts[b].evicted_chunks):
            assert np.array_equal(Ka, Kb) and np.array_equal(Va, Vb)
    with pytest.raises(AssertionError):
        layer.prefill(0, rand(n_sink + 1, H_kv, d), rand(n_sink + 1, H_kv, d))


def test_a_reset_rollout_behaves_like_a_fresh_one_and_leaves_the_others_alone():
    B, H_q, H_kv, d, W, C = 2, 2, 1, 3, 7, 2
    layer, enc = _layer(B, H_q, H_kv, d, W, C)
    fresh, _ = _layer(1, H_q, H_kv, d, W, C)
    fresh.__init__(1, H_q, H_kv, d, W, C, enc["q_g"], enc["WaQ"], enc["WaK"], enc["WaV"], enc["k_g"], enc["v_g"])
    Q, K, V = rand(20, B, H_q, d), rand(20, B, H_kv, d), rand(20, B, H_kv, d)
    for t in range(11):
        layer.step(Q[t], K[t], V[t])
    S_other = layer.state()[0].copy()
    n_other = layer.counters()[0][0]
    layer.reset_rollout(1)
    assert layer.counters()[0][1] == 0 and layer.counters()[1][1] == 0 and np.array_equal(layer.state()[1], layer.S0)
    assert layer.counters()[0][0] == n_other and np.array_equal(layer.state()[0], S_other)
    for t in range(11, 20):
        out = layer.step(Q[t], K[t], V[t])
        ref = fresh.step(Q[t][1:], K[t][1:], V[t][1:])
        assert np.allclose(out[1], ref[0], atol=1e-14)
    assert np.allclose(layer.state()[1], fresh.state()[0], atol=1e-14)


def test_ring_model_with_reserved_question_slots():
    ring = RingModel(1, 12, 3, n_sink=4)
    slots = [int(ring.step()[0]) for _ in range(20)]
    assert slots[:9] == [4, 5, 6, 7, 8, 9, 10, 11, 4]                 # ring of 8 behind 4 reserved slots
    assert ring.base[0] == 3 * -(-(20 - 8) // 3) and min(slots) >= 4
    assert ring.evictions[0][0].tolist() == [4, 5, 6]
    assert ring.live_slots(0).tolist() == [4 + p % 8 for p in range(int(ring.base[0]), 20)]


# ---------------------------------------------------------------------------------------------
# ring model against a brute-force deque, incl. C not dividing W, C = 1, C = W, rotated start
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("W,C,start", [(8, 3, 0), (8, 8, 0), (5, 1, 0), (6, 4, 13), (16, 4, 7)])
def test_ring_model_against_deque(W, C, start):
    from collections import deque
    ring = RingModel(1, W, C, start=start)
    dq = deque()
    store = {}
    for t in range(5 * W):
        if len(dq) == W:
            ev = [dq.popleft() for _ in range(C)]
            assert ring.evict()[0] == 1
            assert np.array_equal(ring.evictions[0][-1], np.array([(p + start) % W for p in ev]))
        else:
            assert ring.evict()[0] == 0
        slot = ring.append()[0]
        assert slot == (t + start) % W
        store[slot] = t
        dq.append(t)
        assert [store[s] for s in ring.live_slots(0)] == list(dq)
        assert ring.n_live()[0] == len(dq) == n_live_closed_form(t + 1, W, C)


def test_closed_forms_small_table():
    # W = 4, C = 2: live counts seen by attention at steps 1..9 and cumulative evictions
    assert [n_live_closed_form(t, 4, 2) for t in range(1, 10)] == [1, 2, 3, 4, 3, 4, 3, 4, 3]
    assert [evicted_closed_form(t, 4, 2) for t in range(1, 10)] == [0, 0, 0, 0, 2, 2, 4, 4, 6]
    # the Llama-shaped run: 16 384 steps, window 8 192, chunk 256 -> 8 192 tokens evicted
    assert evicted_closed_form(16384, 8192, 256) == 8192
