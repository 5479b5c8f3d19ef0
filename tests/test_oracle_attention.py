"""Pins for the oracle's ragged decode attention (closed forms, a hand loop, a library
softmax, invariances)."""
import math
import random

import numpy as np
from scipy import special

from oracle import kvzap_oracle as O


def _caches(rng, B, H, D, lens):
    return [[(rng.standard_normal((lens[b][h], D)), rng.standard_normal((lens[b][h], D)))
             for h in range(H)] for b in range(B)]


def test_zero_query_gives_mean_of_values():
    rng = np.random.default_rng(0)
    c = _caches(rng, 2, 2, 8, [[5, 1], [9, 3]])
    out = O.attend_decode(np.zeros((2, 4, 8)), c, 0.3)
    for b in range(2):
        for g in range(4):
            np.testing.assert_allclose(out[b, g], c[b][g // 2][1].mean(axis=0), atol=1e-14)


def test_dominant_key_selects_its_value_and_single_row():
    rng = np.random.default_rng(1)
    D = 6
    K = rng.standard_normal((7, D)); V = rng.standard_normal((7, D))
    q = rng.standard_normal(D)
    K[4] = 50.0 * q / np.dot(q, q)            # score 50 vs O(1) for the others
    out = O.attend_decode(q[None, None, :], [[(K, V)]], 1.0)
    assert np.abs(out[0, 0] - V[4]).max() < 1e-12 * 1e6   # weight of the rest ~ e^-45
    one = O.attend_decode(q[None, None, :], [[(K[:1], V[:1])]], 1.0)
    np.testing.assert_array_equal(one[0, 0], V[0])


def test_against_hand_loop_and_library_softmax():
    rnd = random.Random(5)
    D, n = 4, 6
    K = [[rnd.uniform(-1, 1) for _ in range(D)] for _ in range(n)]
    V = [[rnd.uniform(-1, 1) for _ in range(D)] for _ in range(n)]
    q = [rnd.uniform(-1, 1) for _ in range(D)]
    scale = 1.0 / math.sqrt(D)
    s = [scale * sum(q[d] * K[i][d] for d in range(D)) for i in range(n)]
    z = sum(math.exp(x) for x in s)
    want = [sum(math.exp(s[i]) / z * V[i][d] for i in range(n)) for d in range(D)]
    out = O.attend_decode(np.array(q)[None, None, :], [[(np.array(K), np.array(V))]], scale)
    np.testing.assert_allclose(out[0, 0], want, atol=1e-15)
    lib = special.softmax(np.array(s)) @ np.array(V)
    np.testing.assert_allclose(out[0, 0], lib, atol=1e-15)


def test_row_order_and_score_shift_invariance_and_gqa_mapping():
    rng = np.random.default_rng(2)
    B, H, G, D = 2, 3, 2, 8
    lens = [[4, 7, 2], [3, 3, 9]]
    c = _caches(rng, B, H, D, lens)
    q = rng.standard_normal((B, H * G, D))
    ref = O.attend_decode(q, c, 0.25)
    perm = [[(K[::-1].copy(), V[::-1].copy()) for K, V in row] for row in c]
    np.testing.assert_allclose(O.attend_decode(q, perm, 0.25), ref, atol=1e-14)
    # adding a constant vector u to every key shifts all scores of a head by q.u: no change
    u = rng.standard_normal(D)
    shifted = [[(K + u[None, :], V) for K, V in row] for row in c]
    np.testing.assert_allclose(O.attend_decode(q, shifted, 0.25), ref, atol=1e-12)
    # query heads 2h and 2h+1 read KV head h: swapping two KV heads swaps the outputs' sources
    swapped = [[row[1], row[0], row[2]] for row in c]
    q2 = q.copy(); q2[:, [0, 1, 2, 3]] = q[:, [2, 3, 0, 1]]
    out2 = O.attend_decode(q2, swapped, 0.25)
    np.testing.assert_allclose(out2[:, [2, 3, 0, 1]], ref[:, [0, 1, 2, 3]], atol=1e-14)


def test_pruned_cache_with_tau_minus_inf_equals_full_attention():
    # keeping everything (tau = -inf) and attending over the compacted rows is plain attention
    rng = np.random.default_rng(3)
    B, H, T, D = 1, 2, 30, 4
    S = rng.standard_normal((B, H, T))
    Kf = rng.standard_normal((B, H, T, D)); Vf = rng.standard_normal((B, H, T, D))
    r = O.prune(S, -np.inf, 5)
    c = [[(Kf[0, h][r.idx[0][h]], Vf[0, h][r.idx[0][h]]) for h in range(H)]]
    q = rng.standard_normal((B, H, D))
    out = O.attend_decode(q, c, 0.5)
    for h in range(H):
        w = special.softmax(0.5 * Kf[0, h] @ q[0, h])
        np.testing.assert_allclose(out[0, h], w @ Vf[0, h], atol=1e-14)
