"""Pins of the oracle's teacher scores (KVzip, Eq. 1; KVzip+, Eq. 3), CPU only."""
import numpy as np
from scipy.special import softmax

from oracle import kvzap_oracle as O


def _case(rng, H=2, G=2, T=6, instr=3, D=8, gain=1.0):
    Tq, Tk = T, T + instr + T
    q = rng.standard_normal((H * G, Tq, D)) * gain
    k = rng.standard_normal((H, Tk, D))
    return q, k, T


def test_uniform_attention_closed_form():
    # zero queries: a_ji = 1 / (P0 + j + 1), largest for the first repeated token
    rng = np.random.default_rng(0)
    q, k, T = _case(rng)
    q[:] = 0.0
    P0 = k.shape[1] - q.shape[1]
    got = O.teacher_log_scores(q, k, 0.3, T)
    assert np.allclose(got, -np.log(P0 + 1.0), atol=1e-12)
    vn = rng.uniform(0.5, 2.0, (2, T)); hn = rng.uniform(0.5, 2.0, q.shape[1])
    got = O.teacher_log_scores(q, k, 0.3, T, vn, hn)
    want = np.log(vn) + np.max(-np.log(P0 + 1.0 + np.arange(q.shape[1])) - np.log(hn))
    assert np.allclose(got, want, atol=1e-12)


def test_equals_a_plain_softmax_matrix_and_a_hand_loop():
    rng = np.random.default_rng(1)
    q, k, T = _case(rng, gain=2.0)
    HQ, Tq, D = q.shape
    H, Tk, _ = k.shape
    G, P0, scale = HQ // H, Tk - Tq, 0.25
    vn = rng.uniform(0.1, 3.0, (H, T)); hn = rng.uniform(0.5, 5.0, Tq)
    got = O.teacher_log_scores(q, k, scale, T, vn, hn)
    want = np.zeros((H, T))
    for h in range(H):
        for i in range(T):
            best = 0.0
            for g in range(h * G, (h + 1) * G):
                for j in range(Tq):
                    logits = [scale * float(q[g, j] @ k[h, ii]) for ii in range(P0 + j + 1)]
                    a = softmax(np.array(logits))
                    best = max(best, a[i] * vn[h, i] / hn[j])
            want[h, i] = best
    assert np.allclose(np.exp(got), want, rtol=1e-10)
    # Eq. 1 is the case of unit norms
    got1 = O.teacher_log_scores(q, k, scale, T)
    got2 = O.teacher_log_scores(q, k, scale, T, np.ones((H, T)), np.ones(Tq))
    assert np.array_equal(got1, got2)


def test_copy_task_gives_scores_near_one():
    # the repeated token j attends to its original i = j: one dominant key per query
    rng = np.random.default_rng(2)
    T, instr, D = 5, 2, 16
    k = rng.standard_normal((1, T + instr + T, D))
    q = 60.0 * k[:, :T].copy()                     # query j = a multiple of key j
    s = O.teacher_log_scores(q, k, 1.0, T)
    assert (np.exp(s) > 0.99).all() and (s <= 1e-12).all()


def test_invariances():
    rng = np.random.default_rng(3)
    q, k, T = _case(rng, H=2, G=3, gain=1.5)
    vn = rng.uniform(0.5, 2.0, (2, T)); hn = rng.uniform(0.5, 2.0, q.shape[1])
    base = O.teacher_log_scores(q, k, 0.2, T, vn, hn)
    # a common shift of all keys along q_j changes every logit of row j equally: no effect
    # (realised here by scaling vnorm / hnorm instead, whose effect is known in closed form)
    assert np.allclose(O.teacher_log_scores(q, k, 0.2, T, 3.0 * vn, hn), base + np.log(3.0))
    assert np.allclose(O.teacher_log_scores(q, k, 0.2, T, vn, 2.0 * hn), base - np.log(2.0))
    # the group maximum dominates every single query head, and equals the max of the singles
    singles = [O.teacher_log_scores(q[g:g + 1], k[g // 3:g // 3 + 1], 0.2, T, vn[g // 3:g // 3 + 1], hn)
               for g in range(6)]
    for h in range(2):
        assert np.allclose(base[h], np.max([singles[g][0] for g in range(3 * h, 3 * h + 3)], axis=0))
    # scores are attention weights: at most 1 before the norms
    assert (O.teacher_log_scores(q, k, 0.2, T) <= 1e-12).all()


def test_causality_future_keys_are_invisible():
    # rows j <= j0 must not depend on keys behind position P0 + j0: truncating the extended
    # prompt after query j0 gives the same scores as the full one with the later queries
    # silenced (huge ||h_j||) and the later keys replaced by anything
    rng = np.random.default_rng(4)
    q, k, T = _case(rng, H=1, G=2, T=7, instr=2, gain=2.0)
    Tq = q.shape[1]
    P0 = k.shape[1] - Tq
    for j0 in (0, 3, Tq - 2):
        short = O.teacher_log_scores(q[:, :j0 + 1], k[:, :P0 + j0 + 1], 0.3, T)
        k2 = k.copy()
        k2[:, P0 + j0 + 1:] = 50.0 * rng.standard_normal(k2[:, P0 + j0 + 1:].shape)
        hn = np.ones(Tq)
        hn[j0 + 1:] = 1e300
        full = O.teacher_log_scores(q, k2, 0.3, T, None, hn)
        assert np.allclose(short, full, atol=1e-12), j0
