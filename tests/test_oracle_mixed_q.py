"""Pins for the oracle when every component draws its own number of neighbours q_i (CPU only).

Algorithm 1's REQUIRE lines only bound q by 2p, and Section 3.3 picks a (p, q) pair per
deployment; the library lets q differ from component to component.  Expected values come
from outside the oracle: Section 2.2's statement that q = 2p uses every neighbour, the
statistics of a uniform choice without replacement, and dense row-stochastic matrices over
enumerated neighbour assignments.
"""
import itertools

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(19090910)


def _state(K, P, dtype=np.float64):
    w0 = RNG.normal(0, 0.05, size=P)
    theta = (w0 + RNG.normal(0, 0.01, size=(K, P))).astype(dtype)
    omega = np.broadcast_to(w0, (K, P)).astype(dtype).copy()
    delta = RNG.normal(0, 0.01, size=(K, P)).astype(dtype)
    return theta, omega, delta


def _dense_reference_q(off, nbr, q, theta, omega, delta, eta, zeta, mode):
    """Float64 statement of the sync branch, the average of component i as a dense matrix
    product with A_i[w, v] = 1/(q_i + 1) for v in {w} + the first q_i entries of nbr[i, w]."""
    m, K, _ = nbr.shape
    th, om, de = theta.copy(), omega.copy(), delta.copy()
    for i in range(m):
        A = np.zeros((K, K))
        for w in range(K):
            A[w, w] += 1.0
            for v in nbr[i, w, :q[i]]:
                A[w, v] += 1.0
        assert (A.sum(axis=1) == q[i] + 1).all() and A.max() == 1.0
        A /= (q[i] + 1)
        sl = slice(off[i], off[i + 1])
        avg = A @ theta[:, sl]
        if mode == oracle.MODE_GOSSIP_MA:
            th[:, sl] = avg
            continue
        start = omega[:, sl] + eta * delta[:, sl] if mode == oracle.MODE_PAPER else omega[:, sl]
        G = avg - start
        de[:, sl] = eta * delta[:, sl] + zeta * G
        om[:, sl] = omega[:, sl] + de[:, sl]
        th[:, sl] = om[:, sl] if mode == oracle.MODE_NO_RESTART else om[:, sl] + eta * de[:, sl]
    return th, om, de


def _rows_of(K, p, qi):
    """every possible row of a component with qi neighbours, per worker"""
    return [list(itertools.combinations(sorted(oracle.ring_candidates(w, K, p).tolist()), qi)) for w in range(K)]


def test_rows_have_q_i_valid_entries_and_minus_one_beyond():
    K, p = 16, 3
    q = [0, 1, 2, 3, 6, 2, 0, 5]
    for rnd in (0, 3):
        t = oracle.neighbour_table(len(q), K, p, q, seed=77, round=rnd)
        assert t.shape == (len(q), K, 6)
        for i, qi in enumerate(q):
            assert (t[i, :, qi:] == -1).all()
            for w in range(K):
                row = t[i, w, :qi]
                cand = set(oracle.ring_candidates(w, K, p).tolist())
                assert (np.diff(row) > 0).all() and set(row.tolist()) <= cand and w not in row
    wide = oracle.neighbour_table(len(q), K, p, q, seed=77, round=3, width=9)
    assert wide.shape[2] == 9 and (wide[:, :, :6] == t).all() and (wide[:, :, 6:] == -1).all()


def test_components_with_q_equal_2p_take_all_neighbours_whatever_the_others_draw():
    # Section 2.2: with q = 2p every neighbour is included -- per component here
    for K, p in [(4, 1), (8, 2), (16, 3), (5, 3)]:
        C = len(oracle.ring_candidates(0, K, p))
        q = [C, 0, C, 1 if C > 1 else 0, C]
        for seed, rnd in [(0, 0), (2**63 + 1, 2**40)]:
            t = oracle.neighbour_table(len(q), K, p, q, seed, rnd)
            for i in (0, 2, 4):
                for w in range(K):
                    assert t[i, w, :C].tolist() == sorted(oracle.ring_candidates(w, K, p).tolist())


def test_each_component_is_uniform_at_its_own_q():
    # component i: every candidate with probability q_i / C (chi-square per q)
    K, p = 16, 3
    C = 2 * p
    reps = 1500
    qs = [1, 2, 3, 4, 5]
    q = np.array(qs * reps, dtype=np.int32)              # component i draws qs[i % 5]
    t = oracle.neighbour_table(len(q), K, p, q, seed=4242, round=9)
    pos = [{v: j for j, v in enumerate(oracle.ring_candidates(w, K, p).tolist())} for w in range(K)]
    for k, qi in enumerate(qs):
        cnt = np.zeros(C)
        for w in range(K):
            lut = np.full(K, -1)
            for v, j in pos[w].items():
                lut[v] = j
            np.add.at(cnt, lut[t[k::5, w, :qi]].ravel(), 1)
        exp = reps * K * qi / C
        chi2 = ((cnt - exp) ** 2 / exp).sum()
        assert cnt.sum() == reps * K * qi
        assert chi2 < 40.0, (qi, chi2)                   # 5 dof; sampling without replacement only shrinks it


def test_components_stay_independent_across_different_q():
    # Section 2.2, last paragraph: every component draws afresh.  Neighbouring components with
    # q = 1 and q = 2: the single pick is inside the pair with probability 2/C, as for
    # independent draws.
    K, p, m = 16, 3, 4000
    q = np.tile([1, 2], m // 2).astype(np.int32)
    t = oracle.neighbour_table(m, K, p, q, seed=5, round=1)
    inside = (t[0::2, :, :1] == t[1::2, :, :2]).any(axis=2).mean()
    assert abs(inside - 2 / 6) < 0.02, inside


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_brute_force_mixed_q_on_K4(mode):
    # K = 4, p = 2 (C = 3), components with q = (1, 2, 0, 3): every row of one component
    # enumerated (81 tables each for q = 1 and q = 2) while the others take seeded rows
    K, p = 4, 2
    q = [1, 2, 0, 3]
    off = np.array([0, 4, 9, 11, 16], dtype=np.int64)
    theta, omega, delta = _state(K, 16)
    eta, zeta = 0.9, 0.75
    rows = [_rows_of(K, p, qi) for qi in q]
    pick = np.random.default_rng(mode)
    n = 0
    for vary in (0, 1):
        for combo in itertools.product(*rows[vary]):
            nbr = np.full((4, K, 3), -1, dtype=np.int32)
            for i, qi in enumerate(q):
                for w in range(K):
                    r = combo[w] if i == vary else rows[i][w][pick.integers(len(rows[i][w]))]
                    nbr[i, w, :qi] = r
            want = _dense_reference_q(off, nbr, q, theta, omega, delta, eta, zeta, mode)
            got = [a.copy() for a in (theta, omega, delta)]
            oracle.sync_table(off, nbr, *got, eta, zeta, mode, q=q)
            for g, e in zip(got, want):
                np.testing.assert_allclose(g, e, rtol=1e-12, atol=1e-14)
            g32 = [a.astype(np.float32) for a in (theta, omega, delta)]
            oracle.sync_table(off, nbr, *g32, np.float32(eta), np.float32(zeta), mode, q=q)
            for g, e in zip(g32, want):
                np.testing.assert_allclose(g, e, rtol=1e-6, atol=1e-7)
            n += 1
    assert n == 162


def test_entries_beyond_q_i_are_ignored():
    K, p, q = 8, 2, [1, 3, 2]
    off = np.array([0, 7, 20, 31], dtype=np.int64)
    theta, omega, delta = _state(K, 31)
    nbr = oracle.neighbour_table(3, K, p, q, seed=3, round=0)
    junk = nbr.copy()
    for i, qi in enumerate(q):
        junk[i, :, qi:] = 12345                           # not even a worker id
    a = [x.copy() for x in (theta, omega, delta)]
    b = [x.copy() for x in (theta, omega, delta)]
    oracle.sync_table(off, nbr, *a, 0.9, 1.0, 1, q=q)
    oracle.sync_table(off, junk, *b, 0.9, 1.0, 1, q=q)
    for x, y in zip(a, b):
        assert (x == y).all()


def test_multi_round_sampled_mixed_q_against_the_dense_reference():
    K, p = 16, 3
    q = [2, 6, 0, 3, 1]
    off = np.array([0, 5, 5, 40, 41, 64], dtype=np.int64)
    theta, omega, delta = _state(K, 64)
    ref = [x.copy() for x in (theta, omega, delta)]
    got = [x.copy() for x in (theta, omega, delta)]
    for r in range(6):
        nbr = oracle.neighbour_table(5, K, p, q, seed=11, round=r)
        ref = list(_dense_reference_q(off, nbr, q, *ref, 0.9, 1.0, 1))
        oracle.sync(off, K, p, q, 11, r, *got, 0.9, 1.0, 1)
    for g, e in zip(got, ref):
        np.testing.assert_allclose(g, e, rtol=1e-11, atol=1e-13)


def test_mixed_q_rejects_bad_arguments():
    K, p = 8, 2
    off = np.array([0, 4, 8], dtype=np.int64)
    theta, omega, delta = _state(K, 8)
    with pytest.raises(ValueError):
        oracle.neighbour_table(2, K, p, [1, 5], seed=0, round=0)          # q_i <= 2p
    with pytest.raises(ValueError):
        oracle.neighbour_table(2, K, p, [1, -1], seed=0, round=0)
    with pytest.raises(ValueError):
        oracle.neighbour_table(2, K, p, [1, 3], seed=0, round=0, width=2)  # rows too short
    nbr = oracle.neighbour_table(2, K, p, [1, 3], seed=0, round=0)
    bad = nbr.copy()
    bad[1, 0, 2] = K
    with pytest.raises(ValueError):
        oracle.sync_table(off, bad, theta, omega, delta, 0.9, 1.0, 1, q=[1, 3])
    with pytest.raises(ValueError):
        oracle.sync_table(off, nbr, theta, omega, delta, 0.9, 1.0, 1, q=[1, 4])
