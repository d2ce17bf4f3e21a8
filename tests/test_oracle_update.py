"""Pins for the oracle's averaging and block-momentum arithmetic (CPU only).

Nothing here calls the oracle to produce an expected value: expectations come from dense
row-stochastic matrices enumerated over every neighbour assignment, from a textbook
scalar-state BMUF-NBM loop, from closed forms and from invariants of Algorithm 1.
"""
import itertools

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(20190909)


def _state(K, P, stride=None, dtype=np.float64, delta_scale=0.01):
    stride = P if stride is None else stride
    w0 = RNG.normal(0, 0.05, size=stride)
    theta = (w0 + RNG.normal(0, 0.01, size=(K, stride))).astype(dtype)
    omega = np.broadcast_to(w0, (K, stride)).astype(dtype).copy()
    delta = RNG.normal(0, delta_scale, size=(K, stride)).astype(dtype)
    return theta, omega, delta


def _dense_reference(off, nbr, theta, omega, delta, eta, zeta, mode):
    """Float64 statement of Algorithm 1's sync branch with the average as a dense matrix
    product: A_i[w, v] = 1/(q+1) for v in {w} + neighbours(w, i)."""
    m, K, q = nbr.shape
    th, om, de = theta.copy(), omega.copy(), delta.copy()
    for i in range(m):
        A = np.zeros((K, K))
        for w in range(K):
            A[w, w] += 1.0
            for v in nbr[i, w]:
                A[w, v] += 1.0
        assert (A.sum(axis=1) == q + 1).all() and A.max() == 1.0
        A /= (q + 1)
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


def _all_tables(K, p, q, m):
    per_worker = [list(itertools.combinations(sorted(oracle.ring_candidates(w, K, p).tolist()), q))
                  for w in range(K)]
    slots = [per_worker[w] for _ in range(m) for w in range(K)]
    for combo in itertools.product(*slots):
        yield np.array(combo, dtype=np.int32).reshape(m, K, q)


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_brute_force_every_neighbour_assignment_K4(mode):
    # K=4, p=1, q=1, m=2: 2 choices per (component, worker) -> 2^8 = 256 tables
    K, p, q = 4, 1, 1
    off = np.array([0, 5, 12], dtype=np.int64)
    theta, omega, delta = _state(K, 12)
    eta, zeta = 0.9, 0.75
    n = 0
    for nbr in _all_tables(K, p, q, 2):
        want = _dense_reference(off, nbr, theta, omega, delta, eta, zeta, mode)
        t64, o64, d64 = theta.copy(), omega.copy(), delta.copy()
        oracle.sync_table(off, nbr, t64, o64, d64, eta, zeta, mode)
        for got, exp in zip((t64, o64, d64), want):
            np.testing.assert_allclose(got, exp, rtol=1e-12, atol=1e-14)
        t32, o32, d32 = (a.astype(np.float32) for a in (theta, omega, delta))
        oracle.sync_table(off, nbr, t32, o32, d32, np.float32(eta), np.float32(zeta), mode)
        for got, exp in zip((t32, o32, d32), want):
            np.testing.assert_allclose(got, exp, rtol=1e-6, atol=1e-7)
        n += 1
    assert n == 256


@pytest.mark.parametrize("K,p,q,m", [(3, 1, 2, 2), (4, 2, 2, 1), (4, 2, 3, 2), (2, 1, 1, 3), (4, 1, 0, 2)])
def test_brute_force_other_small_shapes(K, p, q, m):
    off = np.cumsum([0] + [3 + 2 * i for i in range(m)]).astype(np.int64)
    theta, omega, delta = _state(K, int(off[-1]), stride=int(off[-1]) + 3)
    keep = [a.copy() for a in (theta, omega, delta)]
    for nbr in itertools.islice(_all_tables(K, p, q, m), 300):
        for mode in (0, 1, 2, 3):
            want = _dense_reference(off, nbr, theta, omega, delta, 0.8, 1.0, mode)
            got = [a.copy() for a in (theta, omega, delta)]
            oracle.sync_table(off, nbr, *got, 0.8, 1.0, mode)
            for g, e in zip(got, want):
                np.testing.assert_allclose(g, e, rtol=1e-12, atol=1e-14)
            # the padding between P and stride is never touched
            for g, k in zip(got, keep):
                assert (g[:, off[-1]:] == k[:, off[-1]:]).all()


def test_multi_round_brute_force_with_sampled_tables():
    # several rounds, tables drawn by the sampler, dense reference carried along
    K, p, q = 4, 1, 1
    off = np.array([0, 4, 4, 9, 20], dtype=np.int64)      # includes an empty component
    theta, omega, delta = _state(K, 20, delta_scale=0.0)
    ref = [a.copy() for a in (theta, omega, delta)]
    got = [a.copy() for a in (theta, omega, delta)]
    for rnd in range(6):
        nbr = oracle.neighbour_table(4, K, p, q, seed=3, round=rnd)
        ref = list(_dense_reference(off, nbr, *ref, 0.9, 1.0, oracle.MODE_PAPER))
        oracle.sync(off, K, p, q, 3, rnd, *got, 0.9, 1.0, oracle.MODE_PAPER)
        drift = RNG.normal(0, 0.01, size=theta.shape)      # the local steps between syncs
        ref[0] += drift
        got[0] += drift
    for g, e in zip(got, ref):
        np.testing.assert_allclose(g, e, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("K", [4, 8, 5])
def test_all_neighbours_reduces_to_textbook_bmuf_nbm(K):
    # every worker averages all workers => conventional BMUF with Nesterov block momentum:
    # one global model W, one Delta, G = mean_k(theta^k) - W_start, W_start = W + eta*Delta
    P, R, eta, zeta = 37, 8, 0.9, 1.0
    off = np.array([0, 10, 37], dtype=np.int64)
    w0 = RNG.normal(0, 0.05, size=P)
    theta = np.tile(w0, (K, 1)); omega = theta.copy(); delta = np.zeros_like(theta)
    W, D, W_start = w0.copy(), np.zeros(P), w0.copy()
    for rnd in range(R):
        drift = RNG.normal(0, 0.02, size=(K, P))
        theta += drift                                     # local training of each worker
        local = W_start + drift                            # textbook: workers start from W_start
        G = local.mean(axis=0) - W_start
        D = eta * D + zeta * G
        W = W + D
        W_start = W + eta * D
        oracle.sync(off, K, K // 2, K - 1, 11, rnd, theta, omega, delta, eta, zeta, oracle.MODE_PAPER)
        for a in (theta, omega, delta):
            assert (a == a[0]).all()                       # all workers bit-identical
        np.testing.assert_allclose(theta[0], W_start, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(omega[0], W, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(delta[0], D, rtol=1e-12, atol=1e-14)


def test_all_neighbours_no_restart_reduces_to_classical_block_momentum():
    K, P, eta, zeta = 4, 16, 0.8, 0.9
    off = np.array([0, 16], dtype=np.int64)
    w0 = RNG.normal(0, 0.05, size=P)
    theta = np.tile(w0, (K, 1)); omega = theta.copy(); delta = np.zeros_like(theta)
    W, D = w0.copy(), np.zeros(P)
    for rnd in range(6):
        drift = RNG.normal(0, 0.02, size=(K, P))
        theta += drift
        G = (W + drift).mean(axis=0) - W
        D = eta * D + zeta * G
        W = W + D
        oracle.sync(off, K, 2, 3, 5, rnd, theta, omega, delta, eta, zeta, oracle.MODE_NO_RESTART)
        np.testing.assert_allclose(theta[2], W, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(omega[1], W, rtol=1e-12, atol=1e-14)


def test_eta0_zeta1_is_model_averaging():
    # with eta = 0 and zeta = 1 the filter passes the average through: the gossip-MA branch
    K, p, q, P = 8, 2, 2, 50
    off = np.array([0, 20, 50], dtype=np.int64)
    theta, omega, delta = _state(K, P)
    nbr = oracle.neighbour_table(2, K, p, q, 9, 4)
    want_avg = _dense_reference(off, nbr, theta, omega, delta, 0.0, 1.0, oracle.MODE_GOSSIP_MA)[0]
    for mode in (0, 1, 2):
        t, o, d = theta.copy(), omega.copy(), delta.copy()
        oracle.sync_table(off, nbr, t, o, d, 0.0, 1.0, mode)
        np.testing.assert_allclose(t, want_avg, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(o, want_avg, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(d, want_avg - omega, rtol=1e-12, atol=1e-15)
    t = theta.copy()
    oracle.sync_table(off, nbr, t, None, None, 0.0, 1.0, oracle.MODE_GOSSIP_MA)
    np.testing.assert_allclose(t, want_avg, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("K,p,q", [(4, 1, 1), (8, 2, 3), (16, 3, 0), (16, 3, 2), (8, 2, 4), (64, 5, 4)])
def test_identical_replicas_with_zero_delta_are_a_fixed_point(dtype, K, p, q):
    P = 64
    off = np.array([0, 7, 64], dtype=np.int64)
    w0 = RNG.normal(0, 0.05, size=P).astype(dtype)
    theta = np.tile(w0, (K, 1)); omega = theta.copy(); delta = np.zeros_like(theta)
    for rnd in range(5):
        oracle.sync(off, K, p, q, 1, rnd, theta, omega, delta, dtype(0.9), dtype(1.0), oracle.MODE_PAPER)
    if q <= 1:                                              # c and c+c are exact, and so is * 1 or * 0.5
        assert (theta == w0).all() and (omega == w0).all() and (delta == 0).all()
    else:                                                   # c+c+c already rounds: a few ulp off c
        eps = np.finfo(dtype).eps
        np.testing.assert_allclose(theta, np.tile(w0, (K, 1)), rtol=40 * eps, atol=0)
        np.testing.assert_allclose(omega, np.tile(w0, (K, 1)), rtol=40 * eps, atol=0)
        assert np.abs(delta).max() <= 40 * eps * np.abs(w0).max()


def test_zeta1_closed_form_of_the_paper_mode():
    # zeta = 1 (the paper's setting): Delta' = avg - omega, omega' = avg,
    # theta' = avg + eta (avg - omega).  Does NOT hold when G is measured from omega.
    K, p, q, P, eta = 16, 3, 2, 90, 0.9
    off = np.array([0, 30, 90], dtype=np.int64)
    theta, omega, delta = _state(K, P)
    nbr = oracle.neighbour_table(2, K, p, q, 77, 0)
    avg = _dense_reference(off, nbr, theta, omega, delta, 0, 1, oracle.MODE_GOSSIP_MA)[0]
    t, o, d = theta.copy(), omega.copy(), delta.copy()
    oracle.sync_table(off, nbr, t, o, d, eta, 1.0, oracle.MODE_PAPER)
    np.testing.assert_allclose(d, avg - omega, rtol=1e-10, atol=1e-15)
    np.testing.assert_allclose(o, avg, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(t, avg + eta * (avg - omega), rtol=1e-12, atol=1e-15)
    t2, o2, d2 = theta.copy(), omega.copy(), delta.copy()
    oracle.sync_table(off, nbr, t2, o2, d2, eta, 1.0, oracle.MODE_LITERAL)
    assert np.abs(o2 - avg).max() > 1e-4                   # the two readings differ
    t32, o32, d32 = (a.astype(np.float32) for a in (theta, omega, delta))
    oracle.sync_table(off, nbr, t32, o32, d32, np.float32(eta), np.float32(1.0), oracle.MODE_PAPER)
    np.testing.assert_allclose(o32, avg, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(t32, avg + eta * (avg - omega), rtol=1e-6, atol=1e-7)


def test_average_stays_between_min_and_max_of_the_workers():
    K, p, q, P = 16, 3, 3, 200
    off = np.array([0, 200], dtype=np.int64)
    theta = RNG.normal(0, 1, size=(K, P)).astype(np.float32)
    lo, hi = theta.min(axis=0), theta.max(axis=0)
    t = theta.copy()
    oracle.sync(off, K, p, q, 2, 0, t, None, None, 0.0, 1.0, oracle.MODE_GOSSIP_MA)
    slack = 4 * np.finfo(np.float32).eps * np.maximum(np.abs(lo), np.abs(hi))
    assert (t >= lo - slack).all() and (t <= hi + slack).all()
    assert np.abs(t - theta).max() > 0.1


def test_rounds_are_stateless_resume_is_bit_identical():
    K, p, q, P = 8, 2, 2, 33
    off = np.array([0, 10, 33], dtype=np.int64)
    theta, omega, delta = _state(K, P, dtype=np.float32)
    a = [x.copy() for x in (theta, omega, delta)]
    for rnd in range(7):
        oracle.sync(off, K, p, q, 8, rnd, *a, np.float32(0.9), np.float32(1.0))
    b = [x.copy() for x in (theta, omega, delta)]
    for rnd in range(3):
        oracle.sync(off, K, p, q, 8, rnd, *b, np.float32(0.9), np.float32(1.0))
    b = [np.array(x.tolist(), dtype=np.float32) for x in b]          # "checkpoint"
    for rnd in range(3, 7):
        oracle.sync(off, K, p, q, 8, rnd, *b, np.float32(0.9), np.float32(1.0))
    for x, y in zip(a, b):
        assert (x == y).all()


def test_inactive_components_are_left_alone():
    # Algorithm 1: a component only syncs when t mod H_i == 0
    K, p, q = 8, 2, 2
    off = np.array([0, 10, 25, 40], dtype=np.int64)
    theta, omega, delta = _state(K, 40)
    nbr = oracle.neighbour_table(3, K, p, q, 1, 0)
    full = [x.copy() for x in (theta, omega, delta)]
    oracle.sync_table(off, nbr, *full, 0.9, 1.0)
    part = [x.copy() for x in (theta, omega, delta)]
    oracle.sync_table(off, nbr, *part, 0.9, 1.0, active=[1, 0, 1])
    for f, g, orig in zip(full, part, (theta, omega, delta)):
        assert (g[:, 10:25] == orig[:, 10:25]).all()
        assert (g[:, :10] == f[:, :10]).all() and (g[:, 25:] == f[:, 25:]).all()


def test_q0_is_purely_local_block_momentum_and_K1_works():
    P = 9
    off = np.array([0, 9], dtype=np.int64)
    theta, omega, delta = _state(1, P)
    t, o, d = theta.copy(), omega.copy(), delta.copy()
    oracle.sync(off, 1, 1, 0, 0, 0, t, o, d, 0.9, 1.0)
    dn = 0.9 * delta + (theta - (omega + 0.9 * delta))
    np.testing.assert_allclose(d, dn, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(o, omega + dn, rtol=1e-12)
    np.testing.assert_allclose(t, omega + dn + 0.9 * dn, rtol=1e-12)


def test_fp32_writing_stays_close_to_fp64_over_the_longest_run():
    # 50 rounds at eta = 0.9 (the second benchmark configuration's schedule)
    K, p, q, P, R = 8, 2, 2, 4000, 50
    off = np.array([0, 1000, 4000], dtype=np.int64)
    w0 = RNG.uniform(-0.05, 0.05, size=P)
    theta = w0 + RNG.normal(0, 0.02, size=(K, P))
    omega = np.tile(w0, (K, 1)); delta = np.zeros((K, P))
    s32 = [a.astype(np.float32) for a in (theta, omega, delta)]
    s64 = [a.astype(np.float32).astype(np.float64) for a in (theta, omega, delta)]
    for rnd in range(R):
        oracle.sync(off, K, p, q, 1, rnd, *s32, np.float32(0.9), np.float32(1.0))
        oracle.sync(off, K, p, q, 1, rnd, *s64, float(np.float32(0.9)), 1.0)
    # The recurrence has a unit eigenvalue along the consensus direction, so rounding errors
    # add up over rounds and are amplified by the momentum's gain 1/(1-eta): the bound is
    # R/(1-eta) * eps * max|state|.  This is why the HIP path is gated against the fp32
    # writing (same operations, same order) and not against fp64 at 1e-6.
    eps = float(np.finfo(np.float32).eps)
    bound = R / (1 - 0.9) * eps * max(np.abs(b).max() for b in s64)
    for a, b in zip(s32, s64):
        assert np.abs(a - b).max() < bound
    assert np.abs(s32[0] - s64[0]).max() > 1e-6    # and the difference is real: fp64 is not the gate


def test_bad_arguments_are_rejected():
    K, P = 4, 10
    theta, omega, delta = _state(K, P)
    ok_off = np.array([0, 4, 10], dtype=np.int64)
    nbr = oracle.neighbour_table(2, K, 1, 1, 0, 0)
    with pytest.raises(ValueError):
        oracle.sync_table(np.array([0, 6, 4], dtype=np.int64), nbr, theta, omega, delta, 0.9, 1.0)
    with pytest.raises(ValueError):
        oracle.sync_table(np.array([1, 4, 10], dtype=np.int64), nbr, theta, omega, delta, 0.9, 1.0)
    with pytest.raises(ValueError):
        oracle.sync_table(np.array([0, 4, 11], dtype=np.int64), nbr, theta, omega, delta, 0.9, 1.0)
    bad = nbr.copy(); bad[0, 0, 0] = 4
    with pytest.raises(ValueError):
        oracle.sync_table(ok_off, bad, theta, omega, delta, 0.9, 1.0)
    with pytest.raises(ValueError):
        oracle.sync_table(ok_off, nbr, theta, omega, delta, 0.9, 1.0, mode=7)
    with pytest.raises(ValueError):
        oracle.sync_table(ok_off, nbr, theta, None, None, 0.9, 1.0, mode=1)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_final_average_is_the_mean_over_workers(dtype):
    K, P = 8, 100
    theta = RNG.normal(0, 1, size=(K, P + 5)).astype(dtype)
    got = oracle.final_average(theta, P)
    want = theta[:, :P].astype(np.float64).mean(axis=0)
    # K-1 additions and one multiply, each within half an ulp of a partial sum <= K*max|theta|
    tol = K * np.finfo(dtype).eps * np.abs(theta).max()
    np.testing.assert_allclose(got, want, rtol=0, atol=tol)
    same = np.tile(theta[0], (K, 1))
    np.testing.assert_allclose(oracle.final_average(same, P), same[0, :P],
                               rtol=K * np.finfo(dtype).eps, atol=0)
    two = np.tile(theta[0], (2, 1))                                  # c + c and * 0.5 are exact
    assert (oracle.final_average(two, P) == two[0, :P]).all()
