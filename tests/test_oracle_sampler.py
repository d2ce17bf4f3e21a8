"""Pins for the oracle's topology and neighbour sampler (CPU only).

What fixes the expected values here is outside the oracle: published known-answer vectors
for the generator, hand enumeration of Definition 1, Section 2.2's statement that q = 2p
uses all neighbours, and the statistics of a uniform choice without replacement.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def test_philox_known_answers():
    for ln in _rows("philox4x32_10_kat.txt"):
        w = [int(x, 16) for x in ln.split()]
        got = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in got] == w[6:10], ln


def test_ring_candidates_hand_enumerated():
    for ln in _rows("ring_candidates.txt"):
        left, right = ln.split(":")
        n, k, i = (int(x) for x in left.split())
        want = [int(x) for x in right.split()]
        assert oracle.ring_candidates(i, n, k).tolist() == want, ln


@pytest.mark.parametrize("K", [2, 3, 4, 5, 8, 16, 17, 64])
def test_full_degree_reaches_every_other_worker(K):
    for w in range(K):
        c = oracle.ring_candidates(w, K, K // 2)
        assert sorted(c.tolist()) == [v for v in range(K) if v != w]


def test_ring_is_symmetric():
    # "symmetric" ring: v is a neighbour of w exactly when w is a neighbour of v
    for K, p in [(4, 1), (8, 2), (16, 3), (64, 5), (7, 2)]:
        adj = [set(oracle.ring_candidates(w, K, p).tolist()) for w in range(K)]
        for w in range(K):
            assert len(adj[w]) == min(2 * p, K - 1)
            for v in adj[w]:
                assert w in adj[v]


def test_default_degree_follows_section_3_3():
    # p = log2(n) - 1: the paper's 4-, 8-, 16-GPU settings are p = 1, 2, 3
    assert [oracle.default_p(K) for K in (4, 8, 16)] == [1, 2, 3]
    assert oracle.default_p(64) == 5
    assert oracle.default_p(2) == 1 and oracle.default_p(1) == 1
    assert oracle.default_p(12) == 2  # floor(log2 12) - 1


@pytest.mark.parametrize("K,p,q", [(4, 1, 1), (8, 2, 2), (16, 3, 2), (16, 3, 3), (64, 5, 4), (64, 32, 63), (9, 2, 3)])
def test_rows_are_valid_choices(K, p, q):
    m = 40
    for rnd in (0, 1, 7):
        t = oracle.neighbour_table(m, K, p, q, seed=1234, round=rnd)
        assert t.shape == (m, K, q)
        for w in range(K):
            cand = set(oracle.ring_candidates(w, K, p).tolist())
            rows = t[:, w, :]
            assert (np.diff(rows, axis=1) > 0).all()            # ascending and distinct
            assert (rows != w).all()                              # never itself
            assert set(rows.ravel().tolist()) <= cand             # inside the ring


@pytest.mark.parametrize("K,p", [(4, 1), (8, 2), (16, 3), (64, 5), (5, 3), (2, 1)])
def test_q_equal_2p_takes_all_neighbours(K, p):
    # Section 2.2: with q = 2p "all of the neighbor nodes are included": no randomness left
    C = len(oracle.ring_candidates(0, K, p))
    for seed in (0, 99, 2**63 + 5):
        for rnd in (0, 3, 2**40):
            t = oracle.neighbour_table(5, K, p, C, seed, rnd)
            for w in range(K):
                want = sorted(oracle.ring_candidates(w, K, p).tolist())
                for i in range(5):
                    assert t[i, w].tolist() == want


def test_q_beyond_candidates_is_rejected():
    with pytest.raises(ValueError):
        oracle.sample(8, 2, 5, 0, 0, 0, 0)     # q <= 2p
    with pytest.raises(ValueError):
        oracle.sample(4, 2, 4, 0, 0, 0, 0)     # only K-1 other workers
    assert oracle.sample(1, 1, 0, 0, 0, 0, 0).size == 0   # a single worker has nobody to ask


def _position_of(K, p):
    """candidate id -> its position in the listing of Definition 1, per worker"""
    return [{v: j for j, v in enumerate(oracle.ring_candidates(w, K, p).tolist())} for w in range(K)]


def test_choice_is_uniform_without_replacement():
    # every candidate with probability q/C, every pair with q(q-1)/(C(C-1)): chi-square
    K, p, q, m, rounds = 16, 3, 3, 2000, 4
    C = 2 * p
    pos = _position_of(K, p)
    single = np.zeros(C)
    pair = np.zeros((C, C))
    n = 0
    for rnd in range(rounds):
        t = oracle.neighbour_table(m, K, p, q, seed=42, round=rnd)
        for w in range(K):
            lut = np.full(K, -1)
            for v, j in pos[w].items():
                lut[v] = j
            rows = lut[t[:, w, :]]                 # [m, q] positions
            n += m
            for a in range(q):
                np.add.at(single, rows[:, a], 1)
                for b in range(a + 1, q):
                    lo = np.minimum(rows[:, a], rows[:, b]); hi = np.maximum(rows[:, a], rows[:, b])
                    np.add.at(pair, (lo, hi), 1)
    assert n == 128000
    # singles: each position is Binomial(n, q/C); 6 cells, compare with 5-sigma band
    exp1 = n * q / C
    assert np.all(np.abs(single - exp1) < 5 * np.sqrt(exp1 * (1 - q / C))), single
    # pairs: 15 unordered pairs, each q(q-1)/(C(C-1)) -> q(q-1)/2 pairs per key
    iu = np.triu_indices(C, 1)
    exp2 = n * q * (q - 1) / (C * (C - 1))
    chi2 = (((pair[iu] - exp2) ** 2) / exp2).sum()
    assert chi2 < 50.0, chi2                       # 14 dof: P(chi2 > 50) ~ 6e-6
    # whole subsets: C(6,3) = 20 equally likely sets
    # (checked through the pair table's symmetry above; here: every set occurs)
    t = oracle.neighbour_table(4000, K, p, q, seed=7, round=0)
    sets = {tuple(r) for r in t[:, 0, :].tolist()}
    assert len(sets) == 20


def test_first_draw_is_uniform_over_all_candidates_q1():
    K, p = 64, 5
    t = oracle.neighbour_table(3000, K, p, 1, seed=5, round=11)
    pos = _position_of(K, p)
    cnt = np.zeros(2 * p)
    for w in range(K):
        for v in t[:, w, 0].tolist():
            cnt[pos[w][v]] += 1
    exp = 3000 * K / (2 * p)
    chi2 = ((cnt - exp) ** 2 / exp).sum()
    assert chi2 < 45.0, (chi2, cnt)                # 9 dof


def test_every_key_field_matters_and_components_are_independent():
    # Section 2.2: different components may choose different neighbours in each gossip
    K, p, q, m = 16, 3, 2, 600
    base = oracle.neighbour_table(m, K, p, q, seed=1, round=0)
    assert (oracle.neighbour_table(m, K, p, q, seed=1, round=0) == base).all()   # a function of the key
    for other in (oracle.neighbour_table(m, K, p, q, seed=2, round=0),
                  oracle.neighbour_table(m, K, p, q, seed=1, round=1),
                  oracle.neighbour_table(m, K, p, q, seed=1 + 2**32, round=0),
                  oracle.neighbour_table(m, K, p, q, seed=1, round=2**32)):
        frac_same = (other == base).all(axis=2).mean()
        # two independent uniform 2-subsets of 6 coincide with probability 1/15
        assert abs(frac_same - 1 / 15) < 0.02, frac_same
    # component i and i+1 of the same worker, worker w and w+1 of the same component:
    # relative choices (as positions in the listing) coincide no more often than by chance
    pos = _position_of(K, p)
    rel = np.zeros_like(base)
    for w in range(K):
        lut = np.full(K, -1)
        for v, j in pos[w].items():
            lut[v] = j
        rel[:, w, :] = np.sort(lut[base[:, w, :]], axis=1)
    same_comp = (rel[1:] == rel[:-1]).all(axis=2).mean()
    same_worker = (rel[:, 1:] == rel[:, :-1]).all(axis=2).mean()
    assert abs(same_comp - 1 / 15) < 0.02 and abs(same_worker - 1 / 15) < 0.02


def test_keying_matches_the_documented_counter_layout():
    # spec conformance (not a pin): draw 0 is word 0 of Philox(key = seed halves,
    # counter = (round lo, round hi, component, worker)), mapped by multiply-high
    K, p = 16, 3
    seed, rnd = 0x0123456789ABCDEF, 0x1_0000_0002
    for w in (0, 5, 15):
        for i in (0, 3, 1000):
            u = oracle.philox4x32_10([rnd & 0xFFFFFFFF, rnd >> 32, i, w], [seed & 0xFFFFFFFF, seed >> 32])
            cand = oracle.ring_candidates(w, K, p)
            want = cand[(int(u[0]) * len(cand)) >> 32]
            assert oracle.sample(K, p, 1, seed, rnd, w, i).tolist() == [want]


def test_all_subsets_are_equally_likely():
    # K = 16, p = 3, q = 3: C(6,3) = 20 subsets of the 6 ring neighbours, each with probability 1/20
    K, p, q, m = 16, 3, 3, 2500
    pos = _position_of(K, p)
    counts = {}
    n = 0
    for rnd in range(3):
        t = oracle.neighbour_table(m, K, p, q, seed=99, round=rnd)
        for w in range(K):
            lut = np.full(K, -1)
            for v, j in pos[w].items():
                lut[v] = j
            rows = np.sort(lut[t[:, w, :]], axis=1)
            keys = rows[:, 0] * 36 + rows[:, 1] * 6 + rows[:, 2]
            for k, c in zip(*np.unique(keys, return_counts=True)):
                counts[int(k)] = counts.get(int(k), 0) + int(c)
            n += m
    assert len(counts) == 20
    exp = n / 20
    chi2 = sum((c - exp) ** 2 / exp for c in counts.values())
    assert chi2 < 60.0, chi2                      # 19 dof: P(chi2 > 60) ~ 4e-6


def test_later_draws_use_the_next_counter_block():
    # spec conformance (not a pin): draws 4..7 take the words of the block whose last counter
    # word is worker + 65536; the whole partial shuffle replayed with Python integers
    K, p, q = 33, 7, 9
    seed, rnd = 0xFEDCBA9876543210, 5
    for w in (0, 16, 32):
        for i in (0, 7):
            cand = oracle.ring_candidates(w, K, p).tolist()
            C = len(cand)
            assert C == 14
            words = []
            for blk in range(3):
                words += [int(x) for x in oracle.philox4x32_10([rnd & 0xFFFFFFFF, rnd >> 32, i, w + 65536 * blk],
                                                               [seed & 0xFFFFFFFF, seed >> 32])]
            for j in range(q):
                r = j + ((words[j] * (C - j)) >> 32)
                cand[j], cand[r] = cand[r], cand[j]
            assert oracle.sample(K, p, q, seed, rnd, w, i).tolist() == sorted(cand[:q])
