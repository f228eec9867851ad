"""Pins for the oracle's profiling statistics (Section 3.2) and buddy-list construction (Eq. 4-6). CPU only."""
import numpy as np
import pytest

import oracle
import workloads


def _ids(seed, T, E, K):
    g = np.random.default_rng(seed)
    pop = g.dirichlet(np.full(E, 0.4))                       # heavy-tailed popularity
    return np.stack([g.choice(E, size=K, replace=False, p=pop) for _ in range(T)]).astype(np.int32)


def test_counts_equal_indicator_gram_matrix():
    # X[t][e] = 1 iff e in S(x_t):  A = column sums, M = X^T X without its diagonal
    ids = _ids(1, 500, 24, 4)
    A, M = oracle.coactivation(ids, 24)
    X = np.zeros((500, 24), np.int64)
    X[np.arange(500)[:, None], ids] = 1
    G = X.T @ X
    np.testing.assert_array_equal(A, X.sum(0))
    np.testing.assert_array_equal(np.diag(M), 0)
    np.testing.assert_array_equal(M, G - np.diag(np.diag(G)))
    np.testing.assert_array_equal(M, M.T)
    # every token contributes K to A and K(K-1) ordered pairs to M; row sums: each token with i adds K-1
    assert A.sum() == 500 * 4 and M.sum() == 500 * 4 * 3
    np.testing.assert_array_equal(M.sum(1), A * 3)


def test_counts_hand_case_and_accumulation():
    ids = np.array([[0, 1], [0, 1], [0, 2], [3, -1]], np.int32)     # -1: a slot that requests nothing
    A, M = oracle.coactivation(ids, 4)
    np.testing.assert_array_equal(A, [3, 2, 1, 1])
    np.testing.assert_array_equal(M, [[0, 2, 1, 0], [2, 0, 0, 0], [1, 0, 0, 0], [0, 0, 0, 0]])
    # batches add up
    A2, M2 = oracle.coactivation(ids[:2], 4)
    oracle.coactivation(ids[2:], 4, A2, M2)
    np.testing.assert_array_equal(A2, A); np.testing.assert_array_equal(M2, M)


def test_buddy_lists_hand_case():
    # pivot 0 co-activates 6, 3, 1 times with experts 2, 1, 3:  q = .6, .3, .1
    M = np.array([[0, 3, 6, 1], [3, 0, 0, 0], [6, 0, 0, 2], [1, 0, 2, 0]], np.int64)
    for alpha, want0 in [(0.5, [2, -1, -1]), (0.59, [2, -1, -1]), (0.61, [2, 1, -1]), (0.89, [2, 1, -1]),
                         (0.91, [2, 1, 3]), (1.0, [2, 1, 3])]:
        table, length, q = oracle.build_buddy_lists(M, alpha, 3)
        np.testing.assert_array_equal(table[0], want0, err_msg=str(alpha))
        assert length[0] == sum(x >= 0 for x in want0)
    table, length, q = oracle.build_buddy_lists(M, 1.0, 3)
    np.testing.assert_allclose(q[0], [0.6, 0.3, 0.1])
    np.testing.assert_array_equal(table[1], [0, -1, -1])                 # single peer: t = 1 for any alpha
    np.testing.assert_array_equal(table[2], [0, 3, -1])                  # q = .75, .25
    # the cap K_max cuts the list; a tiny alpha still keeps one buddy (t_i >= 1)
    np.testing.assert_array_equal(oracle.build_buddy_lists(M, 1.0, 2)[0][0], [2, 1])
    np.testing.assert_array_equal(oracle.build_buddy_lists(M, 1e-9, 3)[0][0], [2, -1, -1])
    # an expert that never co-activated has no buddies
    M0 = M.copy(); M0[3, :] = 0; M0[:, 3] = 0
    t0, l0, _ = oracle.build_buddy_lists(M0, 0.9, 3)
    np.testing.assert_array_equal(t0[3], [-1, -1, -1]); assert l0[3] == 0


def test_buddy_lists_exact_boundary_of_eq5():
    # Eq. 5 when a prefix sum lands exactly on alpha.  Counts 6, 3, 1 of 10: the prefix {.6, .3} is .9.
    M = np.array([[0, 3, 6, 1], [3, 0, 0, 0], [6, 0, 0, 2], [1, 0, 2, 0]], np.int64)
    # alpha = 0.9 as an fp64 number: 0.9 * 10 rounds to 9.0 exactly, 9 >= 9.0 holds, the prefix of two is enough
    np.testing.assert_array_equal(oracle.build_buddy_lists(M, 0.9, 3)[0][0], [2, 1, -1])
    # alpha = 0.9 as the fp32 number a C caller passes is 0.89999998: still two entries; the next fp32 value
    # up, 0.90000004, is past the prefix sum and needs the third
    a32 = np.float32(0.9)
    assert float(a32) < 0.9 < float(np.nextafter(a32, np.float32(1)))
    np.testing.assert_array_equal(oracle.build_buddy_lists(M, float(a32), 3)[0][0], [2, 1, -1])
    np.testing.assert_array_equal(oracle.build_buddy_lists(M, float(np.nextafter(a32, np.float32(1))), 3)[0][0], [2, 1, 3])
    # and just past 0.9 in fp64
    np.testing.assert_array_equal(oracle.build_buddy_lists(M, float(np.nextafter(0.9, 1.0)), 3)[0][0], [2, 1, 3])
    # a boundary every format represents exactly: counts 2, 1, 1 of 4 and alpha = 0.75 (prefix {.5, .25})
    M2 = np.array([[0, 2, 1, 1], [2, 0, 0, 0], [1, 0, 0, 0], [1, 0, 0, 0]], np.int64)
    np.testing.assert_array_equal(oracle.build_buddy_lists(M2, 0.75, 3)[0][0], [1, 2, -1])       # ">=" includes equality
    np.testing.assert_array_equal(oracle.build_buddy_lists(M2, 0.5, 3)[0][0], [1, -1, -1])
    np.testing.assert_array_equal(oracle.build_buddy_lists(M2, float(np.nextafter(np.float32(0.75), np.float32(1))), 3)[0][0],
                                  [1, 2, 3])


def test_buddy_lists_against_numpy_ranking():
    ids = _ids(5, 3000, 32, 6)
    _, M = oracle.coactivation(ids, 32)
    for alpha in (0.3137, 0.7071, 0.9531):                      # no prefix sum of counts lands on these
        table, length, q = oracle.build_buddy_lists(M, alpha, 32)
        for i in range(32):
            row = M[i].astype(np.float64); row[i] = 0
            if row.sum() == 0:
                assert length[i] == 0 and (table[i] == -1).all()
                continue
            qi = row / row.sum()                                         # Eq. 4: sums to 1 over the peers
            order = np.lexsort((np.arange(32), -qi))                     # descending q, ties to the lower index
            order = order[qi[order] > 0]
            cum = np.cumsum(qi[order])
            t = int(np.argmax(cum >= alpha - 1e-12)) + 1                 # Eq. 5 (no boundary case in this data)
            assert abs(cum[t - 1] - alpha) > 1e-9
            assert length[i] == t
            np.testing.assert_array_equal(table[i, :t], order[:t])
            assert (table[i, t:] == -1).all()
            np.testing.assert_allclose(q[i, :t], qi[order[:t]], rtol=1e-14)
            assert t == 1 or cum[t - 2] < alpha                          # minimality of the prefix
    # alpha = 1 lists every peer with a positive count, in the generator's ranking order
    table, length, _ = oracle.build_buddy_lists(M, 1.0, 32)
    for i in range(32):
        want = workloads.ranked_peers(M[i], i)
        np.testing.assert_array_equal(table[i, :len(want)], want)
        assert length[i] == len(want)


def test_larger_alpha_never_shrinks_a_list():
    ids = _ids(7, 2000, 40, 4)
    _, M = oracle.coactivation(ids, 40)
    prev = None
    for alpha in (0.1, 0.3, 0.5, 0.8, 0.99):
        table, length, _ = oracle.build_buddy_lists(M, alpha, 12)
        if prev is not None:
            assert (length >= prev[1]).all()
            for i in range(40):                                          # and the shorter list is a prefix
                np.testing.assert_array_equal(table[i, :prev[1][i]], prev[0][i, :prev[1][i]])
        prev = (table, length)
