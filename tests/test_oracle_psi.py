"""Pins for the oracle's token-aware buddy priority (Section 3.1, Eq. 3 with kappa = 0).  CPU only."""
import numpy as np

import oracle
from tests.test_oracle_remap import _random_problem


def _setup(seed, T=300, E=24, K=4, R=6, n_res=9):
    ids, res, table = _random_problem(seed, T=T, E=E, K=K, R=R, n_res=n_res, pad=False)
    g = np.random.default_rng(seed + 1)
    q = -np.sort(-g.dirichlet(np.ones(R), size=E), axis=1)            # rows sorted by q, like a built table
    z = g.normal(size=(T, E)) * 2
    return ids, res, table, q, oracle.softmax_all(z)


def test_softmax_matches_library():
    z = np.random.default_rng(0).normal(size=(50, 13)) * 3
    p = oracle.softmax_all(z)
    e = np.exp(z - z.max(1, keepdims=True))
    np.testing.assert_allclose(p, e / e.sum(1, keepdims=True), rtol=1e-14)
    np.testing.assert_allclose(p.sum(1), 1.0, rtol=1e-14)


def test_eta_zero_is_the_table_order():
    # Psi = q when eta = 0 and the rows are sorted by q: the first acceptable entry wins, i.e. Algorithm 1
    ids, res, table, q, zhat = _setup(1)
    for unique in (False, True):
        a = oracle.buddy_remap(ids, res, table, H=5, unique=unique)
        b = oracle.buddy_remap_psi(ids, res, table, q, zhat, 0.0, H=5, unique=unique)
        np.testing.assert_array_equal(a[0], b[0])
        assert a[2]["n_substituted"] == b[2]["n_substituted"]


def test_hand_case():
    # pivot 0 is offloaded; its buddies 1, 2, 3 have q = .5, .3, .2; all resident.
    res = np.array([0, 1, 1, 1], bool)
    table = np.array([[1, 2, 3], [0, 2, 3], [0, 1, 3], [0, 1, 2]], np.int32)
    q = np.array([[.5, .3, .2]] * 4)
    ids = np.array([[0, 1]], np.int32)                     # the token already holds expert 1
    zhat = np.array([[.1, .1, .1, .7]])
    # eta = 0: Psi = (.5, .3, .2) -> buddy 1 in "first" mode, buddy 2 in unique mode (1 is in U_t)
    assert oracle.buddy_remap_psi(ids, res, table, q, zhat, 0.0)[0].tolist() == [[1, 1]]
    assert oracle.buddy_remap_psi(ids, res, table, q, zhat, 0.0, unique=True)[0].tolist() == [[2, 1]]
    # eta = 5: Psi = .5*1.5, .3*1.5, .2*4.5 = .75, .45, .9 -> buddy 3, the expert this token's router likes
    out, _, _, margin = oracle.buddy_remap_psi(ids, res, table, q, zhat, 5.0)
    assert out.tolist() == [[3, 1]]
    np.testing.assert_allclose(margin, [(0.9 - 0.75) / 0.9])
    # the search depth still applies: H = 2 hides buddy 3
    assert oracle.buddy_remap_psi(ids, res, table, q, zhat, 5.0, H=2)[0].tolist() == [[1, 1]]
    # equal Psi: the earlier entry
    q2 = np.array([[.3, .3, .3]] * 4)
    assert oracle.buddy_remap_psi(ids, res, table, q2, np.full((1, 4), .25), 2.0)[0].tolist() == [[1, 1]]


def test_choice_is_the_argmax_over_acceptable_entries():
    ids, res, table, q, zhat = _setup(3)
    eta = 3.0
    out, _, st, margin = oracle.buddy_remap_psi(ids, res, table, q, zhat, eta, H=6, unique=True)
    n_changed_vs_alg1 = 0
    base = oracle.buddy_remap(ids, res, table, H=6, unique=True)[0]
    for t in range(len(ids)):
        used = set(ids[t].tolist())
        for k in range(ids.shape[1]):
            e = ids[t, k]
            if res[e]:
                assert out[t, k] == e
                continue
            cand = [(q[e, r] * (1 + eta * zhat[t, table[e, r]]), -r, table[e, r]) for r in range(6)
                    if res[table[e, r]] and table[e, r] not in used]
            want = max(cand)[2] if cand else -1
            assert out[t, k] == want
            if want >= 0:
                used.add(want)
        n_changed_vs_alg1 += int((out[t] != base[t]).any())
    assert n_changed_vs_alg1 > 10                          # the token-aware term does change choices here
    assert (margin > 0).all()


def test_gates_still_apply():
    ids, res, table, q, zhat = _setup(5)
    w = np.random.default_rng(9).dirichlet(np.ones(ids.shape[1]), size=len(ids))
    none = oracle.buddy_remap(ids, res, table, H=0, w=w)
    got = oracle.buddy_remap_psi(ids, res, table, q, zhat, 2.0, w=w, rho=0)
    np.testing.assert_array_equal(got[0], none[0])
    got = oracle.buddy_remap_psi(ids, res, table, q, zhat, 2.0, w=w, beta=0.0)
    np.testing.assert_array_equal(got[0], none[0])
