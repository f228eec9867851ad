"""Pins for the oracle's gated substitution: TAE gate and margin gate (Section 3.1), replacement
budget rho (Section 5.1) in front of Algorithm 1.  CPU only."""
import math

import numpy as np
import pytest

import oracle
from tests.test_oracle_remap import _random_problem


def _same(a, b):
    """(ids, w, stats) triples agree; stats compared on the keys both have."""
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    for k in set(a[2]) & set(b[2]):
        assert a[2][k] == b[2][k], k


def _gates(seed, T, K, sharp=3.0):
    g = np.random.default_rng(seed)
    z = g.normal(size=(T, K)) * sharp
    p = np.exp(z - z.max(1, keepdims=True))
    return p / p.sum(1, keepdims=True)


def test_gates_off_equals_algorithm1():
    ids, res, table = _random_problem(11)
    w = _gates(12, *ids.shape)
    for unique in (False, True):
        a = oracle.buddy_remap(ids, res, table, H=4, unique=unique, w=w)
        b = oracle.buddy_remap_gated(ids, res, table, w, H=4, unique=unique)
        _same(a, b)
        # thresholds no token can reach, budget no token can use up: the gates are there but never fire
        c = oracle.buddy_remap_gated(ids, res, table, w, H=4, unique=unique, tau=-1.0, gamma=2.0, rho=ids.shape[1])
        _same(a, c)


@pytest.mark.parametrize("kw", [dict(tau=1.0), dict(gamma=0.0), dict(rho=0)])
def test_gate_that_forbids_everything_equals_empty_search(kw):
    # TAE <= 1 and margin >= 0 always hold; rho = 0 leaves no budget: every miss is dropped, which is
    # what Algorithm 1 does with a search depth of zero.
    ids, res, table = _random_problem(13)
    w = _gates(14, *ids.shape)
    a = oracle.buddy_remap(ids, res, table, H=0, w=w)
    b = oracle.buddy_remap_gated(ids, res, table, w, H=5, **kw)
    _same(a, b)


def test_tae_gate_splits_tokens_at_the_threshold():
    # tokens with TAE (Eq. 1, recomputed here with numpy) above tau behave as ungated, the others as H = 0
    ids, res, table = _random_problem(15, T=400)
    w = _gates(16, *ids.shape)
    K = ids.shape[1]
    tae = -(w * np.log(w)).sum(1) / math.log(K)
    tau = float(np.median(tae))
    full = oracle.buddy_remap(ids, res, table, H=4, unique=True, w=w)
    none = oracle.buddy_remap(ids, res, table, H=0, unique=True, w=w)
    got = oracle.buddy_remap_gated(ids, res, table, w, H=4, unique=True, tau=tau)
    open_ = tae > tau
    assert 0 < open_.sum() < len(tae)
    np.testing.assert_array_equal(got[0], np.where(open_[:, None], full[0], none[0]))
    np.testing.assert_array_equal(got[1], np.where(open_[:, None], full[1], none[1]))


def test_tae_gate_is_scale_free():
    # Eq. 1 is defined on the renormalised gates: unnormalised softmax weights give the same decisions
    ids, res, table = _random_problem(17)
    w = _gates(18, *ids.shape)
    scale = np.random.default_rng(19).uniform(0.05, 0.9, size=(len(w), 1))
    a = oracle.buddy_remap_gated(ids, res, table, w, H=4, tau=0.6, gamma=0.7)
    b = oracle.buddy_remap_gated(ids, res, table, w * scale, H=4, tau=0.6, gamma=0.7)
    np.testing.assert_array_equal(a[0], b[0])


def test_tae_closed_forms_decide():
    # K = 2 gates (p, 1-p): TAE = binary entropy in bits.  H2(0.11) = 0.4999 < 0.5 < H2(0.1101...) ; use
    # p = 0.10 (H2 = 0.4690) and p = 0.12 (H2 = 0.5294) around tau = 0.5.
    res = np.array([0, 1, 1], bool)
    table = np.array([[1], [0], [0]], np.int32)
    ids = np.array([[0, 2], [0, 2]], np.int32)
    w = np.array([[0.10, 0.90], [0.12, 0.88]])
    out, w2, st = oracle.buddy_remap_gated(ids, res, table, w, tau=0.5)
    np.testing.assert_array_equal(out, [[-1, 2], [1, 2]])
    np.testing.assert_array_equal(w2, [[0.0, 0.90], [0.12, 0.88]])
    assert (st["n_miss"], st["n_substituted"], st["n_dropped"]) == (2, 1, 1)
    # uniform gates have TAE = 1 > any tau < 1; a one-hot token has TAE = 0 <= tau = 0
    w = np.array([[0.5, 0.5], [1.0, 0.0]])
    out, _, _ = oracle.buddy_remap_gated(ids, res, table, w, tau=0.0)
    np.testing.assert_array_equal(out, [[1, 2], [-1, 2]])


def test_margin_gate_closed_form():
    # K = 2: margin = |2p - 1|.  gamma = 0.5 forbids p = 0.8 (m = 0.6) and allows p = 0.7 (m = 0.4);
    # the margin is symmetric in which slot holds the larger gate.
    res = np.array([0, 1, 1], bool)
    table = np.array([[1], [0], [0]], np.int32)
    ids = np.array([[0, 2], [0, 2], [2, 0]], np.int32)
    w = np.array([[0.8, 0.2], [0.7, 0.3], [0.2, 0.8]])
    out, _, _ = oracle.buddy_remap_gated(ids, res, table, w, gamma=0.5)
    np.testing.assert_array_equal(out, [[-1, 2], [1, 2], [2, -1]])
    # margin uses the two LARGEST gates, not the first two slots: (0.45, 0.1, 0.45) has m = 0
    res4 = np.array([0, 1, 1, 1, 1], bool)
    table4 = np.array([[4], [0], [0], [0], [0]], np.int32)
    out, _, _ = oracle.buddy_remap_gated(np.array([[1, 0, 2]], np.int32), res4, table4,
                                         np.array([[0.45, 0.10, 0.45]]), gamma=0.2)
    np.testing.assert_array_equal(out, [[1, 4, 2]])
    # either gate alone forbids (logical OR): TAE open, margin closed
    out, _, _ = oracle.buddy_remap_gated(ids[:1], res, table, w[:1], tau=0.1, gamma=0.5)
    np.testing.assert_array_equal(out, [[-1, 2]])


def test_budget_counts_replacements_in_slot_order():
    # three misses with a buddy each; rho = 2 replaces the first two slots and drops the third
    res = np.array([0, 0, 0, 1, 1, 1], bool)
    table = np.array([[3], [4], [5], [0], [0], [0]], np.int32)
    ids = np.array([[0, 1, 2]], np.int32)
    w = np.full((1, 3), 1 / 3)
    for rho, want in [(0, [-1, -1, -1]), (1, [3, -1, -1]), (2, [3, 4, -1]), (3, [3, 4, 5])]:
        out, w2, st = oracle.buddy_remap_gated(ids, res, table, w, rho=rho)
        np.testing.assert_array_equal(out[0], want)
        assert st["n_substituted"] == min(rho, 3) and st["n_dropped"] == 3 - min(rho, 3)
    # a miss without an acceptable buddy uses up no budget
    res = np.array([0, 0, 0, 1, 1, 0], bool)
    out, _, _ = oracle.buddy_remap_gated(ids, res, table, w, rho=1)
    table2 = table.copy(); table2[0, 0] = 5                   # slot 0's only buddy is not resident
    out, _, _ = oracle.buddy_remap_gated(ids, res, table2, w, rho=1)
    np.testing.assert_array_equal(out[0], [-1, 4, -1])


def test_budget_property_on_random_inputs():
    ids, res, table = _random_problem(21, T=500, n_res=8)
    w = _gates(22, *ids.shape)
    full = oracle.buddy_remap(ids, res, table, H=6, unique=True, w=w)[0]
    for rho in (1, 2):
        out, w2, st = oracle.buddy_remap_gated(ids, res, table, w, H=6, unique=True, rho=rho)
        replaced = (out != ids) & (out >= 0)
        assert (replaced.sum(1) <= rho).all()
        assert st["n_substituted"] == int(replaced.sum())
        # until the budget is used up the result is Algorithm 1's own; afterwards every miss is dropped
        for t in range(len(ids)):
            n = 0
            for k in range(ids.shape[1]):
                miss = not res[ids[t, k]]
                if miss and n >= rho:
                    assert out[t, k] == -1 and w2[t, k] == 0.0
                elif miss and out[t, k] >= 0:
                    n += 1
        same = replaced.sum(1) < rho                         # budget never reached: identical to ungated
        np.testing.assert_array_equal(out[same], full[same])


def test_gated_layer_equals_stages():
    # whole-layer oracle with gates == its own stages chained by hand (gates act between routing and experts)
    import workloads
    from workloads.harness import HostLayer
    h = HostLayer(workloads.scaled("c1_tiny"), 24)
    f = h.f32
    K = h.spec.K
    out = oracle.moe_forward(f(h.x), f(h.w_router), h.bias, f(h.wg), f(h.wu), f(h.wd), h.mask, h.table, K,
                             H=2, unique=True, tau=0.55, rho=1)
    ids, w = oracle.route_topk(f(h.x), f(h.w_router), h.bias, K)
    ids2, w2, st = oracle.buddy_remap_gated(ids, h.mask, h.table, w, H=2, unique=True, tau=0.55, rho=1)
    y = oracle.experts_combine(f(h.x), ids2, w2, f(h.wg), f(h.wu), f(h.wd))
    np.testing.assert_array_equal(out["ids_remapped"], ids2)
    np.testing.assert_array_equal(out["y"], y)
    assert out["stats"] == st
    assert 0 < st["n_substituted"] and 0 < st["n_dropped"]


# ------------------------------------------------------------ distribution gate (Eq. 2)


def test_delta_hand_cases():
    # E = 6, experts 0..2 resident.  Batch requests {0, 1, 3, 5}: two of four offloaded.
    res = np.array([1, 1, 1, 0, 0, 0], bool)
    ids = np.array([[0, 3], [1, 3], [5, 0], [3, 1]], np.int32)
    assert oracle.distribution_delta(ids, res) == (0.5, 4, 2)
    # repeated requests count once (a set, not a multiset): 100 tokens asking for (0, 4)
    assert oracle.distribution_delta(np.tile(np.array([[0, 4]], np.int32), (100, 1)), res) == (0.5, 2, 1)
    # all requested resident -> 0; none resident -> 1; slots already dropped (-1) request nothing
    assert oracle.distribution_delta(np.array([[0, 1], [2, 1]], np.int32), res)[0] == 0.0
    assert oracle.distribution_delta(np.array([[3, 4], [5, -1]], np.int32), res) == (1.0, 3, 3)
    assert oracle.distribution_delta(np.zeros((0, 2), np.int32), res) == (0.0, 0, 0)


def test_delta_against_numpy_sets():
    ids, res, _ = _random_problem(31, T=37, E=24, K=4)
    req = np.unique(ids)
    d, n_req, n_cpu = oracle.distribution_delta(ids, res)
    assert n_req == len(req) and n_cpu == int((~res[req]).sum()) and d == n_cpu / n_req
    # delta depends on the set only: permuting tokens and slots changes nothing
    g = np.random.default_rng(0)
    assert oracle.distribution_delta(g.permuted(ids[g.permutation(len(ids))], axis=1), res) == (d, n_req, n_cpu)


def test_distribution_gate_is_all_or_nothing():
    ids, res, table = _random_problem(33, T=64, E=24, K=4, n_res=9)
    w = _gates(34, *ids.shape)
    d, n_req, n_cpu = oracle.distribution_delta(ids, res)
    full = oracle.buddy_remap(ids, res, table, H=4, unique=True, w=w)
    none = oracle.buddy_remap(ids, res, table, H=0, unique=True, w=w)
    for beta, want, byp in [(d + 1e-9, full, 0), (d, none, 1), (d - 1e-9, none, 1), (1.01, full, 0), (0.0, none, 1)]:
        got = oracle.buddy_remap_gated(ids, res, table, w, H=4, unique=True, beta=beta)
        _same(got, want)
        assert (got[2]["n_requested"], got[2]["n_requested_offloaded"], got[2]["bypassed"]) == (n_req, n_cpu, byp)
    # the gate needs no weights
    got = oracle.buddy_remap_gated(ids, res, table, None, H=4, unique=True, beta=d)
    np.testing.assert_array_equal(got[0], none[0])


def test_distribution_gate_sees_the_whole_batch():
    # one token alone: it requests {0 (resident), 3 (offloaded)} -> delta = 1/2.  Together with a token
    # that requests two more resident experts the batch has delta = 1/4: beta = 0.4 bypasses the first
    # batch and not the second, so the same token gets a different result depending on its batch.
    res = np.array([1, 1, 1, 0, 0, 0], bool)
    table = np.array([[1], [0], [0], [2], [2], [2]], np.int32)
    a = oracle.buddy_remap_gated(np.array([[0, 3]], np.int32), res, table, beta=0.4)
    b = oracle.buddy_remap_gated(np.array([[0, 3], [1, 2]], np.int32), res, table, beta=0.4)
    np.testing.assert_array_equal(a[0], [[0, -1]])
    np.testing.assert_array_equal(b[0], [[0, 2], [1, 2]])
    assert a[2]["bypassed"] == 1 and b[2]["bypassed"] == 0


def test_three_stage_order():
    # TAE gate closes token 0, distribution gate open: token 1 is still served.  Then the distribution
    # gate closes: nobody is served, although token 1 passed its own gate.
    res = np.array([1, 1, 0, 0], bool)
    table = np.array([[1], [0], [0], [1]], np.int32)
    ids = np.array([[2, 0], [3, 0]], np.int32)
    w = np.array([[0.95, 0.05], [0.5, 0.5]])
    got = oracle.buddy_remap_gated(ids, res, table, w, tau=0.5, beta=0.9)        # delta = 2/3
    np.testing.assert_array_equal(got[0], [[-1, 0], [1, 0]])
    got = oracle.buddy_remap_gated(ids, res, table, w, tau=0.5, beta=0.6)
    np.testing.assert_array_equal(got[0], [[-1, 0], [-1, 0]])
