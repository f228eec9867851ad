"""Pins for the oracle's token-aware buddy priority (Section 3.1, Eq. 3 with kappa = 0).  CPU only."""
import numpy as np
import pytest

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


def _layer_case(T=48, seed=4):
    import workloads
    from workloads.harness import HostLayer
    h = HostLayer(workloads.scaled("c1_tiny"), T)
    g = np.random.default_rng(seed)
    q = -np.sort(-g.dirichlet(np.ones(h.spec.R), size=h.spec.E), axis=1)
    return h, q


@pytest.mark.parametrize("unique", [False, True])
@pytest.mark.parametrize("gates", [dict(), dict(rho=1), dict(tau=0.55)])
def test_layer_with_token_aware_priority_equals_stages(unique, gates):
    # the layer wrapper == routing -> softmax over ALL experts as z-hat -> Eq. 3 substitution -> experts,
    # chained by hand from the separately pinned stages (Section 3 "Notation", Section 3.1 Eq. 3)
    h, q = _layer_case()
    f, K, eta = h.f32, h.spec.K, 40.0
    out = oracle.moe_forward(f(h.x), f(h.w_router), h.bias, f(h.wg), f(h.wu), f(h.wd), h.mask, h.table, K,
                             H=3, unique=unique, eta=eta, q=q, **gates)
    z = oracle.router_logits(f(h.x), f(h.w_router), h.bias)
    ids, w = oracle.topk_gates(z, K)
    zhat = oracle.softmax_all(z)
    ids2, w2, st, margin = oracle.buddy_remap_psi(ids, h.mask, h.table, q, zhat, eta, w=w, H=3, unique=unique, **gates)
    y = oracle.experts_combine(f(h.x), ids2, w2, f(h.wg), f(h.wu), f(h.wd))
    np.testing.assert_array_equal(out["ids"], ids)
    np.testing.assert_array_equal(out["ids_remapped"], ids2)
    np.testing.assert_array_equal(out["w"], w2)
    np.testing.assert_array_equal(out["y"], y)
    np.testing.assert_array_equal(out["margin"], margin)
    assert out["stats"] == st and st["n_substituted"] > 0
    if not gates:
        # the case discriminates: raw logits as z-hat, or eta = 0 (the table order), choose differently
        raw = oracle.buddy_remap_psi(ids, h.mask, h.table, q, z, eta, w=w, H=3, unique=unique)[0]
        assert (raw != ids2).any()
        plain = oracle.buddy_remap(ids, h.mask, h.table, H=3, unique=unique)[0]
        assert (plain != ids2).any()


def test_layer_with_token_aware_priority_shared_experts_and_bias():
    # every pointer of the long argument list lands where it should: shared experts, bias, a q that is not
    # row-constant, no renormalisation
    import workloads
    from workloads.harness import HostLayer
    h = HostLayer(workloads.scaled("c5_deepseek", d=32, F=64), 40)
    f, K = h.f32, h.spec.K
    g = np.random.default_rng(2)
    q = -np.sort(-g.dirichlet(np.ones(h.spec.R), size=h.spec.E), axis=1)
    out = oracle.moe_forward(f(h.x), f(h.w_router), h.bias, f(h.wg), f(h.wu), f(h.wd), h.mask, h.table, K,
                             renorm=False, unique=True, eta=25.0, q=q, ws_gate=f(h.sg), ws_up=f(h.su), ws_down=f(h.sd))
    z = oracle.router_logits(f(h.x), f(h.w_router), h.bias)
    ids, w = oracle.topk_gates(z, K, renorm=False)
    ids2, w2, st, _ = oracle.buddy_remap_psi(ids, h.mask, h.table, q, oracle.softmax_all(z), 25.0, w=w, unique=True)
    y = oracle.experts_combine(f(h.x), ids2, w2, f(h.wg), f(h.wu), f(h.wd), f(h.sg), f(h.su), f(h.sd))
    np.testing.assert_array_equal(out["ids_remapped"], ids2)
    np.testing.assert_array_equal(out["w"], w2)
    np.testing.assert_array_equal(out["y"], y)
    assert out["stats"] == st and st["n_substituted"] > 0 and st["n_dropped"] > 0
