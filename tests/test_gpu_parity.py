"""Parity of the HIP library against the CPU oracle, stage by stage and for the
whole layer, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

import oracle
import workloads
from helpers import DeviceLayer, HostLayer, err_metric, to_device, tae_margin as _tae_margin, \
    safe_threshold as _threshold, beta_pair

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "f32": 1e-5}


def _torch():
    import torch
    return torch


def _say(*a):
    print(*a, flush=True)


# ----------------------------------------------------------------- routing

ROUTE_CASES = [
    ("c1_tiny", {}, 16),
    ("c1_tiny", dict(d=200, E=37, K=5), 77),
    ("c2_mixtral_decode", dict(d=512), 1),
    ("c2_mixtral_decode", dict(d=512), 100),
    ("c2_mixtral_decode", dict(d=4096), 64),
    ("c5_deepseek", dict(d=256), 333),
    ("c4_qwen3", dict(d=512), 257),
    ("c4_qwen3", dict(d=256, E=200, K=8, n_resident=100), 65),
    ("c4_qwen3", dict(d=256, E=256, K=32, n_resident=100), 40),
]


@pytest.mark.parametrize("name,over,T", ROUTE_CASES)
@pytest.mark.parametrize("renorm", [True, False])
def test_route_topk(name, over, T, renorm):
    torch = _torch()
    import paper_2511_10054_amd as bm
    spec = workloads.scaled(name, F=32, **over)
    _say("route", spec.name, over, T, renorm)
    lay = workloads.get_layer(spec)
    x, _ = lay.tokens(T)
    ids_ref, w_ref = oracle.route_topk(lay.as_f32(x), lay.as_f32(lay.w_router), lay.router_bias, spec.K, renorm)
    desc = bm.LayerDesc(T=T, d=spec.d, E=spec.E, F=0, K=spec.K, n_shared=0, R=0, H=0,
                        dtype=bm.BM_BF16 if spec.dtype == "bf16" else bm.BM_F32,
                        flags=bm.BM_RENORM_TOPK if renorm else 0)
    ids = torch.full((T, spec.K), -9, dtype=torch.int32, device="cuda")
    w = torch.full((T, spec.K), -9.0, dtype=torch.float32, device="cuda")
    bm.bm_route_topk(desc, to_device(x), to_device(lay.w_router), to_device(lay.router_bias), ids, w)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ids.cpu().numpy(), ids_ref)
    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=2e-5, atol=1e-7)


@pytest.mark.parametrize("E,K", [(8, 3), (16, 5), (24, 6), (64, 8), (130, 8), (256, 32)])
def test_route_topk_breaks_ties_towards_the_lowest_index(E, K):
    """Equal logits (hidden state 0, a bias with repeated values, +0 and -0 among them): the
    selection is the oracle's, ties to the lowest expert index, on both top-k code paths."""
    torch = _torch()
    import paper_2511_10054_amd as bm
    _say("route ties", E, K)
    T, d = 37, 64
    g = np.random.default_rng(E * 100 + K)
    levels = np.array([0.0, -0.0, 0.5, -1.25, 2.0, 0.5], dtype=np.float32)
    bias = levels[g.integers(0, len(levels), size=E)].astype(np.float32)
    x = np.zeros((T, d), dtype=np.float32)
    wr = g.standard_normal((E, d)).astype(np.float32)
    ids_ref, w_ref = oracle.route_topk(x, wr, bias, K, True)
    assert (ids_ref[0] == ids_ref[-1]).all()
    desc = bm.LayerDesc(T=T, d=d, E=E, F=0, K=K, n_shared=0, R=0, H=0, dtype=bm.BM_BF16, flags=bm.BM_RENORM_TOPK)
    ids = torch.full((T, K), -9, dtype=torch.int32, device="cuda")
    w = torch.full((T, K), -9.0, dtype=torch.float32, device="cuda")
    bm.bm_route_topk(desc, to_device(workloads.f32_to_bf16_bits(x)), to_device(workloads.f32_to_bf16_bits(wr)),
                     to_device(bias), ids, w)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ids.cpu().numpy(), ids_ref)
    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=2e-5, atol=1e-7)


# ------------------------------------------------------------------- remap


def _random_problem(seed, T, E, K, R, n_res):
    g = np.random.default_rng(seed)
    ids = np.stack([g.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    res = np.zeros(E, bool); res[g.permutation(E)[:n_res]] = True
    table = np.stack([g.permutation([j for j in range(E) if j != i])[:R] for i in range(E)]).astype(np.int32)
    table[g.random((E, R)) < 0.15] = -1
    return ids, res, table


@pytest.mark.parametrize("T,E,K,R,n_res", [(1, 8, 2, 3, 4), (1000, 24, 4, 6, 9), (513, 64, 6, 8, 16),
                                           (300, 130, 8, 8, 50), (257, 256, 32, 32, 40), (64, 8, 2, 7, 0)])
@pytest.mark.parametrize("unique", [False, True])
def test_buddy_remap(T, E, K, R, n_res, unique):
    torch = _torch()
    import paper_2511_10054_amd as bm
    _say("remap", T, E, K, R, n_res, unique)
    ids, res, table = _random_problem(T + E, T, E, K, R, n_res)
    ids[::7, 0] = -1                                   # already-dropped inputs pass through as -1
    w = np.random.default_rng(1).random((T, K)).astype(np.float32)
    for H in {R, R // 2, 0}:
        ref, w_ref, st = oracle.buddy_remap(ids, res, table, H=H, unique=unique, w=w)
        desc = bm.LayerDesc(T=T, d=32, E=E, F=0, K=K, n_shared=0, R=R, H=H, dtype=bm.BM_BF16,
                            flags=bm.BM_REMAP_UNIQUE if unique else 0)
        d_ids = to_device(ids)
        d_out = torch.full((T, K), -9, dtype=torch.int32, device="cuda")
        d_w = to_device(w)
        d_stats = torch.full((6,), -9, dtype=torch.int32, device="cuda")
        bm.bm_buddy_remap(desc, to_device(workloads.pack_bitmap(res)), to_device(table), d_ids, d_out, d_w, d_stats)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_out.cpu().numpy(), ref)
        np.testing.assert_array_equal(d_w.cpu().numpy(), w_ref.astype(np.float32))
        assert d_stats.cpu().tolist() == [st["n_miss"], st["n_substituted"], st["n_dropped"], 0, 0, 0]
        # in place, no weights, no stats
        bm.bm_buddy_remap(desc, to_device(workloads.pack_bitmap(res)), to_device(table), d_ids, d_ids)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_ids.cpu().numpy(), ref)


# ------------------------------------------------------------- permutation


@pytest.mark.parametrize("T,K,E", [(0, 2, 8), (1, 2, 8), (57, 3, 11), (32, 32, 256), (128, 8, 200), (129, 8, 64),
                                   (1000, 6, 64), (4096, 8, 128), (33, 32, 256),
                                   (2100, 4, 256),      # fused scan + placement per tile, ragged last tile
                                   (8192, 8, 256)])     # histogram too large for that: separate scan and placement
def test_permute_by_expert(T, K, E):
    torch = _torch()
    import paper_2511_10054_amd as bm
    _say("permute", T, K, E)
    g = np.random.default_rng(T)
    ids = g.integers(0, E, size=(T, K)).astype(np.int32)
    ids[g.random((T, K)) < 0.2] = -1
    ids[:, 0] = np.minimum(ids[:, 0], 2)               # skew: a few very large groups
    off_ref, perm_ref, inv_ref = oracle.permute(ids, E)
    desc = bm.LayerDesc(T=T, d=0, E=E, F=0, K=K, n_shared=0, R=0, H=0, dtype=bm.BM_BF16, flags=0)   # T, E, K only
    nbytes = bm.bm_workspace_bytes(desc)
    assert 0 < nbytes <= 2 * 4 * E * (T // 32 + 1) + 2 * 4 * E + 6 * 256
    ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
    off = torch.full((E + 1,), -9, dtype=torch.int32, device="cuda")
    perm = torch.full((T * K,), -9, dtype=torch.int32, device="cuda")
    inv = torch.full((T * K,), -9, dtype=torch.int32, device="cuda")
    bm.bm_permute_by_expert(desc, to_device(ids), off, perm, inv, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(off.cpu().numpy(), off_ref)
    np.testing.assert_array_equal(perm.cpu().numpy(), perm_ref)
    np.testing.assert_array_equal(inv.cpu().numpy(), inv_ref)


# ------------------------------------------------------------- whole layer

LAYER_CASES = [
    # name, overrides, T  -- reduced widths, several row tiles and ragged tails
    ("c1_tiny", {}, 16),
    ("c1_tiny", dict(d=72, F=100, E=11, K=3, n_resident=5), 45),
    ("c2_mixtral_decode", dict(d=512, F=1024), 1),
    ("c2_mixtral_decode", dict(d=512, F=1024), 8),
    ("c2_mixtral_decode", dict(d=512, F=1024), 17),       # a full and a one-token 16-token tile
    ("c2_mixtral_decode", dict(d=512, F=1024), 64),
    ("c3_mixtral_prefill", dict(d=512, F=1024), 700),
    ("c3_mixtral_prefill", dict(d=1024, F=416), 333),     # F not a multiple of the column tile
    ("c4_qwen3", dict(d=256, F=384), 300),
    ("c5_deepseek", dict(d=256, F=352), 500),
    # 256-row tiles at short reductions: below four k-steps of 64 the fallback kernel runs, four and five are
    # the persistent kernel's shortest tiles (it looks the next tile up four k-steps before a tile's end, i.e.
    # at the first k-step of a four-step tile, and its loads move on three k-steps before the end); and with
    # shared experts
    ("c3_mixtral_prefill", dict(d=64, F=256), 600),
    ("c3_mixtral_prefill", dict(d=128, F=64), 520),
    ("c3_mixtral_prefill", dict(d=256, F=320), 600),
    ("c5_deepseek", dict(d=256, F=384, E=16, n_resident=6), 700),
    ("c5_deepseek", dict(d=256, F=256, E=16, n_resident=6), 900),     # four k-steps in both projections
    # long reduction of the down projection (the reduction-split tail itself needs more than 256 tiles: it is
    # covered by the full-size Mixtral prefill test)
    ("c3_mixtral_prefill", dict(d=256, F=4096), 2300),
    # the two projections on different tile heights (each walks its own row-tile table): 128-row gate/up tiles
    # with 256-row down tiles, short and long reduction
    ("c4_qwen3", dict(d=256, F=384), 1000),
    ("c3_mixtral_prefill", dict(d=256, F=4096), 600),
]


def _check_layer(host, unique, renorm=True, H=None, **gates):
    ref = host.oracle_forward(oracle, unique=unique, renorm=renorm, H=H, **gates)
    dev = DeviceLayer(host, unique=unique, renorm=renorm, H=H, **gates)
    out = dev.forward()
    spec = host.spec
    np.testing.assert_array_equal(out["ids"], ref["ids"])
    np.testing.assert_array_equal(out["ids_remapped"], ref["ids_remapped"])
    np.testing.assert_allclose(out["w"], ref["w"], rtol=2e-5, atol=1e-7)
    st = ref["stats"]
    assert out["stats"].tolist() == [st["n_miss"], st["n_substituted"], st["n_dropped"], st["n_requested"],
                                     st["n_requested_offloaded"], st["bypassed"]]
    off_ref, perm_ref, inv_ref = oracle.permute(ref["ids_remapped"], spec.E)
    np.testing.assert_array_equal(out["offsets"], off_ref)
    np.testing.assert_array_equal(out["perm"], perm_ref)
    np.testing.assert_array_equal(out["inv_perm"], inv_ref)
    e = err_metric(out["y"], ref["y"])
    _say("   err", e, "stats", st)
    assert e <= TOL[spec.dtype], e
    return out, ref, dev


@pytest.mark.parametrize("name,over,T", LAYER_CASES)
@pytest.mark.parametrize("unique", [False, True])
def test_layer_matches_oracle(name, over, T, unique):
    spec = workloads.scaled(name, **over)
    _say("layer", name, over, T, "unique" if unique else "first")
    host = HostLayer(spec, T)
    _check_layer(host, unique)


def _host_with_group_sizes(spec, sizes, n_dropped=3, pool=16000):
    """A HostLayer (K = 1) whose tokens are picked from a pool so that, after substitution, the expert groups
    have exactly the row counts in `sizes` (largest to the expert that attracts most tokens)."""
    assert spec.K == 1
    big = HostLayer(spec, pool, stream=3)
    ids, _ = oracle.route_topk(big.f32(big.x), big.f32(big.w_router), big.bias, 1)
    final = oracle.buddy_remap(ids, big.mask, big.table, H=spec.H)[0][:, 0]
    have = sorted(((int((final == e).sum()), e) for e in range(spec.E)), reverse=True)
    pick = []
    for want, (n, e) in zip(sorted(sizes, reverse=True), have):
        assert n >= want, (n, want)
        pick.append(np.flatnonzero(final == e)[:want])
    pick.append(np.flatnonzero(final < 0)[:n_dropped])
    sel = np.random.default_rng(len(sizes)).permutation(np.concatenate(pick))
    host = HostLayer(spec, len(sel), base=big)
    host.x = big.x[sel]
    return host


@pytest.mark.parametrize("sizes", [
    [1, 64, 65, 127, 128, 129],                           # 128-row tiles in both projections
    [1, 64, 65, 127, 128, 129, 255, 256],                 # 128-row gate/up tiles, 256-row down tiles
    [2, 16, 17, 130, 384, 385],
    [1, 128, 129, 255, 256, 257, 513, 1600],              # 256-row tiles
])
def test_tile_heights_at_exact_group_sizes(sizes):
    """Row tiles of the grouped projections at group sizes around their edges: a group of exactly one tile, one
    row more, one row less, a single row, for both tile heights of the persistent kernel."""
    spec = workloads.scaled("c4_qwen3", d=256, F=384, K=1, E=16, n_resident=8)
    _say("tile heights", sizes)
    host = _host_with_group_sizes(spec, sizes)
    out, ref, _ = _check_layer(host, unique=False)
    got = np.sort(np.diff(out["offsets"]))[::-1]
    np.testing.assert_array_equal(got[:len(sizes)], np.sort(sizes)[::-1])
    assert (got[len(sizes):] == 0).all()


DECODE_CASES = [
    ("c2_mixtral_decode", dict(d=512, F=1024), 1),
    ("c2_mixtral_decode", dict(d=2048, F=2048), 8),       # persistent kernel shapes
    ("c2_mixtral_decode", dict(d=2048, F=3584), 16),
    ("c2_mixtral_decode", dict(d=1024, F=2048), 64),      # LDS-staged kernel, several passes possible
    ("c2_mixtral_decode", dict(d=1024, F=2048), 128),     # 256 rows over 5 groups: passes of up to 128 rows
    ("c2_mixtral_decode", dict(d=512, F=1024), 250),      # 500 rows: some groups take two of those passes
    ("c4_qwen3", dict(d=256, F=256), 100),                # many experts, few rows each: streaming path past 256 rows
    ("c4_qwen3", dict(d=512, F=768), 40),                 # reduction of three chunks in the down projection, unsplit
    ("c5_deepseek", dict(d=2048, F=1792, E=16, n_resident=4), 4),    # shared experts on the decode path
    ("c4_qwen3", dict(d=256, F=96), 12),                  # odd widths: generic decode kernel
    # hidden size 16 x 256 units: the persistent down kernel aggregates its own results, here with shared
    # experts (their rows follow the routed ones) and with slots dropped
    ("c5_deepseek", dict(d=4096, F=512, E=16, n_resident=4), 5),
]


@pytest.mark.parametrize("name,over,T", DECODE_CASES)
@pytest.mark.parametrize("pack", [False, True])
def test_decode_path_matches_oracle(name, over, T, pack):
    """Decode-sized batches, public and fragment-major (packed) weights; absent experts are NaN."""
    spec = workloads.scaled(name, **over)
    _say("decode", name, over, T, "packed" if pack else "public")
    host = HostLayer(spec, T, only_resident=True, poison=True)
    ref = host.oracle_forward(oracle)
    dev = DeviceLayer(host, pack=pack)
    out = dev.forward()
    np.testing.assert_array_equal(out["ids_remapped"], ref["ids_remapped"])
    assert np.isfinite(out["y"]).all()
    e = err_metric(out["y"], ref["y"])
    _say("   err", e)
    assert e <= TOL["bf16"], e
    if pack:
        # packed and public weights give the same bytes
        out2 = DeviceLayer(host).forward()
        np.testing.assert_array_equal(out["y"], out2["y"])


def test_layer_without_renormalisation_and_short_search():
    spec = workloads.scaled("c5_deepseek", d=256, F=352)
    _say("layer no-renorm H=2")
    _check_layer(HostLayer(spec, 200), unique=True, renorm=False, H=2)


def test_all_resident_is_plain_topk_moe():
    spec = workloads.scaled("c4_qwen3", d=256, F=384)
    _say("layer all resident")
    host = HostLayer(spec, 150, mask=np.ones(spec.E, bool))
    out, ref, _ = _check_layer(host, unique=True)
    np.testing.assert_array_equal(out["ids"], out["ids_remapped"])
    assert out["stats"].tolist() == [0, 0, 0, 0, 0, 0]


def test_nothing_resident_leaves_only_shared_experts():
    spec = workloads.scaled("c5_deepseek", d=256, F=352)
    _say("layer none resident")
    host = HostLayer(spec, 100, mask=np.zeros(spec.E, bool))
    out, ref, _ = _check_layer(host, unique=False)
    assert (out["ids_remapped"] == -1).all() and (out["w"] == 0).all()
    spec0 = workloads.scaled("c4_qwen3", d=256, F=384)
    out, _, _ = _check_layer(HostLayer(spec0, 70, mask=np.zeros(spec0.E, bool)), unique=False)
    assert (out["y"] == 0).all()


def test_non_resident_weights_are_never_read():
    # weights of absent experts are NaN: any read would poison the output
    spec = workloads.scaled("c3_mixtral_prefill", d=512, F=1024)
    _say("layer poison")
    host = HostLayer(spec, 300, only_resident=True, poison=True)
    assert np.isnan(host.f32(host.wg)).any()
    out, _, _ = _check_layer(host, unique=False)
    assert np.isfinite(out["y"]).all()


def test_repeated_calls_give_identical_bytes():
    torch = _torch()
    spec = workloads.scaled("c5_deepseek", d=256, F=352)
    _say("layer determinism")
    dev = DeviceLayer(HostLayer(spec, 400), unique=True)
    a = dev.forward()
    dev.workspace.fill_(0xA5)                         # stale workspace contents must not matter
    b = dev.forward()
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_fp32_output_flag_and_empty_batch():
    torch = _torch()
    import paper_2511_10054_amd as bm
    spec = workloads.scaled("c2_mixtral_decode", d=512, F=1024)
    _say("layer y_f32 / T=0")
    host = HostLayer(spec, 40)
    ref = host.oracle_forward(oracle)
    dev = DeviceLayer(host, y_f32=True)
    out = dev.forward()
    assert dev.y.dtype == torch.float32
    assert err_metric(out["y"], ref["y"]) <= TOL["bf16"]
    empty = DeviceLayer(HostLayer(spec, 0))
    empty.forward(debug=False)                         # no-op, must not fault


# ------------------------------------------------ gates in front of Algorithm 1


@pytest.mark.parametrize("T,E,K,R,n_res", [(1, 8, 2, 3, 4), (1000, 24, 4, 6, 9), (513, 64, 6, 8, 16),
                                           (257, 256, 32, 32, 40)])
@pytest.mark.parametrize("unique", [False, True])
def test_buddy_remap_gated(T, E, K, R, n_res, unique):
    torch = _torch()
    import paper_2511_10054_amd as bm
    _say("remap gated", T, E, K, R, n_res, unique)
    ids, res, table = _random_problem(T + E, T, E, K, R, n_res)
    g = np.random.default_rng(T)
    z = g.normal(size=(T, K)) * 2.0
    w = (np.exp(z) / np.exp(z).sum(1, keepdims=True) * g.uniform(0.2, 1.0, size=(T, 1))).astype(np.float32)
    tae, margin = _tae_margin(w.astype(np.float64))
    tau, gamma = _threshold(tae, 0.4), _threshold(margin, 0.7)
    base = bm.BM_REMAP_UNIQUE if unique else 0
    delta, above = beta_pair(oracle.distribution_delta(ids, res)[0])   # gate closed / one fp32 step on: open
    for gates in (dict(tau=tau), dict(gamma=gamma), dict(rho=1), dict(rho=0), dict(tau=tau, gamma=gamma, rho=2),
                  dict(beta=delta), dict(beta=above), dict(beta=above, tau=tau, rho=1), dict(beta=0.0)):
        ref, w_ref, st = oracle.buddy_remap_gated(ids, res, table, w, H=R, unique=unique, **gates)
        flags = base | (bm.BM_GATE_TAE if "tau" in gates else 0) | (bm.BM_GATE_MARGIN if "gamma" in gates else 0) \
            | (bm.BM_REPLACE_BUDGET if "rho" in gates else 0) | (bm.BM_GATE_DIST if "beta" in gates else 0)
        desc = bm.LayerDesc(T=T, d=32, E=E, F=0, K=K, n_shared=0, R=R, H=R, dtype=bm.BM_BF16, flags=flags,
                            tae_tau=gates.get("tau", 0.0), margin_gamma=gates.get("gamma", 0.0),
                            rho=gates.get("rho", 0), dist_beta=gates.get("beta", 0.0))
        d_out = torch.full((T, K), -9, dtype=torch.int32, device="cuda")
        d_w = to_device(w)
        d_stats = torch.full((6,), -9, dtype=torch.int32, device="cuda")
        bm.bm_buddy_remap(desc, to_device(workloads.pack_bitmap(res)), to_device(table), to_device(ids), d_out,
                          d_w, d_stats)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(d_out.cpu().numpy(), ref, err_msg=str(gates))
        np.testing.assert_array_equal(d_w.cpu().numpy(), w_ref.astype(np.float32))
        assert d_stats.cpu().tolist() == [st["n_miss"], st["n_substituted"], st["n_dropped"], st["n_requested"],
                                          st["n_requested_offloaded"], st["bypassed"]], gates
        if T > 100 and ("tau" in gates or "gamma" in gates):
            assert 0 < st["n_substituted"] and 0 < st["n_dropped"]
        if "beta" in gates:
            # in place: the request set must be read before any id is overwritten
            d_ids = to_device(ids)
            bm.bm_buddy_remap(desc, to_device(workloads.pack_bitmap(res)), to_device(table), d_ids, d_ids,
                              to_device(w))
            torch.cuda.synchronize()
            np.testing.assert_array_equal(d_ids.cpu().numpy(), ref, err_msg="in place " + str(gates))
            assert st["bypassed"] == (0 if gates["beta"] == above else 1)


def test_gates_need_weights():
    import paper_2511_10054_amd as bm
    torch = _torch()
    desc = bm.LayerDesc(T=4, d=32, E=8, F=0, K=2, n_shared=0, R=2, H=2, dtype=bm.BM_BF16, flags=bm.BM_GATE_TAE,
                        tae_tau=0.5)
    ids = torch.zeros((4, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(bm.BuddyMoEError):
        bm.bm_buddy_remap(desc, torch.zeros(1, dtype=torch.int64, device="cuda"),
                          torch.zeros((8, 2), dtype=torch.int32, device="cuda"), ids, ids)


GATED_LAYER_CASES = [
    ("c1_tiny", {}, 16, False),
    ("c2_mixtral_decode", dict(d=512, F=1024), 8, False),       # fused one-workgroup front end
    ("c2_mixtral_decode", dict(d=512, F=1024), 24, True),       # two 16-token tiles; one 32-token tile with the distribution gate
    ("c2_mixtral_decode", dict(d=512, F=1024), 64, True),
    ("c3_mixtral_prefill", dict(d=512, F=1024), 700, False),
    ("c4_qwen3", dict(d=256, F=384), 300, True),
    ("c5_deepseek", dict(d=256, F=352), 500, True),
]


@pytest.mark.parametrize("name,over,T,unique", GATED_LAYER_CASES)
def test_gated_layer_matches_oracle(name, over, T, unique):
    spec = workloads.scaled(name, **over)
    _say("gated layer", name, over, T, unique)
    host = HostLayer(spec, T)
    _, w = oracle.route_topk(host.f32(host.x), host.f32(host.w_router), host.bias, spec.K)
    tae, margin = _tae_margin(w)
    tau, gamma = _threshold(tae, 0.35), _threshold(margin, 0.75)
    _check_layer(host, unique, tau=tau)
    _check_layer(host, unique, gamma=gamma, rho=max(1, spec.K // 2))
    out, ref, _ = _check_layer(host, unique, tau=tau, gamma=gamma, rho=1)
    replaced = (ref["ids_remapped"] != ref["ids"]) & (ref["ids_remapped"] >= 0)
    assert (replaced.sum(1) <= 1).all()
    # distribution gate (Eq. 2) at the batch's own delta (closed) and one fp32 step above it (open)
    ids, _ = oracle.route_topk(host.f32(host.x), host.f32(host.w_router), host.bias, spec.K)
    closed, open_ = beta_pair(oracle.distribution_delta(ids, host.mask)[0])
    out, ref, _ = _check_layer(host, unique, beta=closed)
    assert ref["stats"]["bypassed"] == 1 and ref["stats"]["n_substituted"] == 0
    out, ref, _ = _check_layer(host, unique, beta=open_, tau=tau)
    assert ref["stats"]["bypassed"] == 0 and ref["stats"]["n_substituted"] > 0


# ------------------------------------------------------------------ HIP graph


@pytest.mark.parametrize("name,over,T", [("c2_mixtral_decode", dict(d=512, F=1024), 8),
                                         ("c2_mixtral_decode", dict(d=1024, F=2048), 64),
                                         ("c5_deepseek", dict(d=256, F=352), 500)])
def test_forward_replays_from_a_hip_graph(name, over, T):
    """The whole layer is a fixed sequence of kernel launches on the caller's stream (no allocation, no
    synchronisation, no memset): captured once, replayed with new inputs in the same buffers, with eager
    work in between, every replay must equal the eager result for those inputs."""
    torch = _torch()
    spec = workloads.scaled(name, **over)
    _say("graph", name, T)
    hosts = [HostLayer(spec, T, stream=s) for s in (0, 1, 2)]
    dev = DeviceLayer(hosts[0], unique=True, rho=1)
    eager = []
    for h in hosts:                                             # eager results for the three inputs
        dev.x.copy_(to_device(h.x))
        eager.append(dev.forward(debug=False)["y"].copy())
    assert not np.array_equal(eager[0], eager[1])
    dev.x.copy_(to_device(hosts[0].x))
    side = torch.cuda.Stream()                                  # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dev.bm.bm_moe_forward(dev.desc, dev.x, dev.weights, dev.bitmap, dev.table, dev.y, dev.workspace, None)  # warm-up
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        dev.bm.bm_moe_forward(dev.desc, dev.x, dev.weights, dev.bitmap, dev.table, dev.y, dev.workspace, None)
    for rep in range(2):
        for i in (2, 0, 1):
            dev.x.copy_(to_device(hosts[i].x))
            dev.y.zero_()                                       # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            np.testing.assert_array_equal(dev.y.float().cpu().numpy(), eager[i], err_msg=f"replay {rep} input {i}")


# ------------------------------------------------------------- measurement aid


def test_stream_read_runs_and_leaves_memory_alone():
    """bm_stream_read only reads: the buffer and the sink are unchanged (sizes with and without a tail
    that is not a multiple of the grid's stride, and the empty buffer)."""
    torch = _torch()
    import paper_2511_10054_amd as bm
    _say("stream read")
    sink = torch.full((1,), 12345, dtype=torch.int32, device="cuda")
    for n in (0, 16, 16 * 1000 * 1000 + 48, 1 << 26):
        buf = torch.arange(n // 4, dtype=torch.int32, device="cuda")
        ref = buf.clone()
        bm.bm_stream_read(buf, sink)
        torch.cuda.synchronize()
        assert torch.equal(buf, ref) and int(sink.item()) == 12345
