"""Parity of the device profiling statistics (Section 3.2) and buddy-list builder (Eq. 4-6) against the
oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

import oracle
import workloads
from helpers import DeviceLayer, HostLayer, err_metric, to_device

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _device_counts(ids_batches, E, K):
    torch = _torch()
    import paper_2511_10054_amd as bm
    A = torch.zeros(E, dtype=torch.int64, device="cuda")
    M = torch.zeros((E, E), dtype=torch.int64, device="cuda")
    for ids in ids_batches:
        desc = bm.LayerDesc(T=len(ids), d=32, E=E, F=0, K=K, n_shared=0, R=0, H=0, dtype=bm.BM_BF16, flags=0)
        bm.bm_coactivation_accumulate(desc, to_device(ids), A, M)
    torch.cuda.synchronize()
    return A, M


def _random_ids(seed, T, E, K):
    g = np.random.default_rng(seed)
    pop = g.dirichlet(np.full(E, 0.3))
    pop = (pop + 1e-4) / (pop + 1e-4).sum()
    return np.stack([g.choice(E, size=K, replace=False, p=pop) for _ in range(T)]).astype(np.int32)


@pytest.mark.parametrize("T,E,K", [(1, 8, 2), (777, 8, 2), (5000, 64, 6), (3000, 128, 8), (1000, 256, 32),
                                   (40000, 37, 5)])
def test_coactivation_counts(T, E, K):
    print("coactivation", T, E, K, flush=True)
    ids = _random_ids(T + E, T, E, K)
    ids[::11, 0] = -1                                   # dropped slots request nothing
    if K > 2:
        ids[::13, 2] = ids[::13, 1]                     # an expert listed twice counts once
    A_ref, M_ref = oracle.coactivation(ids, E)
    parts = [ids[: T // 3], ids[T // 3:]] if T > 3 else [ids]
    A, M = _device_counts([p for p in parts if len(p)], E, K)
    np.testing.assert_array_equal(A.cpu().numpy(), A_ref)
    np.testing.assert_array_equal(M.cpu().numpy(), M_ref)


@pytest.mark.parametrize("E,K,R", [(8, 2, 3), (64, 6, 8), (128, 8, 8), (256, 8, 32), (37, 5, 1)])
def test_buddy_table_builder(E, K, R):
    torch = _torch()
    import paper_2511_10054_amd as bm
    print("buddy builder", E, K, R, flush=True)
    ids = _random_ids(E + K, 6000, E, K)
    _, M_ref = oracle.coactivation(ids, E)
    M_ref[E // 2, :] = 0; M_ref[:, E // 2] = 0          # one expert that never co-activated: empty list
    M = to_device(M_ref)
    for alpha in (0.3137, 0.7071, 0.9531, 1.0, 1e-6):
        a32 = float(np.float32(alpha))                  # the value the C ABI carries
        t_ref, l_ref, q_ref = oracle.build_buddy_lists(M_ref, a32, R)
        desc = bm.LayerDesc(T=0, d=32, E=E, F=0, K=K, n_shared=0, R=R, H=R, dtype=bm.BM_BF16, flags=0)
        table = torch.full((E, R), -9, dtype=torch.int32, device="cuda")
        length = torch.full((E,), -9, dtype=torch.int32, device="cuda")
        q = torch.full((E, R), -9.0, dtype=torch.float32, device="cuda")
        bm.bm_build_buddy_table(desc, M, a32, table, length, q)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(table.cpu().numpy(), t_ref, err_msg=str(alpha))
        np.testing.assert_array_equal(length.cpu().numpy(), l_ref)
        np.testing.assert_allclose(q.cpu().numpy(), q_ref, rtol=1e-6, atol=0)
        assert bm.bm_validate_tables(desc, workloads.pack_bitmap(np.ones(E, bool)), table.cpu().numpy()) == 0
        # optional outputs may be left out
        table2 = torch.full((E, R), -9, dtype=torch.int32, device="cuda")
        bm.bm_build_buddy_table(desc, M, a32, table2)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(table2.cpu().numpy(), t_ref)


def test_buddy_table_builder_exact_boundary_of_eq5():
    """Prefix sums that land exactly on alpha (Eq. 5): counts 6, 3, 1 with alpha = fp32(0.9) and its fp32
    neighbours, counts 2, 1, 1 with alpha = 0.75, 0.5 (exact in every format) and their neighbours."""
    torch = _torch()
    import paper_2511_10054_amd as bm
    M1 = np.array([[0, 3, 6, 1], [3, 0, 0, 0], [6, 0, 0, 2], [1, 0, 2, 0]], np.int64)
    M2 = np.array([[0, 2, 1, 1], [2, 0, 0, 0], [1, 0, 0, 0], [1, 0, 0, 0]], np.int64)
    desc = bm.LayerDesc(T=0, d=32, E=4, F=0, K=2, n_shared=0, R=3, H=3, dtype=bm.BM_BF16, flags=0)
    seen = set()
    for M_ref, alphas in ((M1, (0.9, 0.6)), (M2, (0.75, 0.5))):
        M = to_device(M_ref)
        for a in alphas:
            a = np.float32(a)
            for a32 in (np.nextafter(a, np.float32(0)), a, np.nextafter(a, np.float32(1))):
                print("eq5 boundary", float(a32), flush=True)
                t_ref, l_ref, _ = oracle.build_buddy_lists(M_ref, float(a32), 3)
                table = torch.full((4, 3), -9, dtype=torch.int32, device="cuda")
                length = torch.full((4,), -9, dtype=torch.int32, device="cuda")
                bm.bm_build_buddy_table(desc, M, float(a32), table, length)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(table.cpu().numpy(), t_ref, err_msg=str(float(a32)))
                np.testing.assert_array_equal(length.cpu().numpy(), l_ref)
                seen.add((float(a), int(l_ref[0])))
    # the list length does change across each boundary (the cases are not vacuous)
    assert {(float(np.float32(0.9)), 2), (float(np.float32(0.9)), 3), (0.75, 2), (0.75, 3), (0.5, 1), (0.5, 2)} <= seen


@pytest.mark.parametrize("name,over,T", [("c5_deepseek", dict(d=256, F=352), 1500),
                                         ("c4_qwen3", dict(d=256, F=384), 900)])
def test_profile_then_serve(name, over, T):
    """The offline phase feeding the online one on the device: route a profiling batch, count, build the
    table, then run the layer with that table - every step against the oracle's."""
    torch = _torch()
    import paper_2511_10054_amd as bm
    spec = workloads.scaled(name, **over)
    print("profile then serve", name, T, flush=True)
    prof = HostLayer(spec, T, stream=7)                              # profiling tokens: their own stream
    E, K, R = spec.E, spec.K, spec.R
    desc = bm.LayerDesc(T=T, d=spec.d, E=E, F=0, K=K, n_shared=0, R=R, H=R, dtype=bm.BM_BF16, flags=bm.BM_RENORM_TOPK)
    ids = torch.empty((T, K), dtype=torch.int32, device="cuda")
    w = torch.empty((T, K), dtype=torch.float32, device="cuda")
    bm.bm_route_topk(desc, to_device(prof.x), to_device(prof.w_router), to_device(prof.bias), ids, w)
    A = torch.zeros(E, dtype=torch.int64, device="cuda")
    M = torch.zeros((E, E), dtype=torch.int64, device="cuda")
    bm.bm_coactivation_accumulate(desc, ids, A, M)
    table = torch.empty((E, R), dtype=torch.int32, device="cuda")
    alpha = float(np.float32(0.6180))
    bm.bm_build_buddy_table(desc, M, alpha, table)
    torch.cuda.synchronize()
    ids_ref, _ = oracle.route_topk(prof.f32(prof.x), prof.f32(prof.w_router), prof.bias, K)
    A_ref, M_ref = oracle.coactivation(ids_ref, E)
    t_ref, _, _ = oracle.build_buddy_lists(M_ref, alpha, R)
    np.testing.assert_array_equal(A.cpu().numpy(), A_ref)
    np.testing.assert_array_equal(M.cpu().numpy(), M_ref)
    np.testing.assert_array_equal(table.cpu().numpy(), t_ref)
    # serve other tokens with the measured table
    host = HostLayer(spec, 300, stream=1)
    host.table = t_ref.copy()
    ref = host.oracle_forward(oracle, unique=True)
    dev = DeviceLayer(host, unique=True)
    dev.table = table                                                # the device-built table, as is
    out = dev.forward()
    np.testing.assert_array_equal(out["ids_remapped"], ref["ids_remapped"])
    assert ref["stats"]["n_substituted"] > 0
    assert err_metric(out["y"], ref["y"]) <= 2e-2
