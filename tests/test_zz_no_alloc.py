"""bm_moe_forward_static (the entry point on the library's built-in scratch array, for callers that cannot
allocate) against bm_moe_forward: same kernels, so outputs and every index array must be bit-identical - and
with them within the stated tolerance of the oracle.  Two calls in a row share the array, the second with a
smaller input (needs an MI355X)."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads
from helpers import DeviceLayer, HostLayer, err_metric

pytestmark = pytest.mark.gpu


def _both(host, **kw):
    import torch
    import paper_2511_10054_amd as bm
    dev = DeviceLayer(host, **kw)
    assert 0 < bm.bm_workspace_bytes(dev.desc) <= bm.BM_STATIC_WORKSPACE_BYTES
    want = dev.forward()
    T, K, E = host.T, host.spec.K, host.spec.E
    i32 = dict(dtype=torch.int32, device="cuda")
    dbg = dict(ids=torch.full((T, K), -7, **i32), ids_remapped=torch.full((T, K), -7, **i32),
               w=torch.full((T, K), -7.0, dtype=torch.float32, device="cuda"),
               offsets=torch.full((E + 1,), -7, **i32), perm=torch.full((T * K,), -7, **i32),
               inv_perm=torch.full((T * K,), -7, **i32), stats=torch.full((6,), -7, **i32))
    y = torch.full_like(dev.y, float("nan"))
    before = torch.cuda.memory_allocated()
    bm.bm_moe_forward_static(dev.desc, dev.x, dev.weights, dev.bitmap, dev.table, y, dbg)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    got = dict(y=y.float().cpu().numpy(), **{k: v.cpu().numpy() for k, v in dbg.items()})
    for k in want:
        np.testing.assert_array_equal(got[k], want[k], err_msg=k)
    return got


CASES = [
    # (workload, overrides, first T, second - smaller - T, kwargs)
    ("c2_mixtral_decode", dict(), 64, 8, dict()),                        # the benchmark's decode layer, full size
    ("c5_deepseek", dict(d=256, F=352), 700, 90, dict(unique=True)),     # tiled path, shared experts, drops
    ("c4_qwen3", dict(d=256, F=384), 600, 5, dict(rho=1)),               # 128 experts; second call one tile
    ("c1_tiny", dict(), 16, 3, dict()),                                  # fp32
]


@pytest.mark.parametrize("name,over,T1,T2,kw", CASES, ids=[c[0] for c in CASES])
def test_static_workspace_entry_matches_the_workspace_entry(name, over, T1, T2, kw):
    spec = workloads.scaled(name, **over)
    tol = 2e-2 if spec.dtype == "bf16" else 1e-5
    base = None
    for T in (T1, T2):
        print("static workspace", name, T, kw, flush=True)
        host = HostLayer(spec, T, base=base)
        base = base or host
        got = _both(host, **kw)
        ref = host.oracle_forward(oracle, **kw)
        np.testing.assert_array_equal(got["ids_remapped"], ref["ids_remapped"])
        assert err_metric(got["y"], ref["y"]) <= tol


def test_static_workspace_entry_refuses_what_does_not_fit():
    import torch
    import paper_2511_10054_amd as bm
    lib = bm.load_library()
    one = ctypes.c_void_p(256)
    big = bm.LayerDesc(T=4096, d=4096, E=8, F=14336, K=2, n_shared=0, R=7, H=7, dtype=bm.BM_BF16, flags=bm.BM_RENORM_TOPK)
    assert bm.bm_workspace_bytes(big) > bm.BM_STATIC_WORKSPACE_BYTES
    w = bm.Weights(*([256] * 8 + [0] * 5))
    before = torch.cuda.memory_allocated()
    assert lib.bm_moe_forward_static(ctypes.byref(big), one, ctypes.byref(w), one, one, one, None, None) == -4
    assert lib.bm_moe_forward_static(ctypes.byref(big), None, ctypes.byref(w), one, one, one, None, None) == -1
    assert torch.cuda.memory_allocated() == before
