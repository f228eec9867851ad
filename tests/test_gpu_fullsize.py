"""Parity at the full benchmark sizes, in the launch configuration bench.py times:
all index outputs on every token, layer outputs on a seeded sample of tokens that
the oracle can compute one by one (tokens are independent).  Needs an MI355X."""
import numpy as np
import pytest

import oracle
import workloads
from helpers import DeviceLayer, HostLayer, edge_tokens, err_metric, err_unfloored, safe_threshold, tae_margin

pytestmark = pytest.mark.gpu

_cache = {}


def _layers(name, pack=None):
    """Host + device weights of a config, built once per test session.  pack: fragment-major copies of the
    weights for the decode kernels (default: as bench.py does, for the decode config only)."""
    if pack is None:
        pack = name.startswith("c2")
    if name not in _cache:
        _cache.clear()                       # one big layer at a time
        spec = workloads.CONFIGS[name]
        _cache[name] = {"host": HostLayer(spec, 1, only_resident=True, poison=True)}
    entry = _cache[name]
    if pack not in entry:
        entry[pack] = DeviceLayer(entry["host"], pack=pack)
    return entry["host"], entry[pack]


def _check(name, T, n_sample, unique=False, pack=None, **gates):
    spec = workloads.CONFIGS[name]
    base_host, base_dev = _layers(name, pack)
    print(f"fullsize {name} T={T} unique={unique} pack={pack} {gates}", flush=True)
    host = HostLayer(spec, T, base=base_host)
    dev = DeviceLayer(host, unique=unique, base=base_dev, **gates)
    out = dev.forward()
    # indices on all tokens
    lay = host.lay
    ids_ref, w_ref = oracle.route_topk(host.f32(host.x), host.f32(host.w_router), host.bias, spec.K)
    ids2_ref, w2_ref, st = oracle.buddy_remap_gated(ids_ref, host.mask, host.table, w_ref, H=spec.H, unique=unique,
                                                    **gates)
    off_ref, perm_ref, inv_ref = oracle.permute(ids2_ref, spec.E)
    np.testing.assert_array_equal(out["ids"], ids_ref)
    np.testing.assert_array_equal(out["ids_remapped"], ids2_ref)
    np.testing.assert_allclose(out["w"], w2_ref, rtol=2e-5, atol=1e-7)
    assert out["stats"].tolist() == [st["n_miss"], st["n_substituted"], st["n_dropped"], st["n_requested"],
                                     st["n_requested_offloaded"], st["bypassed"]]
    np.testing.assert_array_equal(out["offsets"], off_ref)
    np.testing.assert_array_equal(out["perm"], perm_ref)
    np.testing.assert_array_equal(out["inv_perm"], inv_ref)
    assert host.mask[ids2_ref[ids2_ref >= 0]].all()
    # outputs on a seeded sample of tokens plus the tokens whose rows sit at tile edges: the first and the
    # last row of every expert group and one row from each 128-row half of every 256-row tile
    g = np.random.default_rng(1234 + T)
    rows = g.permutation(T)[: min(T, n_sample)]
    edges = edge_tokens(off_ref, perm_ref, spec.K, cap=max(2 * n_sample, 2 * int((np.diff(off_ref) > 0).sum())), seed=T)
    rows = np.unique(np.concatenate([rows, edges]))
    for e in np.unique(ids2_ref[ids2_ref >= 0]):                 # the sample does hold every group's two end rows
        for pos in (off_ref[e], off_ref[e + 1] - 1):
            assert perm_ref[pos] // spec.K in rows
    if gates:      # the distribution gate sees the whole batch: feed the sampled tokens' final ids and weights
        f = host.f32
        y_ref = oracle.experts_combine(f(host.x)[rows], ids2_ref[rows], w2_ref[rows], f(host.wg), f(host.wu),
                                       f(host.wd), f(host.sg), f(host.su), f(host.sd))
    else:
        ref = host.oracle_forward(oracle, unique=unique, rows=rows)
        np.testing.assert_array_equal(ref["ids_remapped"], ids2_ref[rows])
        y_ref = ref["y"]
    err = err_metric(out["y"][rows], y_ref)
    print(f"   sample {len(rows)} tokens ({len(edges)} at group / tile edges), err {err:.3e}, "
          f"unfloored elementwise {err_unfloored(out['y'][rows], y_ref):.3e}, stats {st}", flush=True)
    assert np.isfinite(out["y"]).all()
    assert err <= 2e-2, err


@pytest.mark.parametrize("T", [1, 8, 32, 64])
def test_c2_mixtral_decode(T):
    _check("c2_mixtral_decode", T, 64)


@pytest.mark.parametrize("T", [1, 16, 64])
def test_c2_mixtral_decode_public_weight_layout(T):
    """The same layer without the packed copies (bench.py --no-pack): the decode kernels read [N][K] rows."""
    _check("c2_mixtral_decode", T, 64, pack=False)


@pytest.mark.parametrize("T", [128, 256, 512, 1024, 2048])
def test_c2_mixtral_between_decode_and_prefill(T):
    """Batches between the benchmark points: 128-rows-per-pass streaming kernel (128), two such passes for the
    largest groups (256), 128-row gate/up tiles with 256-row down tiles of the prefill kernels (512), 256-row
    tiles in both with a last round of few tiles (1024, 2048)."""
    _check("c2_mixtral_decode", T, 64)


def test_c2_small_batches_aggregated_by_the_down_kernel():
    """Up to 16 tokens on this layer (hidden size = 16 x the device's 256 units) the persistent down kernel
    adds up its own results and writes the layer output; checked here on the fp32 output as well, on a batch
    size that is no multiple of anything, and with nothing resident (no live group: the output is zero)."""
    spec = workloads.CONFIGS["c2_mixtral_decode"]
    base_host, base_dev = _layers("c2_mixtral_decode", pack=False)
    for T in (3, 16):
        print(f"fullsize c2 T={T} fp32 output", flush=True)
        host = HostLayer(spec, T, base=base_host)
        out = DeviceLayer(host, y_f32=True, base=base_dev).forward()
        ref = host.oracle_forward(oracle, rows=np.arange(T))
        np.testing.assert_array_equal(out["ids_remapped"], ref["ids_remapped"])
        err = err_metric(out["y"], ref["y"])
        print(f"   err {err:.3e}", flush=True)
        assert err <= 2e-2, err
    print("fullsize c2 T=5 nothing resident", flush=True)
    host = HostLayer(spec, 5, mask=np.zeros(spec.E, bool), base=base_host)
    dev = DeviceLayer(host, base=base_dev)
    dev.y.fill_(7.0)
    out = dev.forward()
    assert (out["ids_remapped"] == -1).all() and (out["y"] == 0).all()


def test_c2_mixtral_decode_unique():
    _check("c2_mixtral_decode", 64, 64, unique=True)


def test_c3_mixtral_prefill():
    _check("c3_mixtral_prefill", 4096, 96)


def test_c4_qwen3():
    _check("c4_qwen3", 2048, 256)


def test_c5_deepseek():
    _check("c5_deepseek", 8192, 256)
    _check("c5_deepseek", 8192, 64, unique=True)


def test_gated_full_size():
    # the paper's best setting uses a budget of 3 replacements per token (Section 5.1) behind the TAE gate;
    # the distribution gate is placed just above the batch's own delta (open) and at it (closed)
    spec = workloads.CONFIGS["c5_deepseek"]
    host = HostLayer(spec, 8192, base=_layers("c5_deepseek")[0])
    _, w = oracle.route_topk(host.f32(host.x), host.f32(host.w_router), host.bias, spec.K)
    tau = safe_threshold(tae_margin(w)[0], 0.15)                  # percentile calibration of Section 3.1
    _check("c5_deepseek", 8192, 64, unique=True, tau=tau, rho=3, beta=0.99)
    _check("c3_mixtral_prefill", 4096, 48, beta=0.5)              # 4 of 8 requested experts offloaded: closed
    _check("c2_mixtral_decode", 8, 8, unique=True, rho=1, beta=0.9)
