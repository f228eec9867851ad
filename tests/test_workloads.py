"""The synthetic-input recipe: determinism, structure, margins (CPU only)."""
import numpy as np
import pytest

import oracle
import workloads
from workloads import CONFIGS, MARGIN


def test_bf16_roundtrip_and_rounding():
    a = np.array([1.0, 1.00390625, 1.005859375, -2.5, 0.0, 3.0e38], np.float32)
    b = workloads.f32_to_bf16_bits(a)
    back = workloads.bf16_bits_to_f32(b)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even (1.0)
    np.testing.assert_array_equal(back[:5], [1.0, 1.0, 1.0078125, -2.5, 0.0])
    np.testing.assert_array_equal(workloads.f32_to_bf16_bits(back), b)
    import torch
    t = torch.randn(1000, dtype=torch.float32)
    want = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(workloads.f32_to_bf16_bits(t.numpy()), want)


@pytest.mark.parametrize("name", list(CONFIGS))
def test_static_tensors(name):
    spec = CONFIGS[name]
    small = spec.replace(d=min(spec.d, 128), F=min(spec.F, 96))
    lay = workloads.get_layer(small)
    assert lay.resident_mask.sum() == spec.n_resident
    tab = lay.buddy_table
    assert tab.shape == (spec.E, spec.R) and tab.dtype == np.int32
    for i in range(spec.E):
        row = tab[i][tab[i] >= 0]
        assert len(set(row.tolist())) == len(row) and i not in row and (row < spec.E).all()
    if lay.coact is not None:
        m = lay.coact
        assert (m == m.T).all() and (np.diag(m) == 0).all() and (m >= 0).all()
        # ranked by conditional co-activation (Eq. 4): q is non-increasing along each row
        q = m / np.maximum(m.sum(1, keepdims=True), 1)
        for i in range(spec.E):
            row = tab[i][tab[i] >= 0]
            qs = q[i, row]
            assert (np.diff(qs) <= 0).all()
            if len(row) < spec.E - 1 and len(row) == spec.R:
                rest = np.setdiff1d(np.arange(spec.E), np.append(row, i))
                assert q[i, rest].max() <= qs[-1]
    if spec.resident == "popular":
        assert set(np.nonzero(lay.resident_mask)[0]) == set(np.argsort(lay.rank)[: spec.n_resident])
    again = workloads.Layer(small)
    np.testing.assert_array_equal(again.w_router, lay.w_router)
    np.testing.assert_array_equal(again.buddy_table, tab)
    np.testing.assert_array_equal(again.expert(1)[2], lay.expert(1)[2])


@pytest.mark.parametrize("name", ["c1_tiny", "c2_mixtral_decode", "c4_qwen3"])
def test_tokens_have_the_logit_margin(name):
    spec = CONFIGS[name].replace(d=min(CONFIGS[name].d, 256), F=32)
    lay = workloads.get_layer(spec)
    x, redraws = lay.tokens(300)
    xf = lay.as_f32(x)
    z = oracle.router_logits(xf, lay.as_f32(lay.w_router), lay.router_bias)
    top = -np.sort(-z, axis=1)[:, : spec.K + 1]
    assert (top[:, :-1] - top[:, 1:]).min() >= MARGIN * (1 - 1e-9)
    if spec.rms_norm:
        np.testing.assert_allclose((xf.astype(np.float64) ** 2).mean(1), 1.0, rtol=2e-2)
    x2, _ = lay.tokens(300)
    np.testing.assert_array_equal(x, x2)
    x3, _ = lay.tokens(300, stream=1)
    assert not np.array_equal(x, x3)


def test_c3_remap_fraction_is_in_the_stated_band():
    # the prefill config keeps 4 of 8 experts: 30-50 % of assignments are rewritten
    spec = CONFIGS["c3_mixtral_prefill"].replace(F=32)
    lay = workloads.get_layer(spec)
    x, _ = lay.tokens(1024)
    ids, w = oracle.route_topk(lay.as_f32(x), lay.as_f32(lay.w_router), lay.router_bias, spec.K)
    _, _, st = oracle.buddy_remap(ids, lay.resident_mask, lay.buddy_table)
    frac = st["n_substituted"] / ids.size
    assert 0.30 <= frac <= 0.50, frac
    assert st["n_dropped"] == 0          # full-length lists: some buddy is always resident


def test_c5_drops_some_assignments():
    spec = CONFIGS["c5_deepseek"].replace(F=32, d=512)
    lay = workloads.get_layer(spec)
    x, _ = lay.tokens(1024)
    ids, w = oracle.route_topk(lay.as_f32(x), lay.as_f32(lay.w_router), lay.router_bias, spec.K)
    _, _, st = oracle.buddy_remap(ids, lay.resident_mask, lay.buddy_table, H=spec.H)
    assert st["n_dropped"] > 0 and st["n_substituted"] > st["n_dropped"]


@pytest.mark.parametrize("name", list(CONFIGS))
def test_fp64_topk_definition_gives_the_oracles_ids(name):
    # The oracle takes its top-k decision on logits rounded to fp32.  On the generated inputs (full hidden
    # size, the token counts the configs are quoted on, capped at 2048) the plain definition - the K largest
    # fp64 logits in descending order - selects the same ids in the same slots, so the rounding is immaterial.
    spec = CONFIGS[name].replace(F=32)
    lay = workloads.get_layer(spec)
    for T in sorted({min(t, 2048) for t in spec.T}):
        x, _ = lay.tokens(T)
        z = oracle.router_logits(lay.as_f32(x), lay.as_f32(lay.w_router), lay.router_bias)
        ids, _ = oracle.topk_gates(z, spec.K)
        want = np.argsort(-z, axis=1, kind="stable")[:, : spec.K]
        np.testing.assert_array_equal(ids, want)
