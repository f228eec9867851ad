"""Pins for the oracle's Algorithm 1 (buddy substitution) and the permutation (CPU only)."""
import json
import os

import numpy as np
import pytest

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_handworked.json")


def _cases():
    with open(GOLDEN) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"][:40])
@pytest.mark.parametrize("mode", ["unique", "first"])
def test_handworked_algorithm1(case, mode):
    ids = np.array(case["ids"], np.int32)
    w = np.arange(1, ids.size + 1, dtype=np.float64).reshape(ids.shape)
    out, w2, st = oracle.buddy_remap(ids, np.array(case["resident"], bool), np.array(case["table"], np.int32),
                                     H=case["H"], unique=(mode == "unique"), w=w)
    want = np.array(case[mode], np.int32)
    np.testing.assert_array_equal(out, want)
    np.testing.assert_array_equal(w2, np.where(want < 0, 0.0, w))   # dropped -> 0, others untouched
    assert [st["n_miss"], st["n_substituted"], st["n_dropped"]] == case["stats_" + mode]


def _random_problem(seed, T=200, E=24, K=4, R=6, n_res=9, pad=True):
    g = np.random.default_rng(seed)
    ids = np.stack([g.permutation(E)[:K] for _ in range(T)]).astype(np.int32)
    res = np.zeros(E, bool); res[g.permutation(E)[:n_res]] = True
    table = np.stack([g.permutation([j for j in range(E) if j != i])[:R] for i in range(E)]).astype(np.int32)
    if pad:
        table[g.random((E, R)) < 0.15] = -1
    return ids, res, table


def test_all_resident_is_identity():
    # Table 1 "BuddyMoE Hit ... Lossless": nothing missing => nothing rewritten
    ids, _, table = _random_problem(1)
    w = np.random.default_rng(2).random(ids.shape)
    for unique in (False, True):
        out, w2, st = oracle.buddy_remap(ids, np.ones(24, bool), table, unique=unique, w=w)
        np.testing.assert_array_equal(out, ids)
        np.testing.assert_array_equal(w2, w)
        assert st == dict(n_miss=0, n_substituted=0, n_dropped=0)


def test_none_resident_drops_everything():
    ids, _, table = _random_problem(3)
    out, w2, st = oracle.buddy_remap(ids, np.zeros(24, bool), table, w=np.ones(ids.shape))
    assert (out == -1).all() and (w2 == 0).all()
    assert st["n_miss"] == ids.size == st["n_dropped"] and st["n_substituted"] == 0


def test_h_zero_drops_every_miss():
    ids, res, table = _random_problem(4)
    out, _, st = oracle.buddy_remap(ids, res, table, H=0)
    np.testing.assert_array_equal(out, np.where(res[ids], ids, -1))
    assert st["n_substituted"] == 0 and st["n_dropped"] == st["n_miss"] == int((~res[ids]).sum())


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("H", [1, 3, 6])
def test_first_mode_is_a_per_expert_lookup(seed, H):
    # without the U_t test the substitute depends on the expert alone: LUT[e] = first resident row entry
    ids, res, table = _random_problem(seed)
    E, R = table.shape
    tab = table[:, :H]
    ok = (tab >= 0) & res[np.clip(tab, 0, E - 1)]
    first = np.where(ok.any(1), np.take_along_axis(tab, ok.argmax(1)[:, None], 1)[:, 0], -1)
    lut = np.where(res, np.arange(E), first)
    out, _, st = oracle.buddy_remap(ids, res, table, H=H, unique=False)
    np.testing.assert_array_equal(out, lut[ids])
    assert st["n_miss"] == int((~res[ids]).sum())
    assert st["n_dropped"] == int((out < 0).sum())
    assert st["n_miss"] == st["n_substituted"] + st["n_dropped"]


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("unique", [False, True])
def test_output_properties(seed, unique):
    """Properties that Algorithm 1's output must have, checked on the output alone."""
    ids, res, table = _random_problem(100 + seed, pad=(seed % 2 == 0))
    E, R = table.shape
    H = R - (seed % 3)
    out, _, st = oracle.buddy_remap(ids, res, table, H=H, unique=unique)
    live = out >= 0
    assert res[out[live]].all()                                  # every surviving id is resident
    np.testing.assert_array_equal(out[res[ids]], ids[res[ids]])  # resident originals untouched
    n_sub = 0
    for t in range(ids.shape[0]):
        held = set(ids[t].tolist())                              # U_t before any substitution
        for k in range(ids.shape[1]):
            e, o = int(ids[t, k]), int(out[t, k])
            if res[e]:
                continue
            row = table[e, :H].tolist()
            def acceptable(b):
                return 0 <= b < E and res[b] and not (unique and b in held)
            if o >= 0:
                n_sub += 1
                r = row.index(o)
                assert acceptable(o)
                assert not any(acceptable(b) for b in row[:r])   # nothing earlier in the row qualified
                if unique:
                    others = [int(v) for j, v in enumerate(out[t]) if j != k]
                    assert o not in others and o not in ids[t]
                held.add(o)
            else:
                assert not any(acceptable(b) for b in row)       # dropped only when nothing qualified
    assert st["n_substituted"] == n_sub
    assert st["n_miss"] == st["n_substituted"] + st["n_dropped"]


def test_unique_equals_first_when_no_collisions_possible():
    # K = 1: U_t holds only the missing expert itself, which is never its own buddy
    ids, res, table = _random_problem(7, K=1)
    a = oracle.buddy_remap(ids, res, table, unique=False)[0]
    b = oracle.buddy_remap(ids, res, table, unique=True)[0]
    np.testing.assert_array_equal(a, b)


def test_aliasing_in_place():
    ids, res, table = _random_problem(8)
    want = oracle.buddy_remap(ids, res, table, unique=True)[0]
    import ctypes
    buf = ids.copy()
    p = buf.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    r8 = res.astype(np.uint8)
    rc = oracle.lib().bm_oracle_buddy_remap(ids.shape[0], ids.shape[1], 24, 6, 6, 1,
                                            r8.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                            table.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), p, p, None, None)
    assert rc == 0
    np.testing.assert_array_equal(buf, want)


def test_h_above_r_is_an_error():
    ids, res, table = _random_problem(9)
    with pytest.raises(ValueError):
        oracle.buddy_remap(ids, res, table, H=7)


# ---------------------------------------------------------------- permutation


@pytest.mark.parametrize("seed", range(5))
def test_permutation_is_library_stable_sort(seed):
    g = np.random.default_rng(seed)
    T, K, E = 57, 3, 11
    ids = g.integers(-1, E, size=(T, K)).astype(np.int32)
    ids[g.random((T, K)) < 0.2] = -1
    off, perm, inv = oracle.permute(ids, E)
    flat = ids.reshape(-1)
    live = np.nonzero(flat >= 0)[0]
    want = live[np.argsort(flat[live], kind="stable")]
    n = len(live)
    assert off[0] == 0 and off[E] == n
    np.testing.assert_array_equal(perm[:n], want)
    assert (perm[n:] == -1).all()
    np.testing.assert_array_equal(np.diff(off), np.bincount(flat[live], minlength=E))
    assert (inv[flat < 0] == -1).all()
    np.testing.assert_array_equal(inv[perm[:n]], np.arange(n))
    for e in range(E):
        seg = perm[off[e]:off[e + 1]]
        assert (flat[seg] == e).all() and (np.diff(seg) > 0).all()


def test_permutation_empty_and_all_dropped():
    off, perm, inv = oracle.permute(np.full((4, 2), -1, np.int32), 5)
    assert (off == 0).all() and (perm == -1).all() and (inv == -1).all()
    off, perm, inv = oracle.permute(np.zeros((0, 2), np.int32), 5)
    assert (off == 0).all() and perm.size == 0


def test_bitmap_packing_convention():
    m = np.zeros(130, bool); m[[0, 63, 64, 129]] = True
    w = workloads.pack_bitmap(m)
    assert w.dtype == np.uint64 and len(w) == 3
    assert int(w[0]) == (1 | (1 << 63)) and int(w[1]) == 1 and int(w[2]) == 2
