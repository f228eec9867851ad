"""Seeded synthetic MoE-layer workloads.

This module manufactures inputs only: hidden states, router and expert
weights, a router popularity bias, a residency mask and a ranked buddy table.
It serves both the CPU oracle and the HIP path and contains none of the hot
path's arithmetic (no softmax, no top-k, no substitution, no FFN).  Two
input-conditioning steps live here because they define *what the inputs are*:

* rejection of tokens whose leading router logits are closer than a margin
  (so that expert ids do not depend on floating-point summation order), and
* turning a synthetic co-activation count matrix into ranked peer lists
  (the offline stage of the method, Section 3.2 Eq. 4 and Section 3.3: peers
  sorted by conditional co-activation; since the normaliser of Eq. 4 is one
  positive number per pivot, sorting a row of counts gives the same order).

Everything is a pure function of (spec, seed); the random stream is numpy's
Philox counter-based generator keyed by (seed, tensor id, index).
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Tuple

import numpy as np

# --------------------------------------------------------------------------
# bf16 <-> fp32 bit helpers (storage conversion only)
# --------------------------------------------------------------------------


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + rounding) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Layer specification
# --------------------------------------------------------------------------

MARGIN = 1e-3  # minimum gap between adjacent leading router logits

_T_ROUTER, _T_BIAS, _T_GATE, _T_UP, _T_DOWN, _T_SGATE, _T_SUP, _T_SDOWN = range(1, 9)
_T_X, _T_RESID, _T_BUDDY, _T_COACT, _T_RANK = range(16, 21)


@dataclasses.dataclass(frozen=True)
class LayerSpec:
    """Shape and recipe of one synthetic MoE layer.

    d hidden, E routed experts, F expert FFN width, K experts per token,
    R buddy-table width, H search limit (H <= R), n_shared always-on experts.
    """

    name: str
    d: int
    E: int
    F: int
    K: int
    R: int
    H: int
    n_resident: int
    dtype: str = "bf16"          # "bf16" or "f32"
    n_shared: int = 0
    zipf_s: float = 0.0          # 0 => no popularity bias
    rms_norm: bool = True        # normalise each token to ||x||^2 = d
    buddy: str = "coact_pop"     # "shuffle" | "coact_pop" | "coact_lowrank"
    coact_rank: int = 8
    resident: str = "popular"    # "popular" | "alternate" (popularity ranks 1,3,5,..) | "shuffle"
    seed: int = 0xB0DD1E00
    T: Tuple[int, ...] = (16,)   # token counts the config is quoted on

    def replace(self, **kw) -> "LayerSpec":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, LayerSpec] = {
    # tiny fp32 layer
    "c1_tiny": LayerSpec("c1_tiny", d=64, E=8, F=128, K=2, R=3, H=3, n_resident=4,
                         dtype="f32", rms_norm=False, buddy="shuffle",
                         resident="shuffle", seed=0xB0DD1E01, T=(16,)),
    # Mixtral-8x7B-shaped, decode
    "c2_mixtral_decode": LayerSpec("c2_mixtral_decode", d=4096, E=8, F=14336, K=2, R=7, H=7,
                                   n_resident=5, zipf_s=1.1, seed=0xB0DD1E02,
                                   T=(1, 8, 32, 64)),
    # Mixtral-8x7B-shaped, prefill (same layer tensors as c2: same seed)
    "c3_mixtral_prefill": LayerSpec("c3_mixtral_prefill", d=4096, E=8, F=14336, K=2, R=7, H=7,
                                    n_resident=4, zipf_s=1.1, seed=0xB0DD1E02,
                                    resident="alternate", T=(4096,)),
    # Qwen3-30B-A3B-shaped
    "c4_qwen3": LayerSpec("c4_qwen3", d=2048, E=128, F=768, K=8, R=8, H=8, n_resident=64,
                          zipf_s=1.0, buddy="coact_lowrank", coact_rank=8,
                          resident="alternate", seed=0xB0DD1E04, T=(2048,)),
    # DeepSeek-MoE-16B-shaped, 2 shared experts
    "c5_deepseek": LayerSpec("c5_deepseek", d=2048, E=64, F=1408, K=6, R=8, H=8, n_resident=16,
                             n_shared=2, zipf_s=1.0, buddy="coact_lowrank", coact_rank=6,
                             resident="alternate", seed=0xB0DD1E05, T=(8192,)),
}


def _rng(seed: int, tensor: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) ^ tensor, index]))


# --------------------------------------------------------------------------
# Layer tensors
# --------------------------------------------------------------------------


class Layer:
    """The static tensors of one layer: router, bias, residency, buddy table.

    Expert weights are produced per expert on demand (`expert(e)`), because
    the Mixtral-shaped layer holds 1.4e9 weights.
    """

    def __init__(self, spec: LayerSpec):
        self.spec = spec
        s = spec
        sigma = 1.0 / np.sqrt(s.d)
        wr = _rng(s.seed, _T_ROUTER).standard_normal((s.E, s.d), dtype=np.float32) * np.float32(sigma)
        self.w_router = self._store(wr)
        # popularity rank (1 = most popular), a seeded permutation of 1..E
        self.rank = _rng(s.seed, _T_RANK).permutation(s.E).astype(np.int64) + 1
        if s.zipf_s > 0:
            # log of the Zipf pmf at the expert's rank, up to a constant
            self.router_bias = (-s.zipf_s * np.log(self.rank)).astype(np.float32)
        else:
            self.router_bias = None
        self.popularity = self.rank.astype(np.float64) ** (-(s.zipf_s if s.zipf_s > 0 else 1.0))
        self.popularity /= self.popularity.sum()
        self.resident_mask = _choose_resident(s, self.rank)
        self.coact = self._coactivation()
        self.buddy_table = self._buddy_table()

    # ---- storage ---------------------------------------------------------
    def _store(self, a: np.ndarray) -> np.ndarray:
        """fp32 array -> the spec's storage dtype (uint16 bf16 bits or fp32)."""
        return f32_to_bf16_bits(a) if self.spec.dtype == "bf16" else np.ascontiguousarray(a, np.float32)

    def as_f32(self, a: np.ndarray) -> np.ndarray:
        return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a

    # ---- residency -------------------------------------------------------
    def with_residency(self, mask: np.ndarray) -> "Layer":
        """Shallow copy with another residency mask (e.g. all resident)."""
        import copy
        other = copy.copy(self)
        other.resident_mask = np.asarray(mask, dtype=bool).copy()
        return other

    @property
    def bitmap(self) -> np.ndarray:
        """Residency as packed uint64 words: bit (e % 64) of word (e // 64)."""
        return pack_bitmap(self.resident_mask)

    # ---- co-activation counts and buddy lists ----------------------------
    def _coactivation(self) -> Optional[np.ndarray]:
        s = self.spec
        if s.buddy == "shuffle":
            return None
        g = _rng(s.seed, _T_COACT)
        if s.buddy == "coact_pop":
            noise = g.uniform(-0.5, 0.5, size=(s.E, s.E))
            noise = (noise + noise.T) * 0.5
            m = 1.0e6 * np.outer(self.popularity, self.popularity) * (1.0 + noise)
        else:
            # low-rank-plus-noise Gram matrix: a few latent "skills" per expert
            # unit-norm rows, so similarity is about direction and no expert is everyone's buddy
            u = g.gamma(shape=0.5, scale=1.0, size=(s.E, s.coact_rank))
            u /= np.linalg.norm(u, axis=1, keepdims=True)
            n = g.standard_normal((s.E, s.E))
            m = 1.0e3 * (u @ u.T + 0.05 * (n + n.T))
        m = np.rint(np.clip(m, 0.0, None)).astype(np.int64)
        np.fill_diagonal(m, 0)
        return m

    def _buddy_table(self) -> np.ndarray:
        s = self.spec
        table = np.full((s.E, s.R), -1, dtype=np.int32)
        if s.buddy == "shuffle":
            g = _rng(s.seed, _T_BUDDY)
            for i in range(s.E):
                others = np.array([j for j in range(s.E) if j != i])
                table[i, : min(s.R, s.E - 1)] = g.permutation(others)[: s.R]
            return table
        for i in range(s.E):
            peers = ranked_peers(self.coact[i], i)
            n = min(s.R, len(peers))
            table[i, :n] = peers[:n]
        return table

    # ---- expert weights --------------------------------------------------
    def expert(self, e: int, shared: bool = False):
        """(w_gate [F][d], w_up [F][d], w_down [d][F]) of one expert, storage dtype."""
        s = self.spec
        sigma = np.float32(1.0 / np.sqrt(s.d))
        tg, tu, td = (_T_SGATE, _T_SUP, _T_SDOWN) if shared else (_T_GATE, _T_UP, _T_DOWN)
        wg = self._store(_rng(s.seed, tg, e).standard_normal((s.F, s.d), dtype=np.float32) * sigma)
        wu = self._store(_rng(s.seed, tu, e).standard_normal((s.F, s.d), dtype=np.float32) * sigma)
        wd = self._store(_rng(s.seed, td, e).standard_normal((s.d, s.F), dtype=np.float32) * sigma)
        return wg, wu, wd

    def stacked_experts(self, only_resident: bool = False, poison: bool = False,
                        shared: bool = False, workers: int = 4):
        """Stack expert weights into [E][F][d], [E][F][d], [E][d][F] (storage dtype).

        only_resident: weights of non-resident experts are not generated; they
        are left zero, or filled with NaN when `poison` is set (the layer must
        never read them).
        """
        s = self.spec
        n = s.n_shared if shared else s.E
        dt = np.uint16 if s.dtype == "bf16" else np.float32
        wg = np.zeros((n, s.F, s.d), dtype=dt)
        wu = np.zeros((n, s.F, s.d), dtype=dt)
        wd = np.zeros((n, s.d, s.F), dtype=dt)
        nan = np.uint16(0x7FC0) if s.dtype == "bf16" else np.float32(np.nan)

        def fill(e):
            if shared or not only_resident or self.resident_mask[e]:
                wg[e], wu[e], wd[e] = self.expert(e, shared=shared)
            elif poison:
                wg[e].fill(nan); wu[e].fill(nan); wd[e].fill(nan)

        if n * s.F * s.d > (1 << 24) and workers > 1:
            with ThreadPoolExecutor(max_workers=workers) as ex:
                list(ex.map(fill, range(n)))
        else:
            for e in range(n):
                fill(e)
        return wg, wu, wd

    # ---- tokens ----------------------------------------------------------
    def tokens(self, T: int, stream: int = 0) -> Tuple[np.ndarray, int]:
        """Hidden states [T][d] in storage dtype, plus the number of re-draws.

        A token is re-drawn (next sub-stream) while any two adjacent values
        among its K+1 largest router logits are closer than MARGIN; the logits
        for this filter are evaluated in fp64 on the stored (rounded) values.
        """
        s = self.spec
        wr = self.as_f32(self.w_router).astype(np.float64)
        bias = np.zeros(s.E) if self.router_bias is None else self.router_bias.astype(np.float64)
        x = np.empty((T, s.d), dtype=np.float32)
        todo = np.arange(T)
        redraws = 0
        attempt = 0
        while len(todo):
            g = _rng(s.seed, _T_X + 32 * attempt, stream)
            # draw the full [T][d] block of this attempt so a token's value
            # does not depend on which other tokens were re-drawn
            block = g.standard_normal((T, s.d), dtype=np.float32)[todo]
            if s.rms_norm:
                block = block / np.sqrt(np.mean(block.astype(np.float64) ** 2, axis=1, keepdims=True)).astype(np.float32)
            block = self.as_f32(self._store(block))
            z = block.astype(np.float64) @ wr.T + bias
            top = -np.sort(-z, axis=1)[:, : min(s.K + 1, s.E)]
            ok = (top[:, :-1] - top[:, 1:]).min(axis=1) >= MARGIN if top.shape[1] > 1 else np.ones(len(todo), bool)
            x[todo[ok]] = block[ok]
            redraws += int((~ok).sum())
            todo = todo[~ok]
            attempt += 1
            if attempt > 64:
                raise RuntimeError("tie-free rejection did not converge")
        return self._store(x), redraws


def _choose_resident(s: LayerSpec, rank: np.ndarray) -> np.ndarray:
    """The simulated expert cache: which n_resident experts are in device memory."""
    mask = np.zeros(s.E, dtype=bool)
    by_popularity = np.argsort(rank, kind="stable")
    if s.resident == "popular":
        mask[by_popularity[: s.n_resident]] = True
    elif s.resident == "alternate":
        # every other expert by popularity (ranks 1, 3, 5, ...), then the rest in order
        order = np.concatenate([by_popularity[0::2], by_popularity[1::2]])
        mask[order[: s.n_resident]] = True
    else:
        mask[_rng(s.seed, _T_RESID).permutation(s.E)[: s.n_resident]] = True
    return mask


def ranked_peers(counts_row: np.ndarray, pivot: int) -> np.ndarray:
    """Peers of `pivot` with a positive count, by descending count, ties -> lowest id."""
    c = np.asarray(counts_row).astype(np.int64).copy()
    c[pivot] = -1
    order = np.lexsort((np.arange(len(c)), -c))
    return order[c[order] > 0].astype(np.int32)


def pack_bitmap(mask: np.ndarray) -> np.ndarray:
    """bool[E] -> uint64[ceil(E/64)], bit (e % 64) of word (e // 64)."""
    mask = np.asarray(mask, dtype=bool)
    words = np.zeros((len(mask) + 63) // 64, dtype=np.uint64)
    for e in np.nonzero(mask)[0]:
        words[e // 64] |= np.uint64(1) << np.uint64(e % 64)
    return words


# --------------------------------------------------------------------------
# Scaled-down variants for parity tests (same recipe, smaller dimensions)
# --------------------------------------------------------------------------


def scaled(name: str, **kw) -> LayerSpec:
    """A config with some dimensions overridden, e.g. scaled('c4_qwen3', d=256, F=96)."""
    return CONFIGS[name].replace(**kw)


_layer_cache: Dict[LayerSpec, Layer] = {}


def get_layer(spec: LayerSpec) -> Layer:
    """Layers are cached by the fields that determine their tensors."""
    key = spec.replace(name="", T=(), n_resident=0, resident="")
    base = _layer_cache.get(key)
    if base is None:
        base = Layer(spec)
        _layer_cache[key] = base
    if (base.spec.n_resident, base.spec.resident, base.spec.name) == (spec.n_resident, spec.resident, spec.name):
        return base
    # same tensors, different residency budget (c2 vs c3)
    lay = Layer.__new__(Layer)
    lay.__dict__.update(base.__dict__)
    lay.spec = spec
    lay.resident_mask = _choose_resident(spec, base.rank)
    return lay
