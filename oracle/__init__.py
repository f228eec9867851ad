"""ctypes front end of the CPU oracle (oracle/bm_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.

All functions take and return numpy arrays; floating-point inputs are fp32
(widen bf16 bit patterns first), floating-point outputs are fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bm_oracle.cpp")
_LIB = os.path.join(_HERE, "libbm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c++17", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (tests load it in a child process
    through BM_ORACLE_LIBRARY, with the sanitizer runtime preloaded)."""
    cmd = ["g++", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fopenmp", "-fPIC", "-shared", "-std=c++17", "-o", out_path, _SRC]
    subprocess.run(cmd, check=True)
    return out_path


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        override = os.environ.get("BM_ORACLE_LIBRARY")     # a differently built copy of the same source (sanitizer run)
        if override:
            _lib = ctypes.CDLL(override)
        else:
            build()
            _lib = ctypes.CDLL(_LIB)
    return _lib


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


_F, _D, _I32, _I64, _U8 = ctypes.c_float, ctypes.c_double, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint8


def num_threads() -> int:
    return int(lib().bm_oracle_num_threads())


def router_logits(x, w_router, bias=None) -> np.ndarray:
    x, w_router, bias = _f32(x), _f32(w_router), _f32(bias)
    T, d = x.shape
    E = w_router.shape[0]
    assert w_router.shape == (E, d)
    z = np.empty((T, E), dtype=np.float64)
    rc = lib().bm_oracle_router_logits(T, d, E, _p(x, _F), _p(w_router, _F), _p(bias, _F), _p(z, _D))
    assert rc == 0
    return z


def topk_gates(z, K: int, renorm: bool = True):
    z = np.ascontiguousarray(z, dtype=np.float64)
    T, E = z.shape
    ids = np.empty((T, K), dtype=np.int32)
    w = np.empty((T, K), dtype=np.float64)
    rc = lib().bm_oracle_topk_gates(T, E, K, int(renorm), _p(z, _D), _p(ids, _I32), _p(w, _D))
    if rc:
        raise ValueError("K > E")
    return ids, w


def route_topk(x, w_router, bias, K: int, renorm: bool = True):
    return topk_gates(router_logits(x, w_router, bias), K, renorm)


def tae(w) -> np.ndarray:
    w = np.ascontiguousarray(w, dtype=np.float64)
    T, K = w.shape
    out = np.empty(T, dtype=np.float64)
    assert lib().bm_oracle_tae(T, K, _p(w, _D), _p(out, _D)) == 0
    return out


def buddy_remap(ids, resident_mask, table, H: Optional[int] = None, unique: bool = False, w=None):
    """Returns (ids_remapped, w_after_drops or None, stats dict)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    res = np.ascontiguousarray(np.asarray(resident_mask, dtype=bool).astype(np.uint8))
    E = len(res)
    table = np.ascontiguousarray(table, dtype=np.int32)
    assert table.shape[0] == E
    R = table.shape[1]
    H = R if H is None else H
    out = np.empty_like(ids)
    w2 = None if w is None else np.array(w, dtype=np.float64, order="C", copy=True)
    stats = np.zeros(3, dtype=np.int64)
    rc = lib().bm_oracle_buddy_remap(T, K, E, R, H, int(unique), _p(res, _U8), _p(table, _I32),
                                     _p(ids, _I32), _p(out, _I32), _p(w2, _D), _p(stats, _I64))
    if rc:
        raise ValueError("H must be in [0, R]")
    return out, w2, dict(n_miss=int(stats[0]), n_substituted=int(stats[1]), n_dropped=int(stats[2]))


def distribution_delta(ids, resident_mask):
    """Eq. 2: (delta, |R(B)|, offloaded among R(B)) for the batch of routed ids [T][K]."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    res = np.ascontiguousarray(np.asarray(resident_mask, dtype=bool).astype(np.uint8))
    counts = np.zeros(2, dtype=np.int64)
    f = lib().bm_oracle_distribution_delta
    f.restype = ctypes.c_double
    f.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 3
    delta = f(T, K, len(res), res.ctypes.data, ids.ctypes.data, counts.ctypes.data)
    return float(delta), int(counts[0]), int(counts[1])


def _stats_dict(stats):
    return dict(n_miss=int(stats[0]), n_substituted=int(stats[1]), n_dropped=int(stats[2]),
                n_requested=int(stats[3]), n_requested_offloaded=int(stats[4]), bypassed=int(stats[5]))


_GATE_ARGS = [ctypes.c_int, _D, ctypes.c_int, _D, ctypes.c_int, ctypes.c_int, ctypes.c_int, _D]


def _gate_values(tau, gamma, rho, beta):
    return (int(tau is not None), float(tau or 0.0), int(gamma is not None), float(gamma or 0.0),
            int(rho is not None), int(rho or 0), int(beta is not None), float(beta or 0.0))


def buddy_remap_gated(ids, resident_mask, table, w=None, H: Optional[int] = None, unique: bool = False,
                      tau: Optional[float] = None, gamma: Optional[float] = None, rho: Optional[int] = None,
                      beta: Optional[float] = None):
    """Algorithm 1 behind the TAE gate (tau), the margin gate (gamma), the distribution gate (beta) and
    the budget (rho); a None switches that gate off.  Returns (ids_remapped, w_after_drops, stats dict)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    res = np.ascontiguousarray(np.asarray(resident_mask, dtype=bool).astype(np.uint8))
    E = len(res)
    table = np.ascontiguousarray(table, dtype=np.int32)
    R = table.shape[1]
    H = R if H is None else H
    out = np.empty_like(ids)
    w2 = None if w is None else np.array(w, dtype=np.float64, order="C", copy=True)
    stats = np.zeros(6, dtype=np.int64)
    f = lib().bm_oracle_buddy_remap_gated
    f.argtypes = [ctypes.c_int] * 6 + _GATE_ARGS + [ctypes.c_void_p] * 6
    rc = f(T, K, E, R, H, int(unique), *_gate_values(tau, gamma, rho, beta), res.ctypes.data, table.ctypes.data,
           ids.ctypes.data, out.ctypes.data, None if w2 is None else w2.ctypes.data, stats.ctypes.data)
    if rc:
        raise ValueError("H must be in [0, R]; the TAE and margin gates need w")
    return out, w2, _stats_dict(stats)


def coactivation(ids, E: int, A=None, M=None):
    """Section 3.2 counts of one batch of routed ids, added to A [E] / M [E][E] (int64; created if None)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    A = np.zeros(E, np.int64) if A is None else A
    M = np.zeros((E, E), np.int64) if M is None else M
    assert A.dtype == np.int64 and M.dtype == np.int64 and M.flags.c_contiguous
    assert lib().bm_oracle_coactivation(T, K, E, _p(ids, _I32), _p(A, _I64), _p(M, _I64)) == 0
    return A, M


def build_buddy_lists(M, alpha: float, k_max: int):
    """Eq. 4-6: (table [E][k_max] padded with -1, lengths [E], q of each entry [E][k_max])."""
    M = np.ascontiguousarray(M, dtype=np.int64)
    E = M.shape[0]
    table = np.empty((E, k_max), np.int32)
    length = np.empty(E, np.int32)
    q = np.empty((E, k_max), np.float64)
    f = lib().bm_oracle_build_buddy_lists
    f.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, _D, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert f(E, k_max, M.ctypes.data, float(alpha), table.ctypes.data, length.ctypes.data, q.ctypes.data) == 0
    return table, length, q


def softmax_all(z) -> np.ndarray:
    z = np.ascontiguousarray(z, dtype=np.float64)
    p = np.empty_like(z)
    assert lib().bm_oracle_softmax(z.shape[0], z.shape[1], _p(z, _D), _p(p, _D)) == 0
    return p


def buddy_remap_psi(ids, resident_mask, table, q, zhat, eta: float, w=None, H: Optional[int] = None,
                    unique: bool = False, tau=None, gamma=None, rho=None, beta=None):
    """Eq. 3 (kappa = 0): the acceptable buddy of largest q * (1 + eta * zhat) instead of the first one.
    Returns (ids_remapped, w_after_drops, stats dict, per-token decision margin)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    res = np.ascontiguousarray(np.asarray(resident_mask, dtype=bool).astype(np.uint8))
    E = len(res)
    table = np.ascontiguousarray(table, dtype=np.int32)
    R = table.shape[1]
    H = R if H is None else H
    q = np.ascontiguousarray(q, dtype=np.float64)
    zhat = np.ascontiguousarray(zhat, dtype=np.float64)
    assert q.shape == (E, R) and zhat.shape == (T, E)
    out = np.empty_like(ids)
    w2 = None if w is None else np.array(w, dtype=np.float64, order="C", copy=True)
    stats = np.zeros(6, dtype=np.int64)
    margin = np.empty(T, dtype=np.float64)
    f = lib().bm_oracle_buddy_remap_psi
    f.argtypes = [ctypes.c_int] * 6 + _GATE_ARGS + [ctypes.c_int, _D] + [ctypes.c_void_p] * 9
    rc = f(T, K, E, R, H, int(unique), *_gate_values(tau, gamma, rho, beta), 1, float(eta), q.ctypes.data,
           zhat.ctypes.data, res.ctypes.data, table.ctypes.data, ids.ctypes.data, out.ctypes.data,
           None if w2 is None else w2.ctypes.data, stats.ctypes.data, margin.ctypes.data)
    if rc:
        raise ValueError("bad arguments")
    return out, w2, _stats_dict(stats), margin


def permute(ids, E: int):
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    offsets = np.empty(E + 1, dtype=np.int32)
    perm = np.empty(T * K, dtype=np.int32)
    inv = np.empty(T * K, dtype=np.int32)
    assert lib().bm_oracle_permute(T, K, E, _p(ids, _I32), _p(offsets, _I32), _p(perm, _I32), _p(inv, _I32)) == 0
    return offsets, perm, inv


def expert_ffn(w_gate, w_up, w_down, x) -> np.ndarray:
    w_gate, w_up, w_down, x = _f32(w_gate), _f32(w_up), _f32(w_down), _f32(x)
    F, d = w_gate.shape
    assert w_up.shape == (F, d) and w_down.shape == (d, F) and x.shape == (d,)
    out = np.empty(d, dtype=np.float64)
    assert lib().bm_oracle_expert_ffn(d, F, _p(w_gate, _F), _p(w_up, _F), _p(w_down, _F), _p(x, _F), _p(out, _D)) == 0
    return out


def experts_combine(x, ids, w, w_gate, w_up, w_down, ws_gate=None, ws_up=None, ws_down=None) -> np.ndarray:
    x, w_gate, w_up, w_down = _f32(x), _f32(w_gate), _f32(w_up), _f32(w_down)
    ws_gate, ws_up, ws_down = _f32(ws_gate), _f32(ws_up), _f32(ws_down)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float64)
    T, d = x.shape
    E, F, _ = w_gate.shape
    K = ids.shape[1]
    n_shared = 0 if ws_gate is None else ws_gate.shape[0]
    assert w_up.shape == (E, F, d) and w_down.shape == (E, d, F)
    y = np.empty((T, d), dtype=np.float64)
    rc = lib().bm_oracle_experts_combine(T, d, E, F, K, n_shared, _p(x, _F), _p(ids, _I32), _p(w, _D),
                                         _p(w_gate, _F), _p(w_up, _F), _p(w_down, _F),
                                         _p(ws_gate, _F), _p(ws_up, _F), _p(ws_down, _F), _p(y, _D))
    assert rc == 0
    return y


def moe_forward(x, w_router, bias, w_gate, w_up, w_down, resident_mask, table, K: int,
                H: Optional[int] = None, renorm: bool = True, unique: bool = False,
                ws_gate=None, ws_up=None, ws_down=None, tau=None, gamma=None, rho=None, beta=None,
                eta=None, q=None):
    """Whole layer. Returns dict(y, ids, ids_remapped, w, stats).  tau / gamma / rho: the TAE gate,
    margin gate, replacement budget and distribution gate (beta) in front of Algorithm 1 (None = off)."""
    x, w_router, bias = _f32(x), _f32(w_router), _f32(bias)
    w_gate, w_up, w_down = _f32(w_gate), _f32(w_up), _f32(w_down)
    ws_gate, ws_up, ws_down = _f32(ws_gate), _f32(ws_up), _f32(ws_down)
    T, d = x.shape
    E, F, _ = w_gate.shape
    res = np.ascontiguousarray(np.asarray(resident_mask, dtype=bool).astype(np.uint8))
    table = np.ascontiguousarray(table, dtype=np.int32)
    R = table.shape[1]
    H = R if H is None else H
    n_shared = 0 if ws_gate is None else ws_gate.shape[0]
    y = np.empty((T, d), dtype=np.float64)
    ids = np.empty((T, K), dtype=np.int32)
    ids2 = np.empty((T, K), dtype=np.int32)
    w = np.empty((T, K), dtype=np.float64)
    stats = np.zeros(6, dtype=np.int64)
    if eta is not None:
        # token-aware buddy priority (Eq. 3): q [E][R] of the table entries, zhat = softmax over all experts
        q = np.ascontiguousarray(q, dtype=np.float64)
        margin = np.empty(T, dtype=np.float64)
        f = lib().bm_oracle_moe_forward_psi
        f.argtypes = [ctypes.c_int] * 10 + _GATE_ARGS + [_D] + [ctypes.c_void_p] * 18
        vp = lambda a: None if a is None else a.ctypes.data
        rc = f(T, d, E, F, K, n_shared, R, H, int(renorm), int(unique), *_gate_values(tau, gamma, rho, beta),
               float(eta), vp(q), vp(x), vp(w_router), vp(bias), vp(w_gate), vp(w_up), vp(w_down), vp(ws_gate),
               vp(ws_up), vp(ws_down), vp(res), vp(table), vp(y), vp(ids), vp(ids2), vp(w), vp(stats), vp(margin))
        if rc:
            raise ValueError("bad shape")
        return dict(y=y, ids=ids, ids_remapped=ids2, w=w, stats=_stats_dict(stats), margin=margin)
    if tau is None and gamma is None and rho is None and beta is None:
        rc = lib().bm_oracle_moe_forward(T, d, E, F, K, n_shared, R, H, int(renorm), int(unique),
                                         _p(x, _F), _p(w_router, _F), _p(bias, _F),
                                         _p(w_gate, _F), _p(w_up, _F), _p(w_down, _F),
                                         _p(ws_gate, _F), _p(ws_up, _F), _p(ws_down, _F),
                                         _p(res, _U8), _p(table, _I32), _p(y, _D), _p(ids, _I32),
                                         _p(ids2, _I32), _p(w, _D), _p(stats, _I64))
    else:
        f = lib().bm_oracle_moe_forward_gated
        f.argtypes = [ctypes.c_int] * 10 + _GATE_ARGS + [ctypes.c_void_p] * 16
        vp = lambda a: None if a is None else a.ctypes.data
        rc = f(T, d, E, F, K, n_shared, R, H, int(renorm), int(unique), *_gate_values(tau, gamma, rho, beta),
               vp(x), vp(w_router), vp(bias), vp(w_gate), vp(w_up), vp(w_down), vp(ws_gate), vp(ws_up),
               vp(ws_down), vp(res), vp(table), vp(y), vp(ids), vp(ids2), vp(w), vp(stats))
    if rc:
        raise ValueError("bad shape")
    return dict(y=y, ids=ids, ids_remapped=ids2, w=w, stats=_stats_dict(stats))

