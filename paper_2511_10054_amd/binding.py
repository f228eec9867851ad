"""ctypes binding of include/buddymoe.h (and the bench aid of include/buddymoe_bench.h).  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
# BUDDYMOE_LIBRARY: another build of the same library (e.g. one with host-side sanitizers) instead of the in-tree one
_LIB_PATH = os.environ.get("BUDDYMOE_LIBRARY") or os.path.join(_HERE, "libbuddymoe.so")
_lib = None

BM_F32, BM_BF16 = 0, 1
BM_RENORM_TOPK, BM_REMAP_UNIQUE, BM_Y_F32 = 1, 2, 4
BM_GATE_TAE, BM_GATE_MARGIN, BM_REPLACE_BUDGET, BM_GATE_DIST, BM_PSI_TOKEN = 8, 16, 32, 64, 128


class BuddyMoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {bm_strerror(status)} (status {status})")


class LayerDesc(ctypes.Structure):
    _fields_ = [("T", ctypes.c_int32), ("d", ctypes.c_int32), ("E", ctypes.c_int32), ("F", ctypes.c_int32),
                ("K", ctypes.c_int32), ("n_shared", ctypes.c_int32), ("R", ctypes.c_int32), ("H", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("flags", ctypes.c_uint32), ("tae_tau", ctypes.c_float),
                ("margin_gamma", ctypes.c_float), ("rho", ctypes.c_int32), ("dist_beta", ctypes.c_float),
                ("psi_eta", ctypes.c_float)]


class Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("w_router", "router_bias", "w_gate", "w_up", "w_down", "ws_gate", "ws_up", "ws_down",
                 "wp_gateup", "wp_down", "wsp_gateup", "wsp_down", "buddy_q")]


class DebugOut(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("ids", "ids_remapped", "w", "offsets", "perm", "inv_perm", "stats")] + \
               [("stage_events", ctypes.c_void_p * 5)]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads libbuddymoe.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2511_10054_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int
        lib.bm_strerror.restype = ctypes.c_char_p
        lib.bm_strerror.argtypes = [i32]
        lib.bm_workspace_bytes.restype = ctypes.c_size_t
        lib.bm_workspace_bytes.argtypes = [ctypes.POINTER(LayerDesc)]
        lib.bm_validate_tables.argtypes = [ctypes.POINTER(LayerDesc), vp, vp]
        lib.bm_packed_bytes.restype = ctypes.c_size_t
        lib.bm_packed_bytes.argtypes = [ctypes.POINTER(LayerDesc), i32]
        lib.bm_pack_weights.argtypes = [ctypes.POINTER(LayerDesc), ctypes.POINTER(Weights), vp, vp]
        lib.bm_pack_weights.restype = i32
        lib.bm_route_topk.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp]
        lib.bm_coactivation_accumulate.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp]
        lib.bm_build_buddy_table.argtypes = [ctypes.POINTER(LayerDesc), vp, ctypes.c_float, vp, vp, vp, vp]
        lib.bm_buddy_remap.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, vp]
        lib.bm_permute_by_expert.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.bm_moe_forward.argtypes = [ctypes.POINTER(LayerDesc), vp, ctypes.POINTER(Weights), vp, vp, vp, vp,
                                       ctypes.c_size_t, ctypes.POINTER(DebugOut), vp]
        lib.bm_moe_forward_static.argtypes = [ctypes.POINTER(LayerDesc), vp, ctypes.POINTER(Weights), vp, vp, vp,
                                              ctypes.POINTER(DebugOut), vp]
        lib.bm_moe_forward_static.restype = i32
        lib.bm_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        lib.bm_stream_read.restype = i32
        for f in (lib.bm_validate_tables, lib.bm_route_topk, lib.bm_buddy_remap, lib.bm_permute_by_expert,
                  lib.bm_moe_forward, lib.bm_coactivation_accumulate, lib.bm_build_buddy_table):
            f.restype = i32
        _lib = lib
    return _lib


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array, None for None."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        assert t.is_contiguous(), "tensors must be contiguous"
        return t.data_ptr()
    return t.ctypes.data


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str):
    if rc != 0:
        raise BuddyMoEError(rc, where)


def bm_strerror(status: int) -> str:
    return load_library().bm_strerror(status).decode()


def bm_workspace_bytes(desc: LayerDesc) -> int:
    return int(load_library().bm_workspace_bytes(ctypes.byref(desc)))


def bm_validate_tables(desc: LayerDesc, bitmap_host, table_host) -> int:
    """Host check of a bitmap (numpy uint64) and buddy table (numpy int32); returns the status."""
    return int(load_library().bm_validate_tables(ctypes.byref(desc), _ptr(bitmap_host), _ptr(table_host)))


def bm_route_topk(desc: LayerDesc, x, w_router, bias, ids, w, stream: Optional[int] = None):
    _check(load_library().bm_route_topk(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(bias), _ptr(ids),
                                        _ptr(w), _stream() if stream is None else stream), "bm_route_topk")


def bm_buddy_remap(desc: LayerDesc, bitmap, table, ids_in, ids_out, w=None, stats=None,
                   stream: Optional[int] = None):
    _check(load_library().bm_buddy_remap(ctypes.byref(desc), _ptr(bitmap), _ptr(table), _ptr(ids_in),
                                         _ptr(ids_out), _ptr(w), _ptr(stats),
                                         _stream() if stream is None else stream), "bm_buddy_remap")


def bm_coactivation_accumulate(desc: LayerDesc, ids, activations, coactivations, stream: Optional[int] = None):
    """Adds the batch's counts to activations [E] / coactivations [E][E] (device int64)."""
    _check(load_library().bm_coactivation_accumulate(ctypes.byref(desc), _ptr(ids), _ptr(activations),
                                                     _ptr(coactivations),
                                                     _stream() if stream is None else stream),
           "bm_coactivation_accumulate")


def bm_build_buddy_table(desc: LayerDesc, coactivations, alpha: float, table, list_len=None, q=None,
                         stream: Optional[int] = None):
    _check(load_library().bm_build_buddy_table(ctypes.byref(desc), _ptr(coactivations), ctypes.c_float(alpha),
                                               _ptr(table), _ptr(list_len), _ptr(q),
                                               _stream() if stream is None else stream), "bm_build_buddy_table")


def bm_permute_by_expert(desc: LayerDesc, ids_remapped, offsets, perm, inv_perm, workspace,
                         stream: Optional[int] = None):
    _check(load_library().bm_permute_by_expert(ctypes.byref(desc), _ptr(ids_remapped), _ptr(offsets), _ptr(perm),
                                               _ptr(inv_perm), _ptr(workspace),
                                               workspace.numel() * workspace.element_size(),
                                               _stream() if stream is None else stream), "bm_permute_by_expert")


def bm_moe_forward(desc: LayerDesc, x, weights: Weights, bitmap, table, y, workspace, dbg: Optional[dict] = None,
                   stream: Optional[int] = None):
    """dbg: optional dict of device tensors keyed by bm_debug_out member names;
    the key "stage_events" takes a sequence of 5 hipEvent_t handles (ints)."""
    d = _debug_struct(dbg)
    _check(load_library().bm_moe_forward(ctypes.byref(desc), _ptr(x), ctypes.byref(weights), _ptr(bitmap),
                                         _ptr(table), _ptr(y), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(),
                                         ctypes.byref(d) if d is not None else None,
                                         _stream() if stream is None else stream), "bm_moe_forward")


def _debug_struct(dbg: Optional[dict]):
    d = None
    if dbg:
        d = DebugOut(**{k: _ptr(v) for k, v in dbg.items() if k != "stage_events"})
        if dbg.get("stage_events") is not None:
            d.stage_events = (ctypes.c_void_p * 5)(*dbg["stage_events"])
    return d


BM_STATIC_WORKSPACE_BYTES = 32 << 20


def bm_moe_forward_static(desc: LayerDesc, x, weights: Weights, bitmap, table, y, dbg: Optional[dict] = None,
                          stream: Optional[int] = None):
    """bm_moe_forward on the library's built-in scratch array: no workspace argument, nothing allocated."""
    d = _debug_struct(dbg)
    _check(load_library().bm_moe_forward_static(ctypes.byref(desc), _ptr(x), ctypes.byref(weights), _ptr(bitmap),
                                                _ptr(table), _ptr(y), ctypes.byref(d) if d is not None else None,
                                                _stream() if stream is None else stream), "bm_moe_forward_static")


def make_weights(w_router, router_bias, w_gate, w_up, w_down, ws_gate=None, ws_up=None, ws_down=None,
                 wp_gateup=None, wp_down=None, wsp_gateup=None, wsp_down=None, buddy_q=None) -> Weights:
    return Weights(*[_ptr(t) for t in (w_router, router_bias, w_gate, w_up, w_down, ws_gate, ws_up, ws_down,
                                       wp_gateup, wp_down, wsp_gateup, wsp_down, buddy_q)])


def bm_stream_read(src, sink, stream: Optional[int] = None):
    """Measurement aid: one streaming read of the whole tensor `src` (see include/buddymoe_bench.h)."""
    _check(load_library().bm_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                         _stream() if stream is None else stream), "bm_stream_read")


def bm_packed_bytes(desc: LayerDesc, which: int) -> int:
    return int(load_library().bm_packed_bytes(ctypes.byref(desc), which))


def bm_pack_weights(desc: LayerDesc, weights: Weights, bitmap=None, stream: Optional[int] = None):
    """Fills the packed buffers named in `weights` (wp_*/wsp_*) from its public arrays."""
    _check(load_library().bm_pack_weights(ctypes.byref(desc), ctypes.byref(weights), _ptr(bitmap),
                                          _stream() if stream is None else stream), "bm_pack_weights")
