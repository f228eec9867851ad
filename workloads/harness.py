"""Shared helpers of the tests: workload -> host fp32 arrays for the oracle and
device tensors for the HIP library."""
from __future__ import annotations

import numpy as np

from . import get_layer as _get_layer


def err_metric(y, ref):
    """max_i |y_i - ref_i| / max(|ref_i|, rms(ref)): relative error with the
    denominator floored at the output's rms, so near-zero entries do not dominate."""
    y = np.asarray(y, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref ** 2))) or 1.0
    return float(np.max(np.abs(y - ref) / np.maximum(np.abs(ref), rms)))


def err_unfloored(y, ref):
    """max_i |y_i - ref_i| / |ref_i| over the entries with ref_i != 0: the plain elementwise relative error
    (dominated by outputs that cancel to almost nothing); reported beside err_metric, not bounded."""
    y = np.asarray(y, np.float64)
    ref = np.asarray(ref, np.float64)
    nz = ref != 0
    return float(np.max(np.abs(y - ref)[nz] / np.abs(ref)[nz])) if nz.any() else 0.0


def edge_tokens(offsets, perm, K, tile_rows=256, cap=None, seed=0):
    """Tokens whose rows sit where tiling mistakes hide, from the grouping (offsets [E+1], perm): the first and
    last row of every expert group, and one seeded row from each 128-row half of every `tile_rows`-row tile of
    every group (the second half of a group's last tile may be partial or empty).  With `cap`, the tile-half
    rows are thinned to keep about `cap` tokens; the group-edge tokens always stay."""
    offsets = np.asarray(offsets, np.int64)
    perm = np.asarray(perm, np.int64)
    g = np.random.default_rng(seed)
    edge, inner = [], []
    for e in range(len(offsets) - 1):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi <= lo:
            continue
        edge += [lo, hi - 1]
        for t0 in range(lo, hi, tile_rows):
            for h0 in (t0, t0 + 128):
                h1 = min(h0 + 128, hi, t0 + tile_rows)
                if h1 > h0:
                    inner.append(int(g.integers(h0, h1)))
    edge = np.unique(perm[np.array(edge, np.int64)] // K) if edge else np.zeros(0, np.int64)
    inner = np.unique(perm[np.array(inner, np.int64)] // K) if inner else np.zeros(0, np.int64)
    inner = np.setdiff1d(inner, edge)
    if cap is not None and len(edge) + len(inner) > cap:
        inner = g.permutation(inner)[: max(cap - len(edge), 0)]
    return np.unique(np.concatenate([edge, inner])).astype(np.int64)


class HostLayer:
    """Host-side view of one workload: storage arrays and fp32 views for the oracle."""

    def __init__(self, spec, T, stream=0, mask=None, only_resident=False, poison=False, base=None):
        """base: another HostLayer of the same spec whose weight arrays are reused."""
        self.spec = spec
        lay = _get_layer(spec)
        if mask is not None:
            lay = lay.with_residency(mask)
        self.lay = lay
        self.T = T
        self.x, self.redraws = lay.tokens(T, stream) if T > 0 else (np.zeros((0, spec.d), np.uint16 if spec.dtype == "bf16" else np.float32), 0)
        if base is not None:
            self.wg, self.wu, self.wd, self.sg, self.su, self.sd = base.wg, base.wu, base.wd, base.sg, base.su, base.sd
        else:
            self.wg, self.wu, self.wd = lay.stacked_experts(only_resident=only_resident, poison=poison)
            self.sg = self.su = self.sd = None
            if spec.n_shared:
                self.sg, self.su, self.sd = lay.stacked_experts(shared=True)
        self.mask = lay.resident_mask
        self.bitmap = lay.bitmap
        self.table = lay.buddy_table
        self.w_router = lay.w_router
        self.bias = lay.router_bias

    def f32(self, a):
        return None if a is None else self.lay.as_f32(a)

    def oracle_forward(self, oracle, unique=False, renorm=True, H=None, rows=None, tau=None, gamma=None, rho=None, beta=None,
                       eta=None, q=None):
        """Oracle on all tokens or on the token subset `rows` (tokens are independent)."""
        x = self.f32(self.x)
        if rows is not None:
            assert beta is None, "the distribution gate looks at the whole batch"
            x = x[rows]
        # non-resident experts are never read by the oracle's FFN either; NaN poison is harmless
        return oracle.moe_forward(x, self.f32(self.w_router), self.bias, self.f32(self.wg), self.f32(self.wu),
                                  self.f32(self.wd), self.mask, self.table, self.spec.K,
                                  H=self.spec.H if H is None else H, renorm=renorm, unique=unique,
                                  ws_gate=self.f32(self.sg), ws_up=self.f32(self.su), ws_down=self.f32(self.sd),
                                  tau=tau, gamma=gamma, rho=rho, beta=beta, eta=eta, q=q)


def to_device(a, device="cuda"):
    """numpy storage array (uint16 bf16 bits / fp32 / ints) -> torch tensor on the GPU."""
    import torch
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


class DeviceLayer:
    """Uploads a HostLayer and runs the library through the Python binding."""

    def __init__(self, host: HostLayer, unique=False, renorm=True, H=None, y_f32=False, base=None, pack=False,
                 tau=None, gamma=None, rho=None, beta=None, eta=None, q=None):
        """base: another DeviceLayer whose uploaded (and packed) weights are reused.
        pack: also build the fragment-major weight copies (bm_pack_weights), once.
        tau / gamma / rho / beta: TAE gate, margin gate, replacement budget, distribution gate (None = off).
        eta, q: token-aware buddy priority with q [E][R] (numpy fp32) of the table entries."""
        import torch
        import paper_2511_10054_amd as bm
        self.bm = bm
        self.host = host
        s = host.spec
        flags = (bm.BM_RENORM_TOPK if renorm else 0) | (bm.BM_REMAP_UNIQUE if unique else 0) | (bm.BM_Y_F32 if y_f32 else 0)
        flags |= (bm.BM_GATE_TAE if tau is not None else 0) | (bm.BM_GATE_MARGIN if gamma is not None else 0)
        flags |= (bm.BM_REPLACE_BUDGET if rho is not None else 0) | (bm.BM_GATE_DIST if beta is not None else 0)
        flags |= bm.BM_PSI_TOKEN if eta is not None else 0
        self.desc = bm.LayerDesc(T=host.T, d=s.d, E=s.E, F=s.F, K=s.K, n_shared=s.n_shared, R=s.R,
                                 H=s.H if H is None else H,
                                 dtype=bm.BM_BF16 if s.dtype == "bf16" else bm.BM_F32, flags=flags,
                                 tae_tau=tau or 0.0, margin_gamma=gamma or 0.0, rho=rho or 0, dist_beta=beta or 0.0, psi_eta=eta or 0.0)
        self.x = to_device(host.x)
        self.w_router = to_device(host.w_router)
        self.bias = to_device(host.bias)
        if base is not None:
            self.wg, self.wu, self.wd, self.sg, self.su, self.sd = base.wg, base.wu, base.wd, base.sg, base.su, base.sd
        else:
            self.wg, self.wu, self.wd = to_device(host.wg), to_device(host.wu), to_device(host.wd)
            self.sg, self.su, self.sd = to_device(host.sg), to_device(host.su), to_device(host.sd)
        self.bitmap = to_device(host.bitmap)
        self.table = to_device(host.table)
        from paper_2511_10054_amd.binding import make_weights
        self.packed = None
        if base is not None and base.packed is not None:
            self.packed = base.packed
        elif pack and s.dtype == "bf16":
            self.packed = [torch.empty(max(bm.bm_packed_bytes(self.desc, i), 16), dtype=torch.uint8, device="cuda")
                           if (i < 2 or s.n_shared) else None for i in range(4)]
        pk = self.packed or [None] * 4
        self.q = to_device(np.ascontiguousarray(q, dtype=np.float32)) if q is not None else None
        self.weights = make_weights(self.w_router, self.bias, self.wg, self.wu, self.wd, self.sg, self.su, self.sd, *pk,
                                    buddy_q=self.q)
        if self.packed is not None and not (base is not None and base.packed is not None):
            bm.bm_pack_weights(self.desc, self.weights, self.bitmap)      # only resident experts are read
            torch.cuda.synchronize()
        nbytes = bm.bm_workspace_bytes(self.desc)
        self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        self.y_dtype = torch.float32 if (y_f32 or s.dtype == "f32") else torch.bfloat16
        self.y = torch.empty((host.T, s.d), dtype=self.y_dtype, device="cuda")

    def forward(self, debug=True):
        import torch
        T, K, E = self.host.T, self.host.spec.K, self.host.spec.E
        dbg = None
        if debug:
            i32 = dict(dtype=torch.int32, device="cuda")
            dbg = dict(ids=torch.full((T, K), -7, **i32), ids_remapped=torch.full((T, K), -7, **i32),
                       w=torch.full((T, K), -7.0, dtype=torch.float32, device="cuda"),
                       offsets=torch.full((E + 1,), -7, **i32), perm=torch.full((T * K,), -7, **i32),
                       inv_perm=torch.full((T * K,), -7, **i32), stats=torch.full((6,), -7, **i32))
        self.bm.bm_moe_forward(self.desc, self.x, self.weights, self.bitmap, self.table, self.y, self.workspace, dbg)
        torch.cuda.synchronize()
        out = dict(y=self.y.float().cpu().numpy())
        if debug:
            out.update({k: v.cpu().numpy() for k, v in dbg.items()})
        return out
