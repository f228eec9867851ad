"""The C-ABI library: loads without a GPU, exports every declared symbol, and
rejects bad arguments on the host before anything is launched (CPU only)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2511_10054_amd as bm
from paper_2511_10054_amd.binding import DebugOut, Weights

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _desc(**kw):
    base = dict(T=16, d=64, E=8, F=128, K=2, n_shared=0, R=3, H=3, dtype=bm.BM_F32, flags=bm.BM_RENORM_TOPK)
    base.update(kw)
    return bm.LayerDesc(**base)


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    assert sorted(os.listdir(inc)) == ["buddymoe.h", "buddymoe_bench.h"]
    header = "".join(open(os.path.join(inc, f)).read() for f in os.listdir(inc))
    names = set(re.findall(r"\b(bm_[a-z_]+)\s*\(", header))
    assert "bm_stream_read" not in open(os.path.join(inc, "buddymoe.h")).read()      # a bench aid, not the layer's ABI
    assert {"bm_route_topk", "bm_buddy_remap", "bm_permute_by_expert", "bm_moe_forward",
            "bm_workspace_bytes", "bm_validate_tables", "bm_strerror", "bm_coactivation_accumulate",
            "bm_build_buddy_table", "bm_moe_forward_static"} <= names
    lib = bm.load_library()
    for n in names:
        assert hasattr(lib, n), n


def test_struct_layouts_match_header(tmp_path):
    # sizes and member offsets as the C compiler sees the header, against the ctypes mirrors
    import subprocess
    hdr = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    members = {"bm_layer_desc": [f[0] for f in bm.LayerDesc._fields_],
               "bm_weights": [f[0] for f in Weights._fields_],
               "bm_debug_out": [f[0] for f in DebugOut._fields_]}
    lines = []
    for st, names in members.items():
        lines.append(f'printf("{st} %zu\\n", sizeof({st}));')
        lines += [f'printf("{st}.{m} %zu\\n", offsetof({st}, {m}));' for m in names]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "buddymoe.h"\nint main(void){'
                   + "".join(lines) + "return 0;}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", hdr, "-o", str(exe), str(src)], check=True)
    got = dict(l.split() for l in subprocess.run([str(exe)], check=True, capture_output=True,
                                                 text=True).stdout.splitlines())
    for st, cls in (("bm_layer_desc", bm.LayerDesc), ("bm_weights", Weights), ("bm_debug_out", DebugOut)):
        assert int(got[st]) == ctypes.sizeof(cls)
        for m in members[st]:
            assert int(got[f"{st}.{m}"]) == getattr(cls, m).offset, (st, m)


def test_strerror_and_workspace_bytes():
    assert bm.bm_strerror(0) == "ok"
    for s in range(-6, 0):
        assert bm.bm_strerror(s) not in ("ok", "unknown status")
    assert bm.bm_strerror(-99) == "unknown status"
    small = bm.bm_workspace_bytes(_desc())
    big = bm.bm_workspace_bytes(_desc(T=4096))
    assert 0 < small < big and small % 256 == 0
    assert bm.bm_workspace_bytes(_desc(K=9)) == 0          # K > E
    # grouping only (d = F = 0): a function of T, E, K - per-tile histograms, no activations
    g = bm.bm_workspace_bytes(_desc(T=4096, d=0, F=0))
    assert 0 < g < 64 * 1024 and g % 256 == 0 and g == bm.bm_workspace_bytes(_desc(T=4096, d=0, F=0, dtype=7, R=99))
    assert bm.bm_workspace_bytes(_desc(T=4096, d=0, F=0, K=9)) == 0
    assert bm.bm_workspace_bytes(_desc(dtype=7)) == 0
    # DeepSeek-shaped layer: h and o for 8192*6 + 2*8192 rows
    n = bm.bm_workspace_bytes(_desc(T=8192, d=2048, E=64, F=1408, K=6, n_shared=2, R=8, H=8, dtype=bm.BM_BF16))
    rows = 8192 * 8
    assert n >= rows * (1408 + 2048) * 2


def test_packed_bytes_and_pack_argument_errors():
    lib = bm.load_library()
    d = _desc(T=8, d=4096, E=8, F=14336, K=2, R=7, H=7, dtype=bm.BM_BF16, n_shared=1)
    one = 14336 * 4096 * 2
    assert bm.bm_packed_bytes(d, 0) == 8 * 2 * one and bm.bm_packed_bytes(d, 1) == 8 * one
    assert bm.bm_packed_bytes(d, 2) == 2 * one and bm.bm_packed_bytes(d, 3) == one
    assert bm.bm_packed_bytes(d, 4) == 0 and bm.bm_packed_bytes(_desc(), 0) == 0      # fp32 layers are not packed
    w = Weights(*([256] * 8 + [0] * 5))
    assert lib.bm_pack_weights(ctypes.byref(_desc()), ctypes.byref(w), None, None) == -3   # dtype
    assert lib.bm_pack_weights(ctypes.byref(d), None, None, None) == -1
    assert lib.bm_pack_weights(ctypes.byref(d), ctypes.byref(w), None, None) == 0          # nothing to fill
    w3 = Weights(256, 0, 0, 256, 256, 0, 0, 0, 256, 0, 0, 0)
    assert lib.bm_pack_weights(ctypes.byref(d), ctypes.byref(w3), None, None) == -1        # source missing


def test_validate_tables():
    d = _desc(E=4, R=3, H=3)
    bitmap = np.array([0b0101], np.uint64)
    table = np.array([[1, 2, 3], [0, 2, -1], [3, -1, -1], [0, 1, 2]], np.int32)
    assert bm.bm_validate_tables(d, bitmap, table) == 0
    bad = table.copy(); bad[2, 1] = 2                       # an expert listed as its own buddy
    assert bm.bm_validate_tables(d, bitmap, bad) == -5
    bad = table.copy(); bad[0, 0] = 4                       # out of range
    assert bm.bm_validate_tables(d, bitmap, bad) == -5
    bad = table.copy(); bad[0, 0] = -2
    assert bm.bm_validate_tables(d, bitmap, bad) == -5
    assert bm.bm_validate_tables(d, np.array([0b10000], np.uint64), table) == -5   # bit past E
    assert bm.bm_validate_tables(_desc(E=4, R=3, H=4), bitmap, table) == -2        # H > R


def test_host_side_argument_errors_launch_nothing():
    """Every call below must return its error from the host checks (no GPU here)."""
    lib = bm.load_library()
    one = ctypes.c_void_p(256)        # non-null dummy, never dereferenced on these paths
    d = _desc()
    assert lib.bm_route_topk(None, one, one, None, one, one, None) == -1
    assert lib.bm_route_topk(ctypes.byref(d), None, one, None, one, one, None) == -1
    assert lib.bm_route_topk(ctypes.byref(_desc(K=9)), one, one, None, one, one, None) == -2
    assert lib.bm_route_topk(ctypes.byref(_desc(E=257)), one, one, None, one, one, None) == -2
    assert lib.bm_route_topk(ctypes.byref(_desc(dtype=3)), one, one, None, one, one, None) == -3
    assert lib.bm_route_topk(ctypes.byref(_desc(dtype=bm.BM_BF16, d=72)), one, one, None, one, one, None) == -2
    assert lib.bm_route_topk(ctypes.byref(_desc(T=0)), None, None, None, None, None, None) == 0   # empty batch
    assert lib.bm_buddy_remap(ctypes.byref(_desc(H=4)), one, one, one, one, None, None, None) == -2
    assert lib.bm_buddy_remap(ctypes.byref(d), None, one, one, one, None, None, None) == -1
    assert lib.bm_buddy_remap(ctypes.byref(_desc(R=33, H=1)), one, one, one, one, None, None, None) == -2
    gated = _desc(flags=bm.BM_GATE_TAE, tae_tau=0.5)
    assert lib.bm_buddy_remap(ctypes.byref(gated), one, one, one, one, None, None, None) == -1   # gates read w
    assert lib.bm_buddy_remap(ctypes.byref(_desc(flags=bm.BM_REPLACE_BUDGET, rho=-1)), one, one, one, one, one,
                              None, None) == -2
    assert lib.bm_buddy_remap(ctypes.byref(_desc(flags=bm.BM_GATE_MARGIN, margin_gamma=float("nan"))), one, one,
                              one, one, one, None, None) == -2
    assert lib.bm_coactivation_accumulate(ctypes.byref(d), one, None, one, None) == -1
    assert lib.bm_coactivation_accumulate(ctypes.byref(_desc(E=300)), one, one, one, None) == -2
    lib.bm_build_buddy_table.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float] + [ctypes.c_void_p] * 4
    assert lib.bm_build_buddy_table(ctypes.byref(d), one, 0.0, one, None, None, None) == -2      # alpha in (0, 1]
    assert lib.bm_build_buddy_table(ctypes.byref(d), one, 1.5, one, None, None, None) == -2
    assert lib.bm_build_buddy_table(ctypes.byref(d), None, 0.5, one, None, None, None) == -1
    assert lib.bm_build_buddy_table(ctypes.byref(_desc(R=0, H=0)), one, 0.5, one, None, None, None) == -2
    assert lib.bm_permute_by_expert(ctypes.byref(d), one, one, one, one, None, 1 << 20, None) == -4
    assert lib.bm_permute_by_expert(ctypes.byref(d), one, one, one, one, one, 16, None) == -4
    assert lib.bm_permute_by_expert(ctypes.byref(d), one, one, one, one, ctypes.c_void_p(264), 1 << 20, None) == -4
    w = Weights(*([256] * 8 + [0] * 5))
    assert lib.bm_moe_forward(ctypes.byref(d), one, ctypes.byref(w), one, one, one, one, 16, None, None) == -4
    assert lib.bm_moe_forward(ctypes.byref(d), one, None, one, one, one, one, 1 << 30, None, None) == -1
    assert lib.bm_moe_forward(ctypes.byref(_desc(n_shared=9)), one, ctypes.byref(w), one, one, one, one, 1 << 30, None, None) == -2
    assert lib.bm_moe_forward(ctypes.byref(_desc(T=0)), None, None, None, None, None, None, 0, None, None) == 0
    # the entry point on the built-in scratch array: same checks, and a layer whose scratch does not fit
    assert lib.bm_moe_forward_static(ctypes.byref(d), one, None, one, one, one, None, None) == -1
    assert lib.bm_moe_forward_static(ctypes.byref(_desc(n_shared=9)), one, ctypes.byref(w), one, one, one, None, None) == -2
    assert lib.bm_moe_forward_static(ctypes.byref(_desc(T=0)), None, None, None, None, None, None, None) == 0
    big = _desc(T=4096, d=4096, E=8, F=14336, K=2, R=7, H=7, dtype=bm.BM_BF16)
    assert bm.bm_workspace_bytes(big) > bm.BM_STATIC_WORKSPACE_BYTES
    assert lib.bm_moe_forward_static(ctypes.byref(big), one, ctypes.byref(w), one, one, one, None, None) == -4
    psi = _desc(flags=bm.BM_PSI_TOKEN, psi_eta=1.0)
    assert lib.bm_moe_forward(ctypes.byref(psi), one, ctypes.byref(w), one, one, one, one, 1 << 30, None, None) == -1  # no q
    assert lib.bm_buddy_remap(ctypes.byref(psi), one, one, one, one, one, None, None) == -2
    w2 = Weights(256, 0, 256, 256, 256, 0, 0, 0, 0, 0, 0, 0, 0)
    assert lib.bm_moe_forward(ctypes.byref(_desc(n_shared=1)), one, ctypes.byref(w2), one, one, one, one, 1 << 30, None, None) == -1


def test_product_package_does_not_import_the_oracle():
    import subprocess, sys
    code = ("import sys; sys.path.insert(0, %r); import paper_2511_10054_amd; "
            "assert 'oracle' not in sys.modules and 'workloads' not in sys.modules") % ROOT
    subprocess.run([sys.executable, "-c", code], check=True)
    for root, _, files in os.walk(os.path.join(ROOT, "paper_2511_10054_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(root, f)).read()
                assert "oracle" not in text.lower() or f == "README.md", f


def test_stream_read_rejects_bad_arguments_on_the_host():
    lib = bm.load_library()
    lib.bm_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    one = ctypes.c_void_p(16)
    assert lib.bm_stream_read(None, 1024, one, None) == -1
    assert lib.bm_stream_read(one, 1024, None, None) == -1
    assert lib.bm_stream_read(one, 1000, one, None) == -2          # not a multiple of 16 bytes


def test_persistent_schedule_is_taken_only_on_the_full_part(tmp_path):
    """The device-shape rule of the persistent prefill kernel (csrc/bm_device_shape.h, plain C++): exactly
    256 compute units in 8 XCDs; a partitioned or different device, or a failed query (0), takes the
    fallback kernels."""
    import subprocess
    src = tmp_path / "shape.cpp"
    src.write_text('#include "bm_device_shape.h"\n#include <cstdio>\nint main() {\n'
                   '  using bm::persistent_schedule_fits;\n'
                   '  int bad = 0;\n'
                   '  bad += !persistent_schedule_fits(256, 8);\n'
                   '  bad += persistent_schedule_fits(0, 0) + persistent_schedule_fits(256, 0) + persistent_schedule_fits(0, 8);\n'
                   '  bad += persistent_schedule_fits(128, 4) + persistent_schedule_fits(64, 2) + persistent_schedule_fits(32, 1);\n'
                   '  bad += persistent_schedule_fits(304, 8) + persistent_schedule_fits(256, 4) + persistent_schedule_fits(255, 8);\n'
                   '  std::printf("%d\\n", bad);\n  return bad;\n}\n')
    exe = tmp_path / "shape"
    subprocess.run(["g++", "-std=c++17", "-I", os.path.join(ROOT, "paper_2511_10054_amd", "csrc"), "-o", str(exe), str(src)],
                   check=True)
    assert subprocess.run([str(exe)], capture_output=True, text=True).stdout.strip() == "0"


def test_small_tile_dealer_hands_out_every_tile_exactly_once(tmp_path):
    """The dealing of 128-row tiles among an XCD's workgroups (csrc/bm_tile_dealer.h, plain C++): for every
    number of 256-row tiles, 128-row tiles and workgroups in a range, each tile goes to exactly one workgroup,
    a workgroup's tiles come in increasing order, and no workgroup ends more than one 256-row tile's worth
    above the lightest one."""
    import subprocess
    src = tmp_path / "dealer.cpp"
    src.write_text(r'''
#include "bm_tile_dealer.h"
#include <cstdio>
#include <vector>
int main() {
    long checked = 0;
    for (int stride = 1; stride <= 32; ++stride)
        for (int n_big = 0; n_big <= 70; ++n_big)
            for (int n_small = 0; n_small <= 90; ++n_small) {
                std::vector<int> owner(n_small, -1), load(stride);
                for (int slot = 0; slot < stride; ++slot) {
                    bm::SmallTileDealer d;
                    d.init(n_big, n_small, stride, slot);
                    load[slot] = 20 * (n_big / stride + (slot < n_big % stride ? 1 : 0));
                    int tile = -1, last = -1, guard = 0;
                    while (d.next(tile)) {
                        if (tile < 0 || tile >= n_small || owner[tile] != -1 || tile <= last || ++guard > n_small) {
                            std::printf("bad deal stride %d big %d small %d slot %d tile %d\n", stride, n_big, n_small, slot, tile);
                            return 1;
                        }
                        owner[tile] = slot; last = tile; load[slot] += 13;
                    }
                }
                int lo = 1 << 30, hi = 0;
                for (int t = 0; t < n_small; ++t) if (owner[t] < 0) { std::printf("tile %d not dealt (%d %d %d)\n", t, stride, n_big, n_small); return 1; }
                for (int v : load) { lo = v < lo ? v : lo; hi = v > hi ? v : hi; }
                if (hi - lo > 20) { std::printf("unbalanced %d..%d (%d %d %d)\n", lo, hi, stride, n_big, n_small); return 1; }
                ++checked;
            }
    std::printf("ok %ld\n", checked);
    return 0;
}
''')
    exe = tmp_path / "dealer"
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "paper_2511_10054_amd", "csrc"), "-o", str(exe), str(src)],
                   check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout


def test_prefill_kernels_keep_the_hand_managed_register_to_themselves(tmp_path):
    """The persistent prefill kernels park the pending result of one vector load in v255, a register the
    compiler does not manage (csrc/bm_gemm_bf16.hip, BM_LOOKUP / BM_ADOPT): the compiler's own values must
    stay below it, and it may appear in the hand-written statements only.  The same kernels must not spill:
    a reload from scratch memory waits for every load and store in flight.  Checked on the assembly the
    build's compiler emits for the build's flags (own code, device side only)."""
    import re
    import subprocess
    from paper_2511_10054_amd import build
    out = tmp_path / "gemm.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.run([build.HIPCC, *flags, "-S", "--cuda-device-only", "-o", str(out),
                    os.path.join(build.CSRC, "bm_gemm_bf16.hip")], check=True, capture_output=True)
    text = out.read_text()
    kernels = re.findall(r"^(_ZN2bm\w*k64w\w*):[^\n]*\n(.*?)\.end_amdhsa_kernel", text, flags=re.S | re.M)
    assert len(kernels) >= 3, [k for k, _ in kernels]
    allowed = (r"global_load_dword v255, v\d+, s\[\d+:\d+\]", r"v_mov_b32 v255, v\d+", r"v_mov_b32 v\d+, v255")
    for name, body in kernels:
        assert "scratch_" not in body, name + " spills vector registers"
        assert "global_load_dword v255" in body and "v255" in body, name
        for line in body.split("\n"):
            code = line.split(";")[0].strip()
            if re.search(r"\bv255\b|v\[\d+:255\]", code):
                assert any(re.fullmatch(a, code) for a in allowed), (name, code)
        used = [int(m) for m in re.findall(r"\bv(\d+)\b", body)] + [int(m) for m in re.findall(r"\bv\[\d+:(\d+)\]", body)]
        assert max(u for u in used if u != 255) < 240, name
        # every MFMA sits in the k-step loop (depth 2 inside the tile loop): were the first k-step ever peeled
        # into straight-line code, the compiler would sink the accumulator zeroing to right in front of the
        # hand-written MFMA statements, inside their wait-state window
        depth, n_mfma = 0, 0
        for line in body.split("\n"):
            if re.match(r"^(\.LBB\S+:|; %bb\.\d+:)", line):          # a block: "... in Loop: Header=BBn_m Depth=N"
                m = re.search(r"in Loop: Header=\S+ Depth=(\d+)", line)
                depth = int(m.group(1)) if m else 0
            elif re.match(r"^\s*;.*Loop Header: Depth=(\d+)", line):   # ... or a loop header, its depth on the next line
                depth = int(re.search(r"Loop Header: Depth=(\d+)", line).group(1))
            elif "v_mfma" in line:
                n_mfma += 1
                assert depth >= 2, (name, "MFMA outside the k-step loop")
        assert n_mfma >= 128, name
