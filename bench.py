#!/usr/bin/env python3
"""Throughput of one MoE layer's forward pass with buddy-expert substitution on one MI355X.

A step is one bm_moe_forward over one batch of synthetic tokens (router ->
gates -> substitution -> grouping -> SwiGLU experts -> aggregation) with all
inputs resident in HBM.  Prints ONE JSON line: tokens/s from K timed calls, the
roofline of the dominant kernel (gate/up projection; its duration comes from
HIP events the library records on the launch stream between the stages, in a
second pass of K calls - an event record costs the GPU about 3 us, so the
events stay out of the pass that gives tokens/s) and the CPU oracle timed on a
bounded sample of the same workload.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5] [--tokens T]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA

# HBM bytes per launch of the gate/up kernel (read + write), from the rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs summarised under profiles/ (counter x copy-kernel calibration); default shapes,
# first-resident mode only.  Re-measure after changing that kernel.
TRAFFIC_BYTES = {
    "c2_mixtral_decode_T64": 1182.4e6,
    "c3_mixtral_prefill_T4096": 3979.2e6,
    "c4_qwen3_T2048": 591.8e6,
    "c5_deepseek_T8192": 1736.1e6,
}

WORKLOADS = {
    "c2": ("c2_mixtral_decode", 64),
    "c3": ("c3_mixtral_prefill", 4096),
    "c4": ("c4_qwen3", 2048),
    "c5": ("c5_deepseek", 8192),
}


class HipEvents:
    """hipEvent_t handles through libamdhip64 (timing plumbing only)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def create(self, n):
        out = []
        for _ in range(n):
            e = ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(e)) == 0
            out.append(e.value)
        return out

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, rc
        return ms.value

    def destroy(self, evs):
        for e in evs:
            self.hip.hipEventDestroy(ctypes.c_void_p(e))


def run_workload(name, T, steps, warmup, with_events=True, unique=False, base=None, pack=False):
    """base: result of an earlier run_workload on the same layer (weights are reused)."""
    import torch
    import workloads
    from workloads.harness import DeviceLayer, HostLayer
    spec = workloads.CONFIGS[name]
    t_gen = time.time()
    host = HostLayer(spec, T, only_resident=True, poison=True, base=base["host"] if base else None)
    dev = DeviceLayer(host, unique=unique, base=base["dev"] if base else None, pack=pack)
    t_gen = time.time() - t_gen
    bm = dev.bm
    E, K = spec.E, spec.K
    i32 = dict(dtype=torch.int32, device="cuda")
    offsets = torch.zeros(E + 1, **i32)
    stats = torch.zeros(6, **i32)
    ids2 = torch.zeros((T, K), **i32)
    hipev = HipEvents()
    events = [hipev.create(5) for _ in range(steps)] if with_events else None

    def step(dbg):
        bm.bm_moe_forward(dev.desc, dev.x, dev.weights, dev.bitmap, dev.table, dev.y, dev.workspace, dbg)

    for _ in range(max(warmup, 1)):                     # warm-up also fetches the grouping for the report
        step(dict(offsets=offsets, stats=stats, ids_remapped=ids2))
    torch.cuda.synchronize()
    # timed region: K calls of the layer and nothing else
    t0 = time.perf_counter()
    for i in range(steps):
        step(None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps

    # K more calls with HIP events recorded on the stream between the stages (per-kernel durations for
    # the roofline).  An event record costs the GPU about 3 us, five of them 5 % of a decode step, so
    # they stay out of the pass above.
    stage_ms = None
    ms_per_step_ev = None
    step_pct = None
    if events is not None:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(dict(stage_events=events[i]))
        torch.cuda.synchronize()
        ms_per_step_ev = (time.perf_counter() - t0) * 1e3 / steps
        acc = np.zeros(4)
        per_step = []
        for evs in events:
            for j in range(4):
                acc[j] += hipev.elapsed_ms(evs[j], evs[j + 1])
            per_step.append(hipev.elapsed_ms(evs[0], evs[4]))
        stage_ms = acc / steps
        step_pct = [float(np.percentile(per_step, q)) for q in (10, 50, 90)]
        for evs in events:
            hipev.destroy(evs)

    off = offsets.cpu().numpy()
    counts = np.diff(off)
    a_live = int(off[E])
    n_touched = int((counts > 0).sum())
    rows = a_live + spec.n_shared * T
    groups = n_touched + spec.n_shared
    return dict(spec=spec, host=host, dev=dev, T=T, ms_per_step=ms_per_step, stage_ms=stage_ms,
                ms_per_step_ev=ms_per_step_ev, step_pct=step_pct,
                a_live=a_live, n_touched=n_touched, rows=rows, groups=groups,
                stats=stats.cpu().tolist(), gen_s=t_gen)


def roofline_gateup(r):
    """Dominant kernel: the gate/up projection with the SwiGLU epilogue.

    Algorithmic bytes per launch: both weight matrices of every touched expert
    once (2*d*F*2 B each group), every row's input once (d*2 B) and its output
    once (F*2 B).  Algorithmic flops: 4*d*F per row.
    """
    s = r["spec"]
    bytes_ = r["groups"] * 2 * s.d * s.F * 2 + r["rows"] * (s.d + s.F) * 2
    flops = 4.0 * s.d * s.F * r["rows"]
    t = r["stage_ms"][1] * 1e-3
    # below ~312 flop/B per launch the kernel cannot leave the HBM roof
    if flops / bytes_ < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        ach = bytes_ / t / 1e9
        return dict(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(ach / PEAK_HBM_GBS, 4), traffic=None,
                    kernel="grouped gate/up projection", kernel_us=round(t * 1e6, 2),
                    algorithmic_bytes=int(bytes_))
    ach = flops / t / 1e12
    return dict(bound="mfma", achieved=round(ach, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                frac=round(ach / PEAK_BF16_TFLOPS, 4), traffic=None,
                kernel="grouped gate/up projection", kernel_us=round(t * 1e6, 2),
                algorithmic_flops=int(flops))


def roofline_layer(r):
    """The whole layer against the same two roofs: every touched group's three weight matrices once,
    router weights, x in and y out (bytes); 6*d*F flops per row."""
    s = r["spec"]
    bytes_ = r["groups"] * 3 * s.d * s.F * 2 + s.E * s.d * 2 + 2 * r["T"] * s.d * 2
    flops = 6.0 * s.d * s.F * r["rows"]
    t = r["ms_per_step"] * 1e-3
    if flops / bytes_ < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        ach = bytes_ / t / 1e9
        return dict(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(ach / PEAK_HBM_GBS, 4), algorithmic_bytes=int(bytes_))
    ach = flops / t / 1e12
    return dict(bound="mfma", achieved=round(ach, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                frac=round(ach / PEAK_BF16_TFLOPS, 4), algorithmic_flops=int(flops))


def read_stream_gbs():
    """Achievable HBM read rate: the library's plain streaming-read kernel over 2 GiB, timed with events."""
    import torch
    import paper_2511_10054_amd as bm
    buf = torch.empty(1 << 31, dtype=torch.uint8, device="cuda").random_(0, 255)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(3):
        bm.bm_stream_read(buf, sink)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    n = 10
    ev[0].record()
    for _ in range(n):
        bm.bm_stream_read(buf, sink)
    ev[1].record()
    torch.cuda.synchronize()
    return buf.numel() * n / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9


def cpu_baseline(r, budget_tokens):
    """The oracle as it stands, timed on the host cores on the first n tokens of the workload."""
    import oracle
    from workloads.harness import err_metric
    host, dev = r["host"], r["dev"]
    n = min(r["T"], budget_tokens)
    rows = np.arange(n)
    oracle.lib()                                   # build / load outside the timed region
    t0 = time.perf_counter()
    ref = host.oracle_forward(oracle, rows=rows)
    dt = time.perf_counter() - t0
    y = dev.y.float().cpu().numpy()[:n]
    err = err_metric(y, ref["y"])
    return dict(value=round(n / dt, 3), unit="tokens/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"first {n} of {r['T']} tokens, whole layer, {dt:.1f} s (includes widening bf16 inputs to fp32)",
                ), err


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=sorted(WORKLOADS))
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unique", action="store_true", help="Algorithm 1's uniqueness test on")
    ap.add_argument("--no-pack", action="store_true",
                    help="decode workload: stream the public weight layout instead of the packed copy")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run plain 1 GiB device copies and exit (reference for the HBM byte counters)")
    ap.add_argument("--also-tokens", default=None,
                    help="comma-separated extra batch sizes on the same layer, reported under 'also'")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (tokens shard "
              "data-parallel with no exchange step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs an MI355X", file=sys.stderr)
        sys.exit(1)
    if args.copy_calibration:
        # a copy kernel of known size: reads 2^30 bytes and writes 2^30 bytes per launch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 5}))
        return
    import paper_2511_10054_amd as bm
    bm.load_library()                                   # fails loudly if the HIP library is not built

    name, T = WORKLOADS[args.workload]
    if args.tokens:
        T = args.tokens
    pack = (args.workload == "c2") and not args.no_pack     # decode: weights repacked once at load time
    r = run_workload(name, T, args.steps, args.warmup, unique=args.unique, pack=pack)
    roof = roofline_gateup(r)
    if not args.unique:
        roof["traffic"] = TRAFFIC_BYTES.get(f"{name}_T{T}")
    out = {
        "metric": "moe_layer_tokens_per_s_with_buddy_remap",
        "value": round(T / (r["ms_per_step"] * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{name}_T{T}", "T": T, "d": r["spec"].d, "E": r["spec"].E, "F": r["spec"].F,
                   "K": r["spec"].K, "n_shared": r["spec"].n_shared, "resident": r["spec"].n_resident,
                   "remap": "unique" if args.unique else "first_resident",
                   "weights": "fragment-major copy made once by bm_pack_weights (untimed)" if pack else "public layout",
                   "a_live": r["a_live"], "experts_touched": r["n_touched"],
                   "n_miss": r["stats"][0], "n_substituted": r["stats"][1], "n_dropped": r["stats"][2]},
        "roofline": roof,
        "layer_roofline": roofline_layer(r),
        "stages_us": {k: round(float(v) * 1e3, 2) for k, v in
                      zip(("front_and_grouping", "gate_up", "down", "combine"), r["stage_ms"])},
        "ms_per_step_with_stage_events": round(r["ms_per_step_ev"], 5),
        "step_ms_p10_p50_p90_with_stage_events": [round(v, 5) for v in r["step_pct"]],
    }
    also = args.also_tokens
    if also is None and args.workload == "c2" and not args.tokens:
        also = "1,8,32"                                   # the other batch sizes the decode config names
    if also:
        out["also"] = {}
        for t2 in [int(v) for v in also.split(",") if v]:
            r2 = run_workload(name, t2, args.steps, args.warmup, unique=args.unique, base=r, pack=pack)
            roof2 = roofline_gateup(r2)
            out["also"][f"T{t2}"] = {"tokens_per_s": round(t2 / (r2["ms_per_step"] * 1e-3), 1),
                                     "ms_per_step": round(r2["ms_per_step"], 5),
                                     "experts_touched": r2["n_touched"],
                                     "gate_up_frac": roof2["frac"], "gate_up_bound": roof2["bound"],
                                     "layer_frac": roofline_layer(r2)["frac"],
                                     "stages_us": {k: round(float(v) * 1e3, 2) for k, v in
                                                   zip(("front_and_grouping", "gate_up", "down", "combine"), r2["stage_ms"])}}
    rs = read_stream_gbs()
    out["hbm_read_stream"] = {"achieved": round(rs, 1), "unit": "GB/s", "bytes": 1 << 31,
                              "note": "bm_stream_read, the practical ceiling of an HBM-bound kernel on this device"}
    if out["layer_roofline"]["bound"] == "hbm":
        out["layer_roofline"]["frac_of_read_stream"] = round(out["layer_roofline"]["achieved"] / rs, 4)
    if roof["bound"] == "hbm":
        roof["frac_of_read_stream"] = round(roof["achieved"] / rs, 4)
    if not args.no_cpu_baseline:
        base, err = cpu_baseline(r, 64 if args.workload == "c2" else 256)
        out["cpu_baseline"] = base
        out["check"] = {"err_vs_oracle_on_sample": float(f"{err:.3e}"), "tolerance": 2e-2}
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
