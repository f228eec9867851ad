#!/usr/bin/env python3
"""Throughput of one MoE layer's forward pass with buddy-expert substitution on one MI355X.

A step is one bm_moe_forward over one batch of synthetic tokens (router ->
gates -> substitution -> grouping -> SwiGLU experts -> aggregation) with all
inputs resident in HBM.  Prints ONE JSON line: tokens/s from K timed calls, the
roofline of the dominant kernel (gate/up projection; its duration comes from
HIP events the library records on the launch stream between the stages, in a
second pass of K calls - an event record costs the GPU about 3 us, so the
events stay out of the pass that gives tokens/s) and the CPU oracle timed on a
bounded sample of the same workload.  Before the W warm-up steps the layer
runs untimed for 150 ms, which is what the chip's clocks need to settle after
the idle time of input generation.

With no --workload the line carries the whole metric: the headline is the decode layer
(c2_mixtral_decode, 64 tokens, public weight layout), "also" holds its other batch sizes,
"packed_weights" the same layer on the optional fragment-major copies, and "also_workloads" the three
prefill-sized layers (c3, c4, c5), each with its own roofline fractions, stage times and oracle check.

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
SETTLE_MS = 150.0            # untimed run of the layer before the warm-up steps (clock settling)

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_of_the_gate_up_kernel.md")


def profiled_traffic(workload, layout, remap):
    """HBM bytes per launch of the gate/up kernel as the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised
    under profiles/ measured them (a table row per workload, weight layout and substitution mode; the
    counters cannot be read from inside this process).  Returns (bytes or None, where it came from / why
    there is none)."""
    try:
        lines = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None, "no traffic table under profiles/"
    for ln in lines:
        c = [v.strip() for v in ln.strip().strip("|").split("|")]
        if len(c) >= 6 and c[0] == workload and c[1] == layout and c[2] == remap:
            return (float(c[3]) + float(c[4])) * 1e6, f"profiles/{os.path.basename(TRAFFIC_TABLE)}: {c[5]}"
    return None, f"no rocprofv3 counter run recorded for {workload} / {layout} / {remap}"


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
    perm = torch.zeros(T * K, **i32)
    hipev = HipEvents()
    events = [hipev.create(5) for _ in range(steps)] if with_events else None

    def step(dbg):
        bm.bm_moe_forward(dev.desc, dev.x, dev.weights, dev.bitmap, dev.table, dev.y, dev.workspace, dbg)

    # Clocks: after idling (input generation, uploads) the chip needs some tens of milliseconds under load
    # before its clocks settle - the first 20 calls after a cold start run 3-10 % slower than every later
    # pass - so the layer is run for SETTLE_MS first; then the W warm-up steps, then the K timed ones.
    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < SETTLE_MS:
        for _ in range(10):
            step(None)
        torch.cuda.synchronize()
    for _ in range(max(warmup, 1)):                     # warm-up also fetches the grouping for the report
        step(dict(offsets=offsets, stats=stats, ids_remapped=ids2, perm=perm))
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
    return dict(spec=spec, host=host, dev=dev, T=T, unique=unique, ms_per_step=ms_per_step, stage_ms=stage_ms,
                ms_per_step_ev=ms_per_step_ev, step_pct=step_pct,
                a_live=a_live, n_touched=n_touched, rows=rows, groups=groups, offsets=off,
                perm=perm.cpu().numpy(), stats=stats.cpu().tolist(), gen_s=t_gen)


RIDGE = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)     # 312.5 flop per byte


def _roof(bytes_, flops, t):
    """Fractions of both roofs; the binding one is the roof the algorithmic intensity falls under."""
    gbs, tfs = bytes_ / t / 1e9, flops / t / 1e12
    both = dict(hbm_frac=round(gbs / PEAK_HBM_GBS, 4), mfma_frac=round(tfs / PEAK_BF16_TFLOPS, 4),
                algorithmic_bytes=int(bytes_), algorithmic_flops=int(flops),
                flop_per_byte=round(flops / bytes_, 1))
    if flops / bytes_ < RIDGE:
        return dict(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(gbs / PEAK_HBM_GBS, 4), **both)
    return dict(bound="mfma", achieved=round(tfs, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                frac=round(tfs / PEAK_BF16_TFLOPS, 4), **both)


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
    out = _roof(bytes_, flops, t)
    out.update(traffic=None, kernel="grouped gate/up projection", kernel_us=round(t * 1e6, 2))
    return out


def roofline_layer(r):
    """The whole layer against the same two roofs: every touched group's three weight matrices once,
    router weights, x in and y out (bytes); 6*d*F flops per row."""
    s = r["spec"]
    bytes_ = r["groups"] * 3 * s.d * s.F * 2 + s.E * s.d * 2 + 2 * r["T"] * s.d * 2
    flops = 6.0 * s.d * s.F * r["rows"]
    return _roof(bytes_, flops, r["ms_per_step"] * 1e-3)


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
    host = r["host"]
    n = min(r["T"], budget_tokens)
    rows = np.arange(n)
    oracle.lib()                                   # build / load outside the timed region
    t0 = time.perf_counter()
    host.oracle_forward(oracle, rows=rows, unique=r["unique"])
    dt = time.perf_counter() - t0
    return dict(value=round(n / dt, 3), unit="tokens/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"first {n} of {r['T']} tokens, whole layer, {dt:.1f} s (includes widening bf16 inputs to fp32)")


def check_against_oracle(r, cap):
    """Layer output against the oracle on the tokens whose rows sit at group and tile edges (the first and last
    row of every expert group, a row from each 128-row half of every 256-row tile), at most about `cap`."""
    import oracle
    from workloads.harness import edge_tokens, err_metric, err_unfloored
    host, dev, s = r["host"], r["dev"], r["spec"]
    rows = edge_tokens(r["offsets"], r["perm"], s.K, cap=cap, seed=r["T"])
    if r["T"] <= cap:
        rows = np.arange(r["T"])
    ref = host.oracle_forward(oracle, rows=rows, unique=r["unique"])
    y = dev.y.float().cpu().numpy()[rows]
    return {"err_vs_oracle_on_sample": float(f"{err_metric(y, ref['y']):.3e}"), "tolerance": 2e-2,
            "err_unfloored_elementwise": float(f"{err_unfloored(y, ref['y']):.3e}"),
            "sample": f"{len(rows)} of {r['T']} tokens: " + ("all" if r["T"] <= cap else
                      "first and last row of every expert group, one row per 128-row half of every row tile")}


def stages(r):
    return {k: round(float(v) * 1e3, 2) for k, v in
            zip(("front_and_grouping", "gate_up", "down", "combine"), r["stage_ms"])}


def config_of(r, name, pack):
    s = r["spec"]
    return {"workload": f"{name}_T{r['T']}", "T": r["T"], "d": s.d, "E": s.E, "F": s.F,
            "K": s.K, "n_shared": s.n_shared, "resident": s.n_resident,
            "remap": "unique" if r["unique"] else "first_resident",
            "weights": "fragment-major copy made once by bm_pack_weights (untimed)" if pack else "public layout",
            "a_live": r["a_live"], "experts_touched": r["n_touched"],
            "n_miss": r["stats"][0], "n_substituted": r["stats"][1], "n_dropped": r["stats"][2]}


def with_traffic(roof, r, name, pack):
    roof["traffic"], roof["traffic_source"] = profiled_traffic(
        f"{name}_T{r['T']}", "packed" if pack else "public", "unique" if r["unique"] else "first_resident")
    return roof


def brief(r, name, pack, check_cap=None):
    """One workload as an entry of the JSON line's side tables."""
    roof = with_traffic(roofline_gateup(r), r, name, pack)
    out = {"tokens_per_s": round(r["T"] / (r["ms_per_step"] * 1e-3), 1), "ms_per_step": round(r["ms_per_step"], 5),
           "experts_touched": r["n_touched"], "a_live": r["a_live"],
           "roofline": roof, "layer_roofline": roofline_layer(r), "stages_us": stages(r)}
    if check_cap:
        out["check"] = check_against_oracle(r, check_cap)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=None, choices=sorted(WORKLOADS),
                    help="one workload only (default: c2 as the headline plus c3, c4, c5 under 'also_workloads')")
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unique", action="store_true", help="Algorithm 1's uniqueness test on")
    ap.add_argument("--pack", action="store_true",
                    help="decode workload: stream the optional fragment-major weight copies (bm_pack_weights) "
                         "instead of the public layout")
    ap.add_argument("--also-workloads", default=None,
                    help="comma-separated further workloads reported under 'also_workloads' (\"\" for none)")
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

    default_line = args.workload is None and not args.tokens
    wl = args.workload or "c2"
    name, T = WORKLOADS[wl]
    if args.tokens:
        T = args.tokens
    # decode: the public layout is the headline (the method's premise is a GPU short of memory; the
    # fragment-major copy of the resident experts is optional and reported beside it)
    pack = args.pack
    r = run_workload(name, T, args.steps, args.warmup, unique=args.unique, pack=pack)
    roof = with_traffic(roofline_gateup(r), r, name, pack)
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
        "config": config_of(r, name, pack),
        "roofline": roof,
        "layer_roofline": roofline_layer(r),
        "stages_us": stages(r),
        "ms_per_step_with_stage_events": round(r["ms_per_step_ev"], 5),
        "step_ms_p10_p50_p90_with_stage_events": [round(v, 5) for v in r["step_pct"]],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(r, 64 if wl == "c2" else 256)
        out["check"] = check_against_oracle(r, 64 if wl in ("c2", "c3") else 256)
    else:
        out["cpu_baseline"] = None
    also = args.also_tokens
    if also is None and wl == "c2" and not args.tokens:
        also = "1,8,32"                                   # the other batch sizes the decode config names
    if also:
        out["also"] = {}
        for t2 in [int(v) for v in also.split(",") if v]:
            r2 = run_workload(name, t2, args.steps, args.warmup, unique=args.unique, base=r, pack=pack)
            e = brief(r2, name, pack)
            out["also"][f"T{t2}"] = {"tokens_per_s": e["tokens_per_s"], "ms_per_step": e["ms_per_step"],
                                     "experts_touched": e["experts_touched"],
                                     "gate_up_frac": e["roofline"]["frac"], "gate_up_bound": e["roofline"]["bound"],
                                     "layer_frac": e["layer_roofline"]["frac"], "stages_us": e["stages_us"]}
    if default_line and not pack:
        # the same decode layer on the optional fragment-major weight copies
        rp = run_workload(name, T, args.steps, args.warmup, unique=args.unique, base=r, pack=True)
        e = brief(rp, name, True)
        out["packed_weights"] = {"note": "same layer and batch on the copies written once by bm_pack_weights "
                                         "(costs the resident experts' memory a second time); not the headline",
                                 "tokens_per_s": e["tokens_per_s"], "ms_per_step": e["ms_per_step"],
                                 "gate_up_frac": e["roofline"]["frac"], "layer_frac": e["layer_roofline"]["frac"],
                                 "stages_us": e["stages_us"]}
        del rp
    rs = read_stream_gbs()
    out["hbm_read_stream"] = {"achieved": round(rs, 1), "unit": "GB/s", "bytes": 1 << 31,
                              "note": "plain streaming read, the practical ceiling of an HBM-bound kernel on this device"}
    if out["layer_roofline"]["bound"] == "hbm":
        out["layer_roofline"]["frac_of_read_stream"] = round(out["layer_roofline"]["achieved"] / rs, 4)
    if roof["bound"] == "hbm":
        roof["frac_of_read_stream"] = round(roof["achieved"] / rs, 4)
    more = args.also_workloads
    if more is None:
        more = "c3,c4,c5" if default_line else ""
    if more:
        import gc
        import torch
        out["also_workloads"] = {}
        del r
        for w2 in [v for v in more.split(",") if v]:
            gc.collect()
            torch.cuda.empty_cache()
            n2, t2 = WORKLOADS[w2]
            r2 = run_workload(n2, t2, args.steps, args.warmup, unique=args.unique, pack=False)
            e = brief(r2, n2, False, check_cap=None if args.no_cpu_baseline else (64 if w2 == "c3" else 256))
            e["config"] = config_of(r2, n2, False)
            out["also_workloads"][w2] = e
            print(f"bench: {w2} done ({e['ms_per_step']} ms/step, generated in {r2['gen_s']:.0f} s)", file=sys.stderr, flush=True)
            del r2
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
