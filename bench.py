#!/usr/bin/env python3
"""Benchmark of libtaq on one MI355X: TAQ cross-attention query-tokens/s at the SD1.5
4096-query shape (batch 2, C=320, 8 heads, context 77x768, 1 fp16 trigger row, int8 K/V,
8-bit probabilities, W8A8 to_q/to_out), synthetic inputs.

A step is one taq_cross_attn call (all per-step rows of the block: hidden-state
quantization, to_q, Q~, scores, softmax, Eq. (3), A^ V~, output quantization, to_out).
taq_quantize_kv runs once per prompt, outside the denoising loop; its latency is
reported separately (`quantize_kv_us`) and as `value_with_quantize_kv_every_step`.

Prints ONE JSON line. Inputs are resident in HBM before timing starts; every step reads
and writes a different (hidden, out) pair of a ring whose touched bytes (hidden + out
only; the workspace, which this shape's single kernel never touches, is shared and not
counted) exceed 512 MB, twice the 256 MB last-level cache, so the figure is not a
cache-resident one (that one is reported as `value_cache_resident`). Before the warm-up
steps an untimed stretch of launches (`prewarm_ms`) brings the clocks up, so that a short
run (--steps 20) also reads the steady state.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

from paper_2603_22943_amd import synth
from paper_2603_22943_amd import taq as T

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0  # dense int8 MFMA, published


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=4096)   # 4096 steps of ~16 us: the timed region lasts ~65 ms
    p.add_argument("--warmup", type=int, default=256)  # enough for the clocks to settle
    p.add_argument("--ring", type=int, default=52,
                   help="distinct (hidden, out) pairs cycled through: 52 x 10.5 MB = 545 MB at the headline shape")
    p.add_argument("--prewarm-ms", type=float, default=60.0, help="untimed launches before the warm-up steps")
    p.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--cpu-seconds", type=float, default=8.0,
                   help="lower bound of oracle time to spend per leg (all threads, one thread)")
    p.add_argument("--profile-only", action="store_true",
                   help="run only warmup + timed steps (for rocprofv3), skip the side measurements")
    p.add_argument("--profile-config3", action="store_true",
                   help="run only the 16-layer UNet step of configs[2] (for rocprofv3)")
    p.add_argument("--traffic-probe", action="store_true",
                   help="for `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE`: a device copy of known size, then eager steps")
    p.add_argument("--summarize-sq", nargs="+", metavar="CSV",
                   help="rocprofv3 --pmc SQ_* counter CSVs of --profile-only runs -> profiles/fused_block_kernel_cfg2_pmc.json")
    p.add_argument("--profile-gemm", action="store_true",
                   help="run only the int8 GEMM of the kernel-per-stage path (to_q at M=2048 C=1280 and M=8192 C=320; for rocprofv3)")
    p.add_argument("--summarize-trace", nargs="+", metavar=("STATS_CSV", "OUT_TXT"),
                   help="STATS_CSV OUT_TXT COMMAND [NOTE...]: the taq:: rows of a rocprofv3 --kernel-trace --stats "
                        "kernel_stats.csv -> profiles/OUT_TXT, with the command and notes as its header")
    p.add_argument("--summarize-sq-by-kernel", nargs="+", metavar="CSV",
                   help="rocprofv3 --pmc SQ_* counter CSVs of any run -> a per-kernel table of counter means on stdout")
    p.add_argument("--kernel-filter", default="", help="comma-separated substrings: --summarize-sq-by-kernel keeps matching kernels")
    p.add_argument("--summarize-pmc", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                   help="turn the two counter_collection CSVs of the traffic probe into profiles/traffic.json")
    return p.parse_args()


class Runner:
    """Replays a list of zero-argument launch closures in order, cyclically, through HIP graphs when possible:
    one graph holds the whole list, and a run that is not a multiple of the list's length ends with one replay of a
    second graph holding just the remaining calls, so that every step of a timed region is a graph node."""

    def __init__(self, calls, use_graph=True):
        self.calls = calls
        self.use_graph = use_graph
        self.graphs = {}
        self.graph = self._capture(len(calls)) if use_graph else None

    def _capture(self, n):
        if n in self.graphs:
            return self.graphs[n]
        try:
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for c in self.calls[:n]:  # warm every kernel on the capture stream first
                    c()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=side):
                for c in self.calls[:n]:
                    c()
        except Exception as e:  # noqa: BLE001
            print(f"[bench] graph capture failed ({e!r}); launching eagerly", file=sys.stderr)
            g = None
            self.use_graph = False
            torch.cuda.synchronize()
        self.graphs[n] = g
        return g

    def prepare(self, steps):
        """Capture whatever graphs a run of `steps` needs, outside any timed region."""
        rem = steps % len(self.calls)
        if self.use_graph and rem:
            self._capture(rem)

    def run(self, steps):
        n = len(self.calls)
        full, rem = divmod(steps, n)
        tail = self._capture(rem) if (self.use_graph and self.graph is not None and rem) else None
        if self.graph is not None:
            for _ in range(full):
                self.graph.replay()
        else:
            for _ in range(full):
                for c in self.calls:
                    c()
        if tail is not None:
            tail.replay()
        else:
            for c in self.calls[:rem]:
                c()

    def time_both(self, steps):
        """(wall seconds, device seconds from HIP events on the launch stream) of EXACTLY `steps` steps, both taken
        over the same region, bracketed by synchronisations."""
        self.prepare(steps)
        st = torch.cuda.current_stream()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(st)
        self.run(steps)
        e1.record(st)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return wall, e0.elapsed_time(e1) * 1e-3

    def time_wall(self, steps):
        return self.time_both(steps)[0]

    def time_events(self, steps):
        """Average device time per step from HIP events on the launch stream."""
        return self.time_both(steps)[1] / steps

    def prewarm(self, ms):
        """Untimed launches for at least `ms` milliseconds of wall time (clock ramp-up). Returns what it took."""
        t0 = time.perf_counter()
        while True:
            self.run(len(self.calls))
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) * 1e3
            if dt >= ms:
                return dt


def cpu_baseline(L, min_seconds):
    """The oracle, as it stands, on the host cores: whole config-2 blocks until min_seconds pass, once with the
    BLAS library's default thread count and once with one thread. Also returns the block's bit-operation counts
    (Section III-C: BOPs = FLOPs x b_w x b_a) from the oracle's closed form."""
    from oracle import taq_oracle as O
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:  # noqa: BLE001
        threadpool_limits = None
        threads = os.cpu_count() or 1
    kv = O.quantize_kv(L.context, L.mask, L.Wk, L.Wv, L.bits_kv, L.H)
    wq, swq = O.quantize_weight(L.Wq)
    wo, swo = O.quantize_weight(L.Wo)

    def leg(max_reps):
        reps, t0 = 0, time.perf_counter()
        while True:
            O.cross_attn(L.hidden, kv, wq, swq, wo, swo, L.bias_o)
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= min_seconds or reps >= max_reps:
                return reps, dt

    reps, dt = leg(64)
    base = {"value": L.B * L.N * reps / dt, "unit": "query-tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{reps} whole config-2 blocks (B={L.B}, N={L.N}) of oracle.cross_attn in {dt:.1f} s, "
                      f"float64 numpy, os.cpu_count()={os.cpu_count()}"}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            reps1, dt1 = leg(16)
        base["single_thread"] = {"value": L.B * L.N * reps1 / dt1, "unit": "query-tokens/s", "cores": 1,
                                 "sample": f"{reps1} whole config-2 blocks in {dt1:.1f} s, BLAS limited to one thread"}
    b32 = O.block_bops(L.B, L.N, L.C, L.T, L.Cc, 32, 32)
    b88 = O.block_bops(L.B, L.N, L.C, L.T, L.Cc, 8, 8)
    b84 = O.block_bops(L.B, L.N, L.C, L.T, L.Cc, 8, 4)
    bops = {"unit": "bit-operations per block (all five contractions, 2 per multiply-accumulate)",
            "w32a32": b32, "w8a8": b88, "w8a4": b84, "ratio_32_32_over_8_8": b32 / b88, "ratio_32_32_over_8_4": b32 / b84}
    return base, bops


def prep_layer(L, dev, bits_q=8, bits_prob=8, prob_grid=T.TAQ_PROB_LINEAR):
    """Device buffers of one synthetic layer, weight codes formed and packed, K~/V~ quantized once."""
    to = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    s = T.make_shape(B=L.B, N=L.N, C=L.C, H=L.H, T=L.T, Cc=L.Cc, bits_kv=L.bits_kv, bits_q=bits_q,
                     bits_prob=bits_prob, w_layout=1 if L.C % 64 == 0 else 0, prob_grid=prob_grid)
    wq, swq = T.taq_quantize_weight(to(L.Wq))
    wo, swo = T.taq_quantize_weight(to(L.Wo))
    if s.w_layout:
        wq, wo = T.taq_pack_weight(wq, s), T.taq_pack_weight(wo, s)
    d = dict(s=s, wq=wq, wo=wo, scales=torch.cat([swq, swo, to(L.bias_o)]).contiguous(), mask=to(L.mask),
             ctx=to(L.context), Wk=to(L.Wk), Wv=to(L.Wv), hidden=to(L.hidden), bits_kv=L.bits_kv,
             out=torch.empty((L.B, L.N, L.C), dtype=torch.float16, device=dev),
             ws=torch.empty(T.taq_workspace_bytes(s), dtype=torch.uint8, device=dev),
             packed=torch.empty(T.taq_kv_packed_bytes(s), dtype=torch.uint8, device=dev))
    T.taq_quantize_kv(d["ctx"], d["mask"], d["Wk"], d["Wv"], L.bits_kv, s, d["packed"], d["ws"])
    return d


def attn_call(d, debug=None):
    return lambda: T.taq_cross_attn(d["hidden"], d["packed"], d["wq"], d["wo"], d["scales"], d["mask"], d["s"],
                                    d["out"], d["ws"], debug=debug)


def profile_config3(dev, use_graph, reps):
    """For rocprofv3: the 16 cross-attention layers of one UNet step (configs[2]) replayed `reps` times from one HIP
    graph, after one taq_quantize_kv per layer. Prints the measured time per 16-layer step."""
    layers = [prep_layer(L, dev) for L in synth.config3()]
    for d in layers:  # once more, so that the trace holds a second sample of the per-prompt kernels
        T.taq_quantize_kv(d["ctx"], d["mask"], d["Wk"], d["Wv"], d["bits_kv"], d["s"], d["packed"], d["ws"])
    r = Runner([attn_call(d) for d in layers], use_graph=use_graph)
    r.run(2 * len(layers))
    us = r.time_events(reps * len(layers)) * len(layers) * 1e6
    print(json.dumps({"workload": "configs[2]: 16 cross-attention layers of one SD1.5 UNet step, batch 2, int4 K/V",
                      "us_per_16_layer_step": round(us, 2), "replays": reps,
                      "launch": "hip-graph" if r.graph is not None else "eager"}), flush=True)


def other_configs(dev, use_graph):
    """Device time per taq_cross_attn call (and per taq_quantize_kv) for configs 1, 3, 4, 5."""
    out = {}
    prep = lambda L, **kw: prep_layer(L, dev, **kw)

    def timed(calls, reps=40):
        r = Runner(calls, use_graph=use_graph)
        r.prewarm(20.0)  # the clocks drop between measurements (graph capture, set-up copies): ramp them up again
        return r.time_events(reps * len(calls)) * len(calls) * 1e6  # us per pass over `calls`

    import dataclasses
    d2 = prep(dataclasses.replace(synth.config2(), bits_kv=4), bits_q=4, bits_prob=4)  # the 8/4 setting (Table 1)
    out["config2_w8a4_int4kv_q4_p4"] = round(timed([attn_call(d2)] * 4) / 4, 2)
    d2 = prep(dataclasses.replace(synth.config2(), bits_kv=4), bits_q=4, bits_prob=4, prob_grid=T.TAQ_PROB_LOG2)
    out["config2_w8a4_log2_probabilities"] = round(timed([attn_call(d2)] * 4) / 4, 2)
    d1 = prep(synth.config1())
    out["config1_64x1280"] = round(timed([attn_call(d1)] * 4) / 4, 2)
    layers = [prep(L) for L in synth.config3()]
    out["config3_16_layers_total"] = round(timed([attn_call(d) for d in layers], reps=10), 2)
    for L in synth.config4():
        d = prep(L)
        out["config4_%dx%d" % (L.N, L.C)] = round(timed([attn_call(d)] * 4) / 4, 2)
    reqs = [prep(L) for L in synth.config5()]
    table = [dict(hidden=d["hidden"], qkv_packed=d["packed"], Wq=d["wq"], Wo=d["wo"], scales=d["scales"],
                  trigger_mask=d["mask"], out=d["out"]) for d in reqs]
    ws5 = torch.empty(16 * T.taq_workspace_bytes(reqs[0]["s"]), dtype=torch.uint8, device=dev)
    out["config5_16_requests_batched"] = round(timed([lambda: T.taq_cross_attn_batched(table, reqs[0]["s"], ws5)] * 2,
                                                     reps=10) / 2, 2)

    # int8 matrix work of the C = 1280 layers (the shapes at which the projections can be compute-bound) against the
    # int8 MFMA peak, next to the ceiling the HBM roofline leaves: whole taq_cross_attn call, weights + hidden + out +
    # K~/V~ as algorithmic bytes. Cache-resident: the same buffers every call.
    mf = {}
    for key, L, us in (("config3_256x1280", synth.config3(layers=[10])[0], None), ("config4_1024x1280", synth.config4()[1], None)):
        d = prep(L)
        us = timed([attn_call(d)] * 4) / 4
        M = L.B * L.N
        ops = 2.0 * M * L.C * L.C * 2 + 2.0 * M * L.T * L.C
        nbytes = M * 4 * L.C + 2 * L.C * L.C + L.B * (L.T * L.C + 8 * L.H * L.T)
        mf[key] = {"us_per_call": round(us, 2), "int8_GOP": ops / 1e9, "achieved_TOPS": ops / us / 1e6,
                   "frac_of_int8_peak": ops / us / 1e6 / INT8_PEAK_TOPS,
                   "ceiling_frac_from_hbm_roofline": min(1.0, ops / nbytes * HBM_PEAK_GBS * 1e9 / (INT8_PEAK_TOPS * 1e12)),
                   "data": "cache-resident (one buffer set)"}
    return out, mf


def gemm_stage_mfma(dev, use_graph, only=("to_q", "to_out")):
    """The int8 GEMM of the kernel-per-stage path alone (stage masks TO_Q / TO_OUT of taq_cross_attn): MFMA utilisation
    at (M = 2048, C = 1280) and (M = 8192, C = 320), cache-resident (one buffer set, re-used by every call), next to the
    ceiling that this GEMM's own bytes leave: A [M, C] + W [C, C] int8 in, [M, C] float32 (to_q) or fp16 (to_out) out,
    at the HBM peak; the time of a launch (a few microseconds at these sizes) is not in the ceiling."""
    res = {}
    for key, L in (("M2048_C1280", synth.config4()[1]), ("M8192_C320", synth.config2())):
        d = prep_layer(L, dev)
        s = d["s"]
        allbits = (T.TAQ_STAGE_HIDDEN_QUANT | T.TAQ_STAGE_TO_Q | T.TAQ_STAGE_Q_QUANT | T.TAQ_STAGE_ATTN_CORE
                   | T.TAQ_STAGE_O_QUANT | T.TAQ_STAGE_TO_OUT)
        attn_call(d, T.make_debug(s, dev, stage_mask=allbits, taps=False)[0])()  # valid stage buffers in the workspace
        M = L.B * L.N
        ops = 2.0 * M * L.C * L.C
        for name, bit, out_bytes in (("to_q", T.TAQ_STAGE_TO_Q, 4), ("to_out", T.TAQ_STAGE_TO_OUT, 2)):
            if name not in only:
                continue
            dbg = T.make_debug(s, dev, stage_mask=bit, taps=False)[0]
            r = Runner([attn_call(d, dbg)] * 8, use_graph=use_graph)
            r.prewarm(20.0)
            t = r.time_events(400)
            nbytes = M * L.C + L.C * L.C + M * L.C * out_bytes
            t_floor = max(ops / (INT8_PEAK_TOPS * 1e12), nbytes / (HBM_PEAK_GBS * 1e9))
            res[key + "_" + name] = {"us": round(t * 1e6, 2), "int8_GOP": ops / 1e9, "achieved_TOPS": ops / t / 1e12,
                                     "frac_of_int8_peak": ops / t / 1e12 / INT8_PEAK_TOPS,
                                     "ceiling_frac_from_hbm_roofline": ops / (INT8_PEAK_TOPS * 1e12) / t_floor,
                                     "bytes": nbytes, "data": "cache-resident (one buffer set)"}
    return res


COPY_BYTES = 256 << 20  # the known-size copy of the traffic probe reads and writes this many bytes
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12  # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3e12 lane-ops/s
#   (the chip's 157.3 TFLOP/s fp32 vector figure is this x 2 for an FMA x 2 for packed fp32, which this build may not use)


def summarize_sq(csvs):
    """Mean per launch of every SQ_* counter over the fused kernel's dispatches (rocprofv3 --pmc, one CSV per pass);
    writes profiles/fused_block_kernel_cfg2_pmc.json, which the ALU-roofline figure of the bench line reads."""
    import csv
    acc = {}
    for path in csvs:
        for r in csv.DictReader(open(path)):
            if "fused_block_kernel" in r["Kernel_Name"]:
                acc.setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    if not acc:
        raise SystemExit("no fused_block_kernel dispatches in " + " ".join(csvs))
    out = {k: sum(v[4:]) / max(1, len(v[4:])) for k, v in sorted(acc.items())}  # skip the first (cold) dispatches
    out["wavefronts_per_launch"] = out.get("SQ_WAVES", 2048.0)
    path = os.path.join(ROOT, "profiles", "fused_block_kernel_cfg2_pmc.json")
    json.dump(out, open(path, "w"), indent=1)
    waves = out["wavefronts_per_launch"]
    with open(path[:-5] + ".txt", "w") as f:
        f.write("# rocprofv3 hardware counters of taq::fused_block_kernel<40, 8, 2, 1, 0, 32, false, 5, false> at configs[1]\n"
                "# (B=2 N=4096 C=320 H=8 T=77). Commands (run from /tmp on the MI355X box, one pass per counter set):\n"
                "#   rocprofv3 --pmc <at most 8 SQ_ counters> --output-format csv -d outK -o p -- python3 bench.py --profile-only --no-graph --steps 64 --warmup 16\n"
                "#   python3 bench.py --summarize-sq out1/p_counter_collection.csv out2/p_counter_collection.csv ...   (writes this file and the .json)\n"
                "# mean over the dispatches of the kernel (first 4 skipped); per wavefront = mean / wavefronts per launch\n"
                "# (SQ_*_CYCLES, SQ_WAIT* and SQ_ACTIVE* tick once per 4 clocks)\n"
                "counter,mean_per_launch,per_wavefront\n")
        for k, v in out.items():
            if k != "wavefronts_per_launch":
                f.write(f"{k},{v:.0f},{v / waves:.1f}\n")
    print(json.dumps(out))


def summarize_trace(stats_csv, out_txt, command, notes):
    """The rows of this library's kernels from a rocprofv3 --kernel-trace --stats kernel_stats.csv, as text."""
    import csv
    rows = [r for r in csv.DictReader(open(stats_csv)) if "taq::" in r["Name"]]
    with open(os.path.join(ROOT, "profiles", out_txt), "w") as f:
        f.write("# rocprofv3 --kernel-trace --stats, this library's kernels. Command (run from /tmp on the MI355X box):\n")
        f.write("#   " + command + "\n")
        f.write("#   python3 bench.py --summarize-trace <the run's kernel_stats.csv> " + out_txt + " '<command>' <notes>\n")
        for n in notes:
            f.write("# " + n + "\n")
        f.write("kernel,calls,total_us,average_us,min_us,max_us,percent\n")
        for r in rows:
            name = r["Name"].split("(")[0].replace("void ", "")
            f.write(f"{name},{r['Calls']},{float(r['TotalDurationNs']) / 1e3:.1f},{float(r['AverageNs']) / 1e3:.2f},"
                    f"{float(r['MinNs']) / 1e3:.2f},{float(r['MaxNs']) / 1e3:.2f},{float(r['Percentage']):.2f}\n")
    print(open(os.path.join(ROOT, "profiles", out_txt)).read())


def summarize_sq_by_kernel(csvs, keep=()):
    """Per kernel (template arguments kept, parameter list dropped) and grid size: the mean over its dispatches of every
    counter found in the CSVs, per launch and per wavefront. Text on stdout, for a summary file under profiles/."""
    import csv
    print("# rocprofv3 hardware counters per kernel of this library. Commands (run from /tmp on the MI355X box, one pass per\n"
          "# counter set, at most 8 SQ_ counters each; <workload> is one of bench.py's --profile-config3 / --profile-gemm /\n"
          "# --profile-only, launched eagerly):\n"
          "#   rocprofv3 --pmc <counters> --output-format csv -d outK -o p -- python3 bench.py <workload> --no-graph\n"
          "#   python3 bench.py --summarize-sq-by-kernel out1/p_counter_collection.csv out2/p_counter_collection.csv ... [--kernel-filter a,b]\n"
          "# mean over all dispatches of the kernel at that grid; SQ_*_CYCLES, SQ_WAIT* and SQ_ACTIVE* tick once per 4 clocks")
    acc = {}
    for path in csvs:
        for r in csv.DictReader(open(path)):
            name = r["Kernel_Name"].split("(")[0].replace("void ", "").replace("taq::", "")
            if "taq::" not in r["Kernel_Name"] or (keep and not any(k in name for k in keep)):
                continue
            key = (name, r.get("Grid_Size", ""), r.get("Workgroup_Size", ""))
            acc.setdefault(key, {}).setdefault(r["Counter_Name"], []).append(float(r["Counter_Value"]))
    for key in sorted(acc, key=lambda k: (k[0], k[1])):
        cs = acc[key]
        n = min(len(v) for v in cs.values())
        waves = sum(cs["SQ_WAVES"]) / len(cs["SQ_WAVES"]) if "SQ_WAVES" in cs else float("nan")
        print(f"{key[0]}  grid {key[1]} wg {key[2]}  dispatches {n}  wavefronts {waves:.0f}")
        for c in sorted(cs):
            m = sum(cs[c]) / len(cs[c])
            print(f"    {c:30s} {m:14.1f} per launch {m / waves:10.1f} per wavefront")


def summarize_pmc(fetch_csv, write_csv):
    """FETCH_SIZE / WRITE_SIZE come in KiB per dispatch. Scale each by what the same counter reads for the
    plain copy kernel of known size, then average over the fused kernel's dispatches."""
    import csv

    def per_kernel(path, counter):
        rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == counter]
        copy = [float(r["Counter_Value"]) for r in rows if "copy" in r["Kernel_Name"].lower()]
        copy = [v for v in copy if v >= 0.5 * max(copy)] if copy else []  # the big probe copies only
        fused = [float(r["Counter_Value"]) for r in rows if "fused_block_kernel" in r["Kernel_Name"]]
        return copy, fused

    out = {}
    for name, path, counter in (("fetch", fetch_csv, "FETCH_SIZE"), ("write", write_csv, "WRITE_SIZE")):
        copy, fused = per_kernel(path, counter)
        if not copy or not fused:
            raise SystemExit(f"{path}: no copy or fused dispatches found")
        copy_kib = sum(copy) / len(copy)
        factor = (COPY_BYTES / 1024.0) / copy_kib  # true KiB per counted KiB
        fused_kib = sum(fused[4:]) / max(1, len(fused[4:]))  # skip the first dispatches (cold caches)
        out[name] = {"copy_counter_KiB": copy_kib, "scale_factor": factor, "fused_counter_KiB": fused_kib,
                     "fused_bytes_per_launch": fused_kib * factor * 1024.0, "dispatches": len(fused)}
    out["fused_bytes_per_launch"] = out["fetch"]["fused_bytes_per_launch"] + out["write"]["fused_bytes_per_launch"]
    path = os.path.join(ROOT, "profiles", "fused_block_kernel_cfg2_hbm_traffic.json")
    json.dump(out, open(path, "w"), indent=1)
    with open(path[:-5] + ".md", "w") as f:
        f.write("# HBM traffic of taq::fused_block_kernel<40, 8, 2, ...> at configs[1] (B=2 N=4096 C=320 H=8 T=77)\n\n"
                "Commands (run from /tmp on the MI355X box; each counter in a pass of its own):\n\n"
                "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d fetch -o p -- python3 bench.py --traffic-probe --steps 64\n"
                "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d write -o p -- python3 bench.py --traffic-probe --steps 64\n"
                "    python3 bench.py --summarize-pmc fetch/p_counter_collection.csv write/p_counter_collection.csv\n\n"
                "`--traffic-probe` first runs four device copies of 256 MiB (known size), then 64 eager `taq_cross_attn`\n"
                "calls over the ring of buffer sets. `--summarize-pmc` scales each counter by what it read for the copy and\n"
                "writes this file and `fused_block_kernel_cfg2_hbm_traffic.json`:\n\n"
                "| counter | copy of 256 MiB reads as | scale factor | fused kernel reads as | bytes per launch |\n|---|---|---|---|---|\n")
        for name, counter in (("fetch", "FETCH_SIZE"), ("write", "WRITE_SIZE")):
            o = out[name]
            f.write(f"| {counter} | {o['copy_counter_KiB']:.1f} KiB | {o['scale_factor']:.3f} | {o['fused_counter_KiB']:.1f} KiB | "
                    f"{o['fused_bytes_per_launch'] / 1e6:.2f} MB |\n")
        tokens, C = 8192, 320
        f.write(f"\nTotal {out['fused_bytes_per_launch'] / 1e6:.2f} MB per launch; the algorithmic bytes of the launch are "
                f"{(tokens * 4 * C + 2 * C * C + 2 * (2 * 77 * C + 2 * 4 * 8 * 77)) / 1e6:.2f} MB (hidden in and out "
                f"{tokens * 4 * C / 1e6:.2f} MB, the rest weights and K~/V~).\n")
    print(json.dumps(out))


def main():
    a = parse()
    if a.summarize_sq:
        summarize_sq(a.summarize_sq)
        return
    if a.summarize_trace:
        summarize_trace(a.summarize_trace[0], a.summarize_trace[1], a.summarize_trace[2], a.summarize_trace[3:])
        return
    if a.summarize_sq_by_kernel:
        summarize_sq_by_kernel(a.summarize_sq_by_kernel, tuple(k for k in a.kernel_filter.split(",") if k))
        return
    if a.summarize_pmc:
        summarize_pmc(*a.summarize_pmc)
        return
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    T.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if a.profile_config3:
        profile_config3(dev, not a.no_graph, reps=50)
        return
    if a.profile_gemm:
        print(json.dumps({"gemm_i8_stage_mfma": gemm_stage_mfma(dev, not a.no_graph, only=("to_q",))}), flush=True)
        return
    L = synth.config2()
    s = T.make_shape(B=L.B, N=L.N, C=L.C, H=L.H, T=L.T, Cc=L.Cc, bits_kv=L.bits_kv, w_layout=1)
    to = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    ctx, mask, Wk, Wv = to(L.context), to(L.mask), to(L.Wk), to(L.Wv)
    wq, swq = T.taq_quantize_weight(to(L.Wq))
    wo, swo = T.taq_quantize_weight(to(L.Wo))
    wq, wo = T.taq_pack_weight(wq, s), T.taq_pack_weight(wo, s)  # once per checkpoint: operand-ordered copy
    scales = torch.cat([swq, swo, to(L.bias_o)]).contiguous()
    ws_bytes = T.taq_workspace_bytes(s)
    packed = torch.empty(T.taq_kv_packed_bytes(s), dtype=torch.uint8, device=dev)
    ws0 = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    T.taq_quantize_kv(ctx, mask, Wk, Wv, L.bits_kv, s, packed, ws0)
    hidden0 = to(L.hidden)
    # The ring: distinct (hidden, out) pairs; ONE workspace shared by all of them (this shape runs as a single kernel
    # that never touches it, so it adds no traffic and is not counted below).
    ring = []
    for _ in range(max(1, a.ring)):
        ring.append(dict(hidden=hidden0.clone(), out=torch.empty((L.B, L.N, L.C), dtype=torch.float16, device=dev),
                         ws=ws0))
    ring_mb = sum(r["hidden"].numel() * 2 + r["out"].numel() * 2 for r in ring) / 1e6  # bytes the timed loop touches
    torch.cuda.synchronize()

    def step_call(r, dbg=None):
        return lambda: T.taq_cross_attn(r["hidden"], packed, wq, wo, scales, mask, s, r["out"], r["ws"], debug=dbg)

    if a.traffic_probe:
        src = torch.empty(COPY_BYTES, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        for i in range(a.steps):
            step_call(ring[i % len(ring)])()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "copy_bytes": COPY_BYTES, "steps": a.steps}), flush=True)
        return
    runner = Runner([step_call(r) for r in ring], use_graph=not a.no_graph)
    runner.prepare(a.steps)
    runner.prepare(a.warmup)
    prewarm_ms = runner.prewarm(a.prewarm_ms) if a.prewarm_ms > 0 else 0.0  # untimed, reported: clock ramp-up
    runner.run(a.warmup)
    # EXACTLY a.steps steps between two synchronisations; HIP events on the launch stream bracket the same region
    wall, dev_s = runner.time_both(a.steps)
    ms_per_step = wall * 1e3 / a.steps
    t_fused = dev_s / a.steps  # one step = one launch of the fused block kernel
    tokens = L.B * L.N
    value = tokens / (wall / a.steps)
    result = {
        "metric": "TAQ cross-attn query-tokens/sec at 4096q SD1.5 shape", "value": value,
        "unit": "query-tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "configs[1]: SD1.5 64x64 cross-attn, B=2 N=4096 C=320 H=8 T=77 Cc=768, "
                               "1 fp16 trigger row, int8 K/V, 8-bit probs, W8A8 to_q/to_out",
                   "launch": "hip-graph" if runner.graph is not None else "eager",
                   "ring_buffer_sets": len(ring), "ring_MB": round(ring_mb, 1),
                   "ring_MB_counts": "hidden + out of every set (the bytes the timed loop reads and writes)"},
        "prewarm_ms": round(prewarm_ms, 1),
        "device_ms_per_step_hip_events": t_fused * 1e3,
    }
    if a.profile_only:
        print(json.dumps(result), flush=True)
        return

    # ---- side measurements (not part of `value`)
    # cache-resident variant: one buffer set reused
    res_runner = Runner([step_call(ring[0])] * 4, use_graph=not a.no_graph)
    res_runner.run(16)
    side_steps = max(a.steps, 512)
    result["value_cache_resident"] = tokens / (res_runner.time_wall(side_steps) / side_steps)
    # taq_quantize_kv, once per prompt
    kv_runner = Runner([lambda: T.taq_quantize_kv(ctx, mask, Wk, Wv, L.bits_kv, s, packed, ws0)] * 4,
                       use_graph=not a.no_graph)
    kv_runner.prewarm(10.0)
    kv_s = kv_runner.time_events(512)
    result["quantize_kv_us"] = kv_s * 1e6
    # same with the to_k / to_v weight codes formed once per checkpoint
    kc, ks_ = T.taq_quantize_weight(Wk)
    vc, vs_ = T.taq_quantize_weight(Wv)
    wkv, swkv = torch.cat([kc, vc]).contiguous(), torch.cat([ks_, vs_]).contiguous()
    kv8_runner = Runner([lambda: T.taq_quantize_kv_w8(ctx, mask, wkv, swkv, L.bits_kv, s, packed, ws0)] * 4,
                        use_graph=not a.no_graph)
    kv8_runner.prewarm(10.0)
    result["quantize_kv_cached_weight_codes_us"] = kv8_runner.time_events(512) * 1e6
    result["value_with_quantize_kv_every_step"] = tokens / (wall / a.steps + kv_s)

    # ---- roofline of the dominant kernel. taq_cross_attn at this shape is ONE kernel (the fused block), so its
    # average launch duration is the device time of the timed region (HIP events on the launch stream) / steps.
    C, H, T_ = L.C, L.H, L.T
    # algorithmic bytes per launch: hidden in (2C) + out (2C) per token, both weight matrices, int8 K~/V~ + scales
    alg_bytes = tokens * 4 * C + 2 * C * C + L.B * (2 * T_ * C + 2 * 4 * H * T_)
    gbs = alg_bytes / t_fused / 1e9
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "fused_block_kernel_cfg2_hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            traffic = tj.get("fused_bytes_per_launch")
            traffic_src = "profiles/fused_block_kernel_cfg2_hbm_traffic.json (rocprofv3 --pmc, committed; not measured in this run)"
        except Exception:  # noqa: BLE001
            traffic = None
    result["roofline"] = {"kernel": "fused_block_kernel<40,8>", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                          "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": t_fused * 1e6}
    # vector-ALU view of the same kernel. Lane-operations per launch = the count of vector instructions
    # (SQ_INSTS_VALU, rocprofv3 --pmc, a committed counter file) x 64 lanes, divided by this run's launch time;
    # transcendentals count once although they issue at quarter rate.
    ppath = os.path.join(ROOT, "profiles", "fused_block_kernel_cfg2_pmc.json")
    if os.path.exists(ppath):
        try:
            pj = json.load(open(ppath))
            valu = float(pj["SQ_INSTS_VALU"])
            lane_ops = valu * 64.0
            result["roofline_alu"] = {"kernel": "fused_block_kernel<40,8>", "bound": "alu",
                                      "achieved": lane_ops / t_fused / 1e12, "peak": ALU_PEAK_TLANEOPS,
                                      "unit": "T lane-op/s", "frac": lane_ops / t_fused / 1e12 / ALU_PEAK_TLANEOPS,
                                      "valu_instructions_per_launch": valu,
                                      "counter_source": "profiles/fused_block_kernel_cfg2_pmc.json (committed counter "
                                                        "file; the launch time is this run's)"}
        except Exception:  # noqa: BLE001
            pass
    # integer matrix work inside the same kernel: to_q + to_out (2*M*C*C each) and K~ Q~^T (2*M*T*C)
    int8_ops = 2.0 * tokens * C * C * 2 + 2.0 * tokens * T_ * C
    result["roofline_mfma_int8"] = {"kernel": "fused_block_kernel<40,8>", "bound": "mfma", "achieved": int8_ops / t_fused / 1e12,
                                    "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": int8_ops / t_fused / 1e12 / INT8_PEAK_TOPS,
                                    "ceiling_frac_from_hbm_roofline": min(1.0, int8_ops / alg_bytes * HBM_PEAK_GBS * 1e9 / (INT8_PEAK_TOPS * 1e12)),
                                    "note": "ceiling = the int8 rate at which this shape's algorithmic bytes would saturate HBM"}
    # ---- the same path as one kernel per stage (general path; other shapes run this way), each timed alone
    stages = [("hidden_quant", T.TAQ_STAGE_HIDDEN_QUANT), ("to_q", T.TAQ_STAGE_TO_Q), ("q_quant", T.TAQ_STAGE_Q_QUANT),
              ("attn_core", T.TAQ_STAGE_ATTN_CORE), ("o_quant", T.TAQ_STAGE_O_QUANT), ("to_out", T.TAQ_STAGE_TO_OUT)]
    per_stage = {}
    sring = [dict(r, ws=torch.empty(ws_bytes, dtype=torch.uint8, device=dev)) for r in ring[:8]]  # stages do use the workspace
    for r in sring:  # fill every workspace once with a whole pass, so that each stage alone reads valid data
        allbits = 0
        for _, bit in stages:
            allbits |= bit
        step_call(r, T.make_debug(s, dev, stage_mask=allbits, taps=False)[0])()
    for name, bit in stages:
        dbgs = [T.make_debug(s, dev, stage_mask=bit, taps=False)[0] for _ in sring]
        rr = Runner([step_call(r, d) for r, d in zip(sring, dbgs)], use_graph=not a.no_graph)
        rr.run(len(sring))
        per_stage[name] = rr.time_events(256)
    core_bytes = tokens * (5 * C + 4 * H)  # int8 Q~ + its scales in, float32 A^ V~ out (what the stage kernel moves)
    gemm_ops = 2.0 * tokens * C * C
    result["unfused_stages"] = {
        "stage_us": {k: round(v * 1e6, 3) for k, v in per_stage.items()},
        "attn_core_GBps": core_bytes / per_stage["attn_core"] / 1e9,
        "attn_core_frac_of_hbm": core_bytes / per_stage["attn_core"] / 1e9 / HBM_PEAK_GBS,
        "to_q_TOPS": gemm_ops / per_stage["to_q"] / 1e12, "to_out_TOPS": gemm_ops / per_stage["to_out"] / 1e12,
        "to_q_frac_of_int8_peak": gemm_ops / per_stage["to_q"] / 1e12 / INT8_PEAK_TOPS,
        "note": "kernel-per-stage path (8 buffer sets, 168 MB with their workspaces' stage buffers: partly cache-resident), "
                "used for shapes the fused kernel is not instantiated for",
    }
    # ---- the other benchmark configurations (latency per call; they are parity-test cases, not bench lines)
    oc, mf = other_configs(dev, not a.no_graph)
    result["other_configs_us"] = oc
    result["roofline_mfma_int8_c1280"] = mf
    result["gemm_i8_stage_mfma"] = gemm_stage_mfma(dev, not a.no_graph)
    if not a.no_cpu_baseline:
        result["cpu_baseline"], result["block_bops"] = cpu_baseline(L, a.cpu_seconds)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
