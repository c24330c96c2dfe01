#!/usr/bin/env python3
"""Benchmark of the AWQ W4A16 hot path on one MI355X.

Headline workload (`config.workload`): the seven projections of a Llama-2-7B-shaped
decoder layer (q/k/v/o 4096x4096, gate/up 11008x4096, down 4096x11008), INT4 group-128
weights, decode at M = 1, each layer issued as ONE grouped launch (awq_w4a16_linear_multi).
One *step* is one pass over `--layers` distinct layers (32 = the whole stack, 3.4 GB of packed
weights: one launch per layer, every weight byte comes from HBM and not from the 256 MB
Infinity Cache).  `value` is algorithmic bytes per step / time per step.  Before the warm-up the
headline launches run for a fixed span of GPU time (`config.settle_ms`), so that a run of a few
steps measures the same steady state as a long one.

Also measured in the same run: the same layer as seven awq_w4a16_linear calls and as the four
dependent launches of a decoder (`config.per_launch_mode`, `config.dependent_launch_mode`),
the M = 2048 prefill GEMM (`roofline.prefill`), and, under `extras`, grouped decode at M = 4
and 16, several layers per launch, awq_quantize_pack, the 3- and 2-bit forms, attention, the
scale search, and the CPU oracle on the host cores (`cpu_baseline`).

Everything timed goes through the C ABI (paper_2306_00978_amd -> libawq_mi355x.so).
Only the cpu_baseline leg imports the oracle.
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

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2516.6


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=150,
                    help="timed steps; one step = one pass over all --layers layers")
    ap.add_argument("--warmup", type=int, default=15)
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="GPU time of headline launches run before the warm-up (clock and power "
                         "state of a fresh process settle within about 20 ms)")
    ap.add_argument("--streams", type=int, default=2,
                    help="streams the launches of a step alternate over in the headline run (the layers of the "
                         "workload are independent); 1 = everything on one stream")
    ap.add_argument("--layers", type=int, default=32,
                    help="distinct layers cycled (cold cache); 32 = the whole Llama-2-7B-shaped stack")
    ap.add_argument("--graph", action="store_true",
                    help="replay the headline step from a hipGraph instead of launching it on the stream "
                         "(slower for a single-kernel step; the multi-launch extras always use graphs)")
    ap.add_argument("--skip-extras", action="store_true",
                    help="only the headline decode measurement (used under rocprofv3)")
    ap.add_argument("--legs", default="modes,prefill,extras",
                    help="comma list of the measurements run after the headline one: modes (the layer as "
                         "7 calls and as 4 dependent launches), prefill (M = 2048 GEMM), extras")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain elementwise copy of known size (256 MiB read, 256 MiB "
                         "written, 5 times): the calibration kernel for rocprofv3 FETCH_SIZE / WRITE_SIZE")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads
    import paper_2306_00978_amd as awq

    awq.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    shapes = workloads.LLAMA2_7B_LAYER
    L = max(1, args.layers)
    legs = set() if args.skip_extras else {t for t in args.legs.split(",") if t}

    # ------------------------------------------------------------------ inputs (resident in HBM)
    # activations / calibration rows per distinct input width, from the seeded generator
    s_by_k, x_by_k, calib_by_k = {}, {}, {}
    for K in (4096, 11008):
        out = workloads.outlier_channels(K, 1, 0, 0)
        calib = workloads.activations(workloads.CALIB_TOKENS, K, 1, 0, 0, workloads.ROLE_CALIB, out)
        x = workloads.activations(workloads.PREFILL_M, K, 1, 0, 0, workloads.ROLE_X, out)
        calib_by_k[K] = calib
        s = awq.awq_act_scale(torch.from_numpy(calib).to(dev), 0.5)
        s_by_k[K] = s
        x_by_k[K] = awq.awq_apply_inv_scale(torch.from_numpy(x).to(dev), s)

    # weights: layer 0 from the numpy generator (also feeds the CPU baseline), the other
    # layers from a seeded device generator with the same distribution
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.BASE_SEED)
    layers = []
    W0 = {}
    arena_bytes = sum((b + 255) // 256 * 256 for _, N, K in shapes for b in awq.awq_packed_sizes(N, K))
    arenas = []
    quant_calls, quant_layer_calls = [], []
    quant_bytes = 0
    for l in range(L):
        packed, mats = [], []
        arena = torch.empty(arena_bytes, dtype=torch.uint8, device=dev)   # one buffer per layer
        arenas.append(arena)
        off = 0
        for p, (name, N, K) in enumerate(shapes):
            if l == 0:
                Wh = workloads.weights(N, K, workloads.SIGMA_7B, 1, 0, p)
                W0[p] = Wh
                W = torch.from_numpy(Wh).to(dev)
            else:
                W = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32)
                     * workloads.SIGMA_7B).to(torch.float16)
            qb, sb, zb = awq.awq_packed_sizes(N, K)
            views = []
            for nb_ in (qb, sb, zb):
                views.append(arena[off:off + nb_])
                off += (nb_ + 255) // 256 * 256
            out = (views[0], views[1].view(torch.float16), views[2])
            quant_calls.append(awq.prepare_quantize_pack(W, s_by_k[K], out))     # keeps W alive
            mats.append((W, s_by_k[K], out))
            quant_bytes += 2 * N * K + qb + sb + zb + 4 * K
            packed.append(out)
            del W
        layers.append(packed)
        quant_layer_calls.append(awq.prepare_quantize_pack_multi(mats))
        del mats
    # configs[4]: ONE awq_quantize_pack pass over all the weight matrices (7 per layer), the fp16
    # sources resident in HBM (13 GB for 32 layers), one call per matrix back to back.  The first
    # pass is the warm-up (code objects, page tables), the second one is timed.
    for call in quant_calls:
        call()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for call in quant_calls:
        call()
    e1.record()
    torch.cuda.synchronize()
    quant_ms = e0.elapsed_time(e1)
    # the same pass as one awq_quantize_pack_multi call per layer (seven matrices per launch)
    for call in quant_layer_calls[:2]:
        call()
    torch.cuda.synchronize()
    e0.record()
    for call in quant_layer_calls:
        call()
    e1.record()
    torch.cuda.synchronize()
    quant_layer_ms = e0.elapsed_time(e1)
    del quant_calls, quant_layer_calls                                           # frees the fp16 sources
    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ decode launch modes
    # "grouped": ONE awq_w4a16_linear_multi per `span` layers (span = 1: the 7 projections of
    #            a layer in one launch);
    # "fused":   4 launches per layer as TinyChat runs it (Q,K,V in one kernel; gate,up in one);
    # "single":  7 awq_w4a16_linear launches per layer.
    ys_by_m = {}
    plans = {}

    def outputs(M):
        return ys_by_m.setdefault(M, [torch.empty((M, N), dtype=torch.float16, device=dev)
                                      for _, N, K in shapes])

    def entries(l, M, ps):
        ys = outputs(M)
        return [(x_by_k[shapes[p][2]][:M], *layers[l][p], ys[p], shapes[p][1]) for p in ps]

    def plan(mode, l, M, span=1):
        key = (mode, l, M, span)
        if key not in plans:       # arguments marshalled once; a call is then one C call
            if mode == "grouped":
                ent = []
                for j in range(span):
                    ent += entries((l + j) % L, M, range(7))
                calls = [awq.prepare_linear_multi(ent)]
            elif mode == "fused":
                calls = [awq.prepare_linear_multi(entries(l, M, ps))
                         for ps in ((0, 1, 2), (3,), (4, 5), (6,))]
            else:
                ys = outputs(M)
                calls = [awq.prepare_linear(x_by_k[K][:M], *layers[l][p], ys[p], N)
                         for p, (name, N, K) in enumerate(shapes)]
            plans[key] = calls
        return plans[key]

    def step_bytes(M):
        return sum(workloads.algorithmic_bytes(M, N, K) for _, N, K in shapes)

    last_spread = {}

    def time_decode(mode, M, steps, warmup, use_graph, span=1, cycle=None, settle_ms=0.0, streams=1):
        """One step = one pass over the L distinct layers (`cycle` of them), `span` layers per
        call of `mode`.  Returns (wall ms, event ms) per step and the launches of a step, so that
        the weights a launch reads were last touched a whole pass (3.4 GB) ago.  streams > 1: the
        calls of a pass go alternately to that many streams of default priority, which join the
        current stream wherever an event is recorded."""
        starts = list(range(0, (cycle or L) - span + 1, span)) or [0]
        graphs = None
        if use_graph:
            graphs = []
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for call in plan(mode, 0, M, span):
                    call()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            for l in starts:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for call in plan(mode, l, M, span):
                        call()
                graphs.append(g)
        per_pass = [plan(mode, l, M, span) for l in starts]
        launches = sum(len(c) for c in per_pass)
        cur = torch.cuda.current_stream()
        side = [torch.cuda.Stream() for _ in range(streams)] if streams > 1 and graphs is None else []
        handles = [st.cuda_stream for st in side]
        flat = [call for calls in per_pass for call in calls]

        def fork():                          # the side streams start behind the current stream
            for st in side:
                st.wait_stream(cur)

        def join():                          # the current stream continues behind the side streams
            for st in side:
                cur.wait_stream(st)

        def one_pass():
            if side:
                for i, call in enumerate(flat):
                    call(handles[i % len(handles)])
                return
            if graphs is not None:
                for g in graphs:
                    g.replay()
            else:
                for calls in per_pass:
                    for call in calls:
                        call()

        fork()
        one_pass()                          # set-up: every layer's weights touched once (page tables)
        join()
        # events around batches of steps as well: the spread of the per-step time.  They are
        # created (and recorded once) before the settling phase, so that nothing but the mandated
        # synchronisation lies between the warm-up and the first timed launch.
        nbat = max(1, min(20, steps // 4))
        bounds = [steps * b // nbat for b in range(nbat + 1)]
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(nbat + 1)]
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for ev in evs + [s0, s1]:
            ev.record()
        # settling phase: the same launches for a fixed span of GPU time, whatever --warmup says
        # (the first ~20 ms of work in a fresh process run at a lower clock)
        settled = 0.0
        while settled < settle_ms:
            s0.record()
            fork()
            for _ in range(4):
                one_pass()
            join()
            s1.record()
            s1.synchronize()
            settled += s0.elapsed_time(s1)
        fork()
        for i in range(warmup):
            one_pass()
        join()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        evs[0].record()
        for b in range(nbat):
            fork()
            for i in range(bounds[b], bounds[b + 1]):
                one_pass()
            join()
            evs[b + 1].record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        ev_ms = evs[0].elapsed_time(evs[-1])
        per = [evs[b].elapsed_time(evs[b + 1]) / (bounds[b + 1] - bounds[b]) for b in range(nbat)]
        per.sort()
        last_spread.clear()
        last_spread.update({"median": per[len(per) // 2], "p10": per[len(per) // 10],
                            "p90": per[min(len(per) - 1, (9 * len(per)) // 10)],
                            "settle_ms": settled})
        return wall_ms / steps, ev_ms / steps, launches

    use_graph = args.graph
    # The kernel's own launch duration (roofline): everything on one stream, one launch after the other.
    wall1_ms, ev_ms, launches = time_decode("grouped", 1, args.steps, args.warmup, use_graph,
                                            settle_ms=args.settle_ms)
    spread1 = dict(last_spread)
    spread1.pop("settle_ms")
    # The headline (whole-job throughput): the same launches, alternating over --streams streams.  The
    # layers of configs[1] / configs[4] carry no data dependence, so the run-out of one launch may
    # overlap the start of the next.
    n_streams = 1 if use_graph else max(1, args.streams)
    if n_streams > 1:
        wall_ms, evh_ms, _ = time_decode("grouped", 1, args.steps, args.warmup, False,
                                         settle_ms=args.settle_ms, streams=n_streams)
        spread = dict(last_spread)
        settle_ms = spread.pop("settle_ms")
    else:
        wall_ms, evh_ms, spread = wall1_ms, ev_ms, dict(spread1)
        settle_ms = args.settle_ms
    bytes_m1 = step_bytes(1)                 # one layer = one launch
    bytes_step = bytes_m1 * launches
    value = bytes_step / (wall_ms * 1e-3) / 1e9

    # read-only reference on the same buffers: one streaming pass over a layer's packed arrays
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for i in range(L):
        awq.awq_read_probe(arenas[i], sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps_probe = L * max(2, min(args.steps, 8))
    e0.record()
    for i in range(reps_probe):
        awq.awq_read_probe(arenas[i % L], sink)
    e1.record()
    torch.cuda.synchronize()
    probe_us = e0.elapsed_time(e1) / reps_probe * 1e3
    probe_gbs = arena_bytes / (probe_us * 1e-6) / 1e9

    def clocks():
        """Active clock levels from the driver's sysfs files (no child process involved)."""
        import glob
        found = {}
        for kind in ("sclk", "mclk"):
            for path in sorted(glob.glob(f"/sys/class/drm/card*/device/pp_dpm_{kind}")):
                try:
                    active = [ln.strip() for ln in open(path) if ln.strip().endswith("*")]
                except OSError:
                    continue
                if active:
                    found[kind] = active[0].rstrip("* ").strip()
                    break
        return found or {"unavailable": "no pp_dpm_* files readable"}
    kernel_us = ev_ms * 1e3 / launches                     # average per launch, HIP events
    achieved = bytes_m1 / (kernel_us * 1e-6) / 1e9

    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE.  The figure in
    # profiles/traffic.txt is a measurement of one kernel revision: it is reported only while the
    # kernel's source is still the one that was profiled (sha256 recorded beside the figure).
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.txt")
    if os.path.exists(tpath):
        import hashlib
        rec = {}
        for line in open(tpath):
            if "=" in line and not line.startswith("#"):
                k, v = line.split("=", 1)
                rec[k.strip()] = v.strip()
        src = os.path.join(ROOT, "paper_2306_00978_amd", "csrc", "awq_gemv_stream.hip")
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest() if os.path.exists(src) else ""
        if rec.get("decode_grouped_7b_layer_m1_kernel_source_sha256") == sha:
            try:
                traffic = int(rec["decode_grouped_7b_layer_m1_bytes_per_launch"])
                traffic_source = ("profiles/decode_grouped_7b_layer_m1_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE, "
                                  "WRITE_SIZE; awq_gemv_stream.hip sha256 " + sha[:12] + ")")
            except (KeyError, ValueError):
                traffic = None
        else:
            traffic_source = "profiles/traffic.txt was measured on another revision of awq_gemv_stream.hip: not reported"

    def gbs(b, ms):
        return round(b / (ms * 1e-3) / 1e9, 1)

    def pct(g):
        return round(100.0 * g / HBM_PEAK_GBS, 2)

    result = {
        "metric": "W4A16 decode GEMV HBM GB/s (Llama-2-7B layer shapes, M=1)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 weights, f16 activations, f32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: the 7 projections of a Llama-2-7B-shaped layer, M=1, group 128; "
                        f"one step = {L} distinct layers once each (cold cache: {L} x 105 MB of packed "
                        "weights, the linear stack of configs[4])",
            "launch": "one grouped launch (awq_w4a16_linear_multi) of the 7 projections per layer"
                      + (", replayed from a hipGraph" if use_graph else
                         (f", the launches of a step alternating over {n_streams} streams of default priority "
                          "(the layers of this workload are independent)" if n_streams > 1 else ", launched on the stream")),
            "streams": n_streams,
            "one_stream": {"what": "the same step with every launch on one stream, one after the other: the "
                                   "launch duration that `roofline` reports",
                           "ms_per_step": round(wall1_ms, 5), "GB/s": round(bytes_step / (wall1_ms * 1e-3) / 1e9, 1),
                           "pct_of_hbm_peak": round(100.0 * bytes_step / (wall1_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
                           "ms_per_step_by_events": {k: round(v, 5) for k, v in spread1.items()}},
            "launches_per_step": launches,
            "bytes_per_step": bytes_step,
            "bytes_per_launch": bytes_m1,
            "settle_ms": round(settle_ms, 1),
            "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
            "ms_per_step_by_events": {k: round(v, 5) for k, v in spread.items()},
            "read_only_reference": {"what": "awq_read_probe over one layer's packed arrays "
                                            f"({arena_bytes} B), one launch per layer, same cycling",
                                    "us": round(probe_us, 3), "GB/s": round(probe_gbs, 1),
                                    "value_over_reference": round(value / probe_gbs, 4)},
        },
        "roofline": {
            "kernel": "gemv_stream_kernel (grouped decode, 7 linears, M=1)",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": traffic_source,
            "avg_launch_us": round(kernel_us, 3),
            "avg_launch_us_measured": "HIP events around the timed steps with every launch on one stream; in the "
                                      "headline run two launches share the chip and a launch's duration is not "
                                      "the kernel's own",
            "algorithmic_bytes_per_launch": bytes_m1,
        },
    }

    result["config"]["quantize_pack_pass"] = {
        "what": f"configs[4]: one awq_quantize_pack call per matrix over all {L * len(shapes)} matrices, back to back",
        "ms_total": round(quant_ms, 3), "GB/s": round(quant_bytes / (quant_ms * 1e-3) / 1e9, 1),
        "pct_of_hbm_peak": round(100 * quant_bytes / (quant_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "one_call_per_layer": {
            "what": "awq_quantize_pack_multi: the seven matrices of a layer per launch",
            "ms_total": round(quant_layer_ms, 3), "GB/s": round(quant_bytes / (quant_layer_ms * 1e-3) / 1e9, 1),
            "pct_of_hbm_peak": round(100 * quant_bytes / (quant_layer_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2)}}

    # ---- the same layer the way the benchmark spec's call is named (one awq_w4a16_linear per projection) and
    # the way a decoder orders it (Q,K,V | o | gate,up | down: four dependent launches)
    msteps, mwarm = max(2, min(args.steps, 6)), max(1, min(args.warmup, 2))
    if "modes" in legs:
        w, e, n = time_decode("single", 1, msteps, mwarm, False)
        wg_, eg_, _ = time_decode("single", 1, msteps, mwarm, True)
        w2s, e2s, _ = time_decode("single", 1, msteps, mwarm, False, streams=max(2, args.streams))
        result["config"]["per_launch_mode"] = {
            "what": "seven awq_w4a16_linear calls per layer (gemv_kernel), same cycling",
            "launches_per_step": n,
            "on_the_stream": {"us_per_layer": round(e * 1e3 / L, 2), "GB/s": gbs(bytes_step, e), "pct_of_hbm_peak": pct(gbs(bytes_step, e))},
            "alternating_over_streams": {"streams": max(2, args.streams), "us_per_layer": round(e2s * 1e3 / L, 2),
                                         "GB/s": gbs(bytes_step, e2s), "pct_of_hbm_peak": pct(gbs(bytes_step, e2s))},
            "graph_replay": {"us_per_layer": round(eg_ * 1e3 / L, 2), "GB/s": gbs(bytes_step, eg_), "pct_of_hbm_peak": pct(gbs(bytes_step, eg_))}}
        # reference point, not part of the path: the same layer in fp16 through the vendor library (seven
        # torch.matmul calls per layer on unquantized weights of the same shapes, four layers cycled:
        # 1.6 GB, nothing stays cached) -- what Sec. 4.2 measures W4A16 against
        try:
            Wf = [[(torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32)
                    * workloads.SIGMA_7B).to(torch.float16) for _, N, K in shapes] for _ in range(4)]
            yf = [torch.empty((1, N), dtype=torch.float16, device=dev) for _, N, K in shapes]
            xf = [x_by_k[K][:1] for _, N, K in shapes]

            def dense_layer(l):
                for p in range(len(shapes)):
                    torch.matmul(xf[p], Wf[l & 3][p].t(), out=yf[p])
            for l in range(16):
                dense_layer(l)
            torch.cuda.synchronize()
            ef0, ef1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ef0.record()
            for l in range(64):
                dense_layer(l)
            ef1.record()
            torch.cuda.synchronize()
            usf = ef0.elapsed_time(ef1) / 64 * 1e3
            fp16_bytes = sum(2 * N * K + 2 * K + 2 * N for _, N, K in shapes)
            result["config"]["fp16_dense_reference"] = {
                "what": "the same layer unquantized: seven torch.matmul calls (fp16 weights, M=1) per layer, one stream",
                "us_per_layer": round(usf, 2), "fp16_bytes_per_layer": fp16_bytes,
                "GB/s_of_fp16_bytes": round(fp16_bytes / usf / 1e3, 1),
                "grouped_w4a16_launch_speedup": round(usf / kernel_us, 2)}
            del Wf, yf, xf
        except Exception as exc:                               # a reference only: never fails the run
            result["config"]["fp16_dense_reference"] = {"unavailable": str(exc)[:200]}
        torch.cuda.empty_cache()
        w, e, n = time_decode("fused", 1, msteps, mwarm, True)
        result["config"]["dependent_launch_mode"] = {
            "what": "Q,K,V in one launch | o | gate,up in one launch | down: the four launches a decoder's "
                    "data dependences allow, replayed from a graph",
            "launches_per_step": n, "us_per_layer": round(e * 1e3 / L, 2),
            "GB/s": gbs(bytes_step, e), "pct_of_hbm_peak": pct(gbs(bytes_step, e))}

        # the same four stages in ONE launch (awq_w4a16_linear_chain), now with real data dependences:
        # o reads v's output, gate and up read o's, down reads gate's
        ysc = outputs(1)
        sync = awq.chain_sync()

        def chain_for(l):
            w = layers[l]
            def lin(p, x):
                return dict(x=x, qweight=w[p][0], scales=w[p][1], zeros=w[p][2], y=ysc[p], N=shapes[p][1])
            x0 = x_by_k[4096][:1]
            return awq.prepare_linear_chain([[lin(0, x0), lin(1, x0), lin(2, x0)], [lin(3, ysc[2])],
                                             [lin(4, ysc[3]), lin(5, ysc[3])], [lin(6, ysc[4])]], sync)
        chains = [chain_for(l) for l in range(L)]
        for c in chains:
            c()
        torch.cuda.synchronize()
        assert int(sync.cpu().abs().sum()) == 0, "a chained launch gave up"
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(mwarm):
            for c in chains:
                c()
        e0.record()
        for _ in range(msteps):
            for c in chains:
                c()
        e1.record()
        torch.cuda.synchronize()
        ech = e0.elapsed_time(e1) / msteps
        assert int(sync.cpu().abs().sum()) == 0, "a chained launch gave up"
        result["config"]["dependent_chain_mode"] = {
            "what": "awq_w4a16_linear_chain: Q,K,V -> o -> gate,up -> down with their data dependences in ONE "
                    "launch per layer (resident workgroups, weights of the next stage requested before the wait)",
            "launches_per_step": L, "us_per_layer": round(ech * 1e3 / L, 2),
            "GB/s": gbs(bytes_step, ech), "pct_of_hbm_peak": pct(gbs(bytes_step, ech))}

    # ---- prefill GEMM, M = 2048, the three distinct shapes (the second half of the metric)
    if "prefill" in legs:
        M = workloads.PREFILL_M
        pre = {}
        tot_fl, tot_ms = 0, 0.0
        for p in (0, 4, 6):
            name, N, K = shapes[p]
            y = torch.empty((M, N), dtype=torch.float16, device=dev)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            e1.record()
            done, i = 0.0, 0
            while done < 15.0:                    # settle under this kernel's own load
                e0.record()
                for _ in range(10):
                    q, sc, zp = layers[i % L][p]
                    awq.awq_w4a16_linear(x_by_k[K], q, sc, zp, N, out=y)
                    i += 1
                e1.record()
                e1.synchronize()
                done += e0.elapsed_time(e1)
            reps = 60
            e0.record()
            for i in range(reps):
                q, sc, zp = layers[i % L][p]
                awq.awq_w4a16_linear(x_by_k[K], q, sc, zp, N, out=y)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            fl = workloads.flops(M, N, K)
            pre[f"{N}x{K}"] = {"us": round(ms * 1e3, 2), "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 1)}
            tot_fl += fl
            tot_ms += ms
            del y
        # reference point, not part of the path: the vendor library's dense fp16 product (torch.matmul,
        # weights already fp16, nothing to dequantize) on the same shapes, the same activations and
        # weights of the same distribution, several matrices cycled
        dense = {}
        d_fl, d_ms = 0, 0.0
        try:
            for p in (0, 4, 6):
                name, N, K = shapes[p]
                Wd = [(torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32)
                       * workloads.SIGMA_7B).to(torch.float16) for _ in range(8)]
                yd = torch.empty((M, N), dtype=torch.float16, device=dev)
                for i in range(100):
                    torch.matmul(x_by_k[K], Wd[i % 8].t(), out=yd)
                torch.cuda.synchronize()
                e0.record()
                for i in range(40):
                    torch.matmul(x_by_k[K], Wd[i % 8].t(), out=yd)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / 40
                fl = workloads.flops(M, N, K)
                dense[f"{N}x{K}"] = {"us": round(ms * 1e3, 2), "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 1)}
                d_fl += fl
                d_ms += ms
                del Wd, yd
            dense["TFLOP/s"] = round(d_fl / (d_ms * 1e-3) / 1e12, 1)
            dense["what"] = "torch.matmul fp16 (the vendor library's dense kernel) on the same shapes and activations"
        except Exception as exc:                               # a reference only: never fails the run
            dense = {"unavailable": str(exc)[:200]}
        torch.cuda.empty_cache()
        tf = tot_fl / (tot_ms * 1e-3) / 1e12
        result["roofline"]["prefill"] = {
            "kernel": "gemm_kernel (prefill, M=2048, configs[2]: 4096x4096, 11008x4096, 4096x11008)",
            "bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(tf / MFMA_F16_PEAK_TFLOPS, 4), "flops": tot_fl,
            "avg_launch_us": round(tot_ms * 1e3 / 3, 2), "shapes": pre,
            "dense_fp16_reference": dense}
        result["config"]["prefill_m2048_TFLOP/s"] = round(tf, 1)
        result["config"]["prefill_pct_of_mfma_peak"] = round(100 * tf / MFMA_F16_PEAK_TFLOPS, 2)
    result["config"]["clocks_after_run"] = clocks()

    if "extras" in legs:
        extras = {}
        xsteps, xwarm = max(2, min(args.steps, 6)), max(1, min(args.warmup, 2))   # passes: the side legs stay short
        xlaunch = 200                                                              # launches of the single-kernel legs
        w, e, n = time_decode("grouped", 1, 200, 20, use_graph, cycle=1)
        extras["decode_m1_grouped_warm_cache"] = {
            "note": "the same layer every launch: its 105 MB stay in the 256 MB Infinity Cache; not the headline",
            "us_per_launch": round(e * 1e3, 3), "GB/s": gbs(bytes_m1, e), "pct_of_hbm_peak": pct(gbs(bytes_m1, e))}
        w2, e2, n = time_decode("grouped", 1, xsteps, xwarm, not use_graph)
        extras["decode_m1_grouped_plain_stream" if use_graph else "decode_m1_grouped_graph_replay"] = {
            "us_per_launch": round(e2 * 1e3 / n, 3), "GB/s": gbs(bytes_step, e2)}
        span = min(8, L)
        if span > 1:
            w, e, n = time_decode("grouped", 1, xsteps, xwarm, use_graph, span=span)
            extras[f"decode_m1_grouped_{span}_layers_per_launch"] = {
                "note": "launch amortisation only: the benchmark models no data dependence between "
                        "linears, a real decoder has one between layers",
                "us_per_launch": round(e * 1e3 / n, 3), "GB/s": gbs(bytes_m1 * span * n, e),
                "pct_of_hbm_peak": pct(gbs(bytes_m1 * span * n, e))}
            # configs[4]: the whole stack token by token (all L layers once per token step)
            extras[f"decode_m1_full_stack_{L}_layers"] = {
                "bytes_per_token_step": bytes_step,
                "one_launch_per_layer": {"launches_per_token_step": launches,
                                         "ms_per_token_step": round(ev_ms, 4),
                                         "GB/s": gbs(bytes_step, ev_ms)},
                f"one_launch_per_{span}_layers": {"launches_per_token_step": n,
                                                  "ms_per_token_step": round(e, 4),
                                                  "GB/s": gbs(bytes_m1 * span * n, e)}}
        def on_streams(calls, reps, nst):
            """ms per call with the calls going alternately to nst streams of default priority."""
            cur = torch.cuda.current_stream()
            side = [torch.cuda.Stream() for _ in range(nst)]
            hs = [st.cuda_stream for st in side]
            a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for timed in (False, True):
                if timed:
                    a.record()
                for st in side:
                    st.wait_stream(cur)
                for i in range(reps):
                    calls[i % len(calls)](hs[i % nst])
                for st in side:
                    cur.wait_stream(st)
                if timed:
                    b_.record()
                torch.cuda.synchronize()
            return a.elapsed_time(b_) / reps

        for M in (4, 16):
            w, e, n = time_decode("grouped", M, xsteps, xwarm, use_graph)
            b = step_bytes(M) * n
            extras[f"decode_m{M}_grouped"] = {"us_per_layer": round(e * 1e3 / n, 3), "GB/s": gbs(b, e),
                                              "pct_of_hbm_peak": pct(gbs(b, e))}
            if n_streams > 1:
                w, e, n = time_decode("grouped", M, xsteps, xwarm, False, streams=n_streams)
                extras[f"decode_m{M}_grouped"]["alternating_over_streams"] = {
                    "streams": n_streams, "us_per_layer": round(e * 1e3 / n, 3), "GB/s": gbs(b, e),
                    "pct_of_hbm_peak": pct(gbs(b, e))}
        # INT3-g128 variant: the seven projections of a layer as seven launches of its decode
        # kernel, M = 1 (0.39453125 B per weight), L distinct layers cycled
        lay3 = []
        for l in range(min(L, 8)):
            packed = []
            for name, N, K in shapes:
                W = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32)
                     * workloads.SIGMA_7B).to(torch.float16)
                packed.append(awq.awq_quantize_pack_w3(W, s_by_k[K]))
                del W
            lay3.append(packed)
        ys3 = [torch.empty((1, N), dtype=torch.float16, device=dev) for _, N, K in shapes]
        def step3(l):
            for p, (name, N, K) in enumerate(shapes):
                awq.awq_w3a16_linear(x_by_k[K][:1], *lay3[l][p], N, out=ys3[p])
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step3(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graphs3 = []
        for l in range(len(lay3)):                      # replayed from graphs like the INT4 single launches
            g3 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g3):
                step3(l)
            graphs3.append(g3)
        for i in range(8):
            graphs3[i % len(graphs3)].replay()
        torch.cuda.synchronize()
        reps = 100
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            graphs3[i % len(graphs3)].replay()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        b3 = sum(sum(awq.awq_packed_sizes_w3(N, K)) + 2 * K + 2 * N for _, N, K in shapes)
        calls3 = [awq.prepare_linear_multi_w3([(x_by_k[K][:1], *lay3[l][p], ys3[p], N)
                                               for p, (_, N, K) in enumerate(shapes)]) for l in range(len(lay3))]
        for i in range(2 * len(calls3)):
            calls3[i % len(calls3)]()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(xlaunch):
            calls3[i % len(calls3)]()
        e1.record()
        torch.cuda.synchronize()
        msg = e0.elapsed_time(e1) / xlaunch
        b3g = sum(sum(awq.awq_packed_sizes_w3(N, K)) + 2 * K + 2 * N for _, N, K in shapes)
        extras["decode_m1_int3_grouped"] = {
            "bytes_per_step": b3g, "ms_per_step": round(msg, 5), "GB/s": gbs(b3g, msg),
            "pct_of_hbm_peak": round(100 * gbs(b3g, msg) / HBM_PEAK_GBS, 2),
            "time_vs_int4_grouped": round(msg * 1e3 / kernel_us, 3),
            "note": "one grouped launch of the 7 projections in the 3-bit layout (0.76 of the INT4 bytes)"}
        extras["decode_m1_int3_7_single_launches"] = {
            "bytes_per_step": b3, "ms_per_step": round(ms, 5), "GB/s": gbs(b3, ms),
            "pct_of_hbm_peak": round(100 * gbs(b3, ms) / HBM_PEAK_GBS, 2),
            "note": "compare decode_m1_7_single_launches (INT4): same launches, 0.76 of the bytes"}
        # 3-bit prefill, M = 2048, 4096 x 4096: re-pack into the 4-bit layout + the 4-bit GEMM
        Mp, (_, N3, K3) = workloads.PREFILL_M, shapes[0]
        y3 = torch.empty((Mp, N3), dtype=torch.float16, device=dev)
        ws3 = torch.empty(awq.load().awq_w3a16_prefill_workspace_bytes(N3, K3, 128), dtype=torch.uint8, device=dev)
        for _ in range(3):
            awq.awq_w3a16_linear(x_by_k[K3], *lay3[0][0], N3, out=y3, workspace=ws3)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(20):
            awq.awq_w3a16_linear(x_by_k[K3], *lay3[i % len(lay3)][0], N3, out=y3, workspace=ws3)
        e1.record()
        torch.cuda.synchronize()
        ms3 = e0.elapsed_time(e1) / 20
        extras["prefill_m2048_int3_4096x4096"] = {
            "us": round(ms3 * 1e3, 2), "TFLOP/s": round(workloads.flops(Mp, N3, K3) / (ms3 * 1e-3) / 1e12, 1),
            "note": "awq_w3a16_linear_prefill: codes re-packed into the 4-bit layout (one pass over the packed "
                    "weights), then the 4-bit prefill kernel"}
        del graphs3, lay3, y3, ws3

        # INT2-g64 variant: the seven projections of a layer in one launch of its decode kernel,
        # M = 1 (0.28515625 B per weight), L distinct layers cycled
        lay2 = []
        for l in range(min(L, 8)):
            packed = []
            for name, N, K in shapes:
                W = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32)
                     * workloads.SIGMA_7B).to(torch.float16)
                packed.append(awq.awq_quantize_pack_w2(W, s_by_k[K]))
                del W
            lay2.append(packed)
        ys2 = [torch.empty((1, N), dtype=torch.float16, device=dev) for _, N, K in shapes]
        calls2 = [awq.prepare_linear_multi_w2([(x_by_k[K][:1], *lay2[l][p], ys2[p], N)
                                               for p, (_, N, K) in enumerate(shapes)]) for l in range(len(lay2))]
        for i in range(2 * len(calls2)):
            calls2[i % len(calls2)]()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(xlaunch):
            calls2[i % len(calls2)]()
        e1.record()
        torch.cuda.synchronize()
        ms2 = e0.elapsed_time(e1) / xlaunch
        b2g = sum(sum(awq.awq_packed_sizes_w2(N, K)) + 2 * K + 2 * N for _, N, K in shapes)
        extras["decode_m1_int2_g64_grouped"] = {
            "bytes_per_step": b2g, "ms_per_step": round(ms2, 5), "GB/s": gbs(b2g, ms2),
            "pct_of_hbm_peak": round(100 * gbs(b2g, ms2) / HBM_PEAK_GBS, 2),
            "time_vs_int4_grouped": round(ms2 * 1e3 / kernel_us, 3),
            "note": "one launch of the 7 projections in the 2-bit layout, group size 64 (0.55 of the INT4 bytes)"}
        del lay2, calls2

        # configs[3]: the seven projections of a Llama-2-70B-shaped layer (444.5 MB per launch), M = 1
        # and 8, one grouped launch per step, two distinct layers cycled
        shapes70 = workloads.LLAMA2_70B_LAYER
        # inputs by the recipe of configs[3]: 1 % outlier channels x 20, s from 64 calibration rows per
        # distinct input width, weights quantized with that s, activations divided by it
        s70, x70 = {}, {}
        for K70 in (8192, 28672):
            out70 = workloads.outlier_channels(K70, 3, 0, 0)
            cal70 = workloads.activations(workloads.CALIB_TOKENS, K70, 3, 0, 0, workloads.ROLE_CALIB, out70)
            s70[K70] = awq.awq_act_scale(torch.from_numpy(cal70).to(dev), 0.5)
            xr = workloads.activations(8, K70, 3, 0, 0, workloads.ROLE_X, out70)
            x70[K70] = awq.awq_apply_inv_scale(torch.from_numpy(xr).to(dev), s70[K70])
        lay70 = []
        for l in range(2):
            packed = []
            for name, N, K in shapes70:
                W = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32)
                     * workloads.SIGMA_70B).to(torch.float16)
                packed.append(awq.awq_quantize_pack(W, s70[K]))
                del W
            lay70.append(packed)
        for M70 in (1, 8):
            ys70 = [torch.empty((M70, N), dtype=torch.float16, device=dev) for _, N, K in shapes70]
            calls70 = [awq.prepare_linear_multi([(x70[K][:M70], *lay70[l][p], ys70[p], N)
                                                 for p, (_, N, K) in enumerate(shapes70)]) for l in range(2)]
            for i in range(6):
                calls70[i % 2]()
            torch.cuda.synchronize()
            reps = 40
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(reps):
                calls70[i % 2]()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            b70 = sum(workloads.algorithmic_bytes(M70, N, K) for _, N, K in shapes70)
            extras[f"decode_m{M70}_llama70b_layer_grouped"] = {
                "bytes_per_launch": b70, "ms_per_launch": round(ms, 5), "GB/s": gbs(b70, ms),
                "pct_of_hbm_peak": round(100 * gbs(b70, ms) / HBM_PEAK_GBS, 2)}
            if n_streams > 1:
                ms2s = on_streams(calls70, reps, n_streams)
                extras[f"decode_m{M70}_llama70b_layer_grouped"]["alternating_over_streams"] = {
                    "streams": n_streams, "ms_per_launch": round(ms2s, 5), "GB/s": gbs(b70, ms2s),
                    "pct_of_hbm_peak": round(100 * gbs(b70, ms2s) / HBM_PEAK_GBS, 2)}
        del lay70

        M = workloads.PREFILL_M
        # a short prefill: 64 tokens, 4096 x 4096 (decode kernels on blocks of 16 tokens, one grouped launch)
        x64 = x_by_k[4096][:64].contiguous()
        y64 = torch.empty((64, 4096), dtype=torch.float16, device=dev)
        for i in range(4):
            awq.awq_w4a16_linear(x64, *layers[i % L][0], 4096, out=y64)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(40):
            awq.awq_w4a16_linear(x64, *layers[i % L][0], 4096, out=y64)
        e1.record()
        torch.cuda.synchronize()
        ms64 = e0.elapsed_time(e1) / 40
        extras["prefill_m64_4096x4096"] = {"us": round(ms64 * 1e3, 2),
                                           "TFLOP/s": round(workloads.flops(64, 4096, 4096) / (ms64 * 1e-3) / 1e12, 1),
                                           "note": "17..128 tokens: blocks of 16 through the decode kernels"}
        # a prompt of 512 tokens, the three distinct shapes: the prefill kernel with K cut into ranges
        # (the workspace of awq_w4a16_linear), next to the same call without the workspace
        pre512 = {}
        for p in (0, 4, 6):
            name, N, K = shapes[p]
            x512 = x_by_k[K][:512].contiguous()
            y512 = torch.empty((512, N), dtype=torch.float16, device=dev)
            need = awq.awq_linear_workspace_bytes(512, N, K)
            us = []
            for ws in (torch.empty(max(need, 16), dtype=torch.uint8, device=dev), False):
                for i in range(4):
                    awq.awq_w4a16_linear(x512, *layers[i % L][p], N, out=y512, workspace=ws)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(40):
                    awq.awq_w4a16_linear(x512, *layers[i % L][p], N, out=y512, workspace=ws)
                e1.record()
                torch.cuda.synchronize()
                us.append(e0.elapsed_time(e1) / 40 * 1e3)
            pre512[f"{N}x{K}"] = {"k_ranges": max(1, need // (512 * N * 4)), "us": round(us[0], 2),
                                  "us_without_workspace": round(us[1], 2),
                                  "TFLOP/s": round(workloads.flops(512, N, K) / us[0] / 1e6, 1)}
            del x512, y512
        extras["prefill_m512"] = pre512
        # quantize with the clipping search (11 range ratios) on the three distinct shapes
        ratios = [1.0 - 0.05 * i for i in range(11)]
        cms, cbytes = 0.0, 0
        for p in (0, 4, 6):
            name, N, K = shapes[p]
            Wd = torch.from_numpy(W0[p]).to(dev)
            outc = awq.awq_quantize_pack_clip(Wd, s_by_k[K], ratios)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                awq.awq_quantize_pack_clip(Wd, s_by_k[K], ratios, out=outc)
            e1.record()
            torch.cuda.synchronize()
            cms += e0.elapsed_time(e1) / 5
            cbytes += 2 * N * K + sum(awq.awq_packed_sizes(N, K)) + 4 * K
            del Wd
        extras["quantize_pack_clip"] = {"ratios": len(ratios), "matrices": 3, "ms_total": round(cms, 3),
                                        "GB/s": round(cbytes / (cms * 1e-3) / 1e9, 1),
                                        "note": "arithmetic-bound: 11 trial quantizations per group"}
        # the same with the error measured on 64 calibration rows (matrix cores)
        ams = 0.0
        for p in (0, 4, 6):
            name, N, K = shapes[p]
            Wd = torch.from_numpy(W0[p]).to(dev)
            xs64 = awq.awq_apply_inv_scale(torch.from_numpy(calib_by_k[K]).to(dev), s_by_k[K])
            outc = awq.awq_quantize_pack_clip(Wd, s_by_k[K], ratios, xs=xs64)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(5):
                awq.awq_quantize_pack_clip(Wd, s_by_k[K], ratios, out=outc, xs=xs64)
            e1.record()
            torch.cuda.synchronize()
            ams += e0.elapsed_time(e1) / 5
            del Wd
        extras["quantize_pack_clip_on_64_rows"] = {"ratios": len(ratios), "matrices": 3, "ms_total": round(ams, 3)}

        # decode attention with rotary embedding and cache update, Llama-2-7B heads, 2048 positions
        Ha, Da, La = 32, 128, 2048
        kcs = [torch.randn((Ha, La, Da), generator=gen, device=dev).to(torch.float16) for _ in range(8)]
        vcs = [torch.randn((Ha, La, Da), generator=gen, device=dev).to(torch.float16) for _ in range(8)]
        qa, ka, va = (torch.randn((Ha, Da), generator=gen, device=dev).to(torch.float16) for _ in range(3))
        outa = torch.empty((Ha, Da), dtype=torch.float16, device=dev)
        wsa = torch.empty(awq.load().awq_decode_attention_workspace_bytes(Ha, Da, La), dtype=torch.uint8, device=dev)
        def att_pass():
            for i in range(8):
                awq.awq_decode_attention(qa, ka, va, kcs[i], vcs[i], La - 1, out=outa, workspace=wsa)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            att_pass()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        ga = torch.cuda.CUDAGraph()
        with torch.cuda.graph(ga):
            att_pass()
        ga.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(25):
            ga.replay()
        e1.record()
        torch.cuda.synchronize()
        msa = e0.elapsed_time(e1) / 200
        ba = 2 * Ha * La * Da * 2
        extras["decode_attention_32_heads_2048_positions"] = {
            "bytes_per_call": ba, "us": round(msa * 1e3, 2), "GB/s": gbs(ba, msa),
            "pct_of_hbm_peak": round(100 * gbs(ba, msa) / HBM_PEAK_GBS, 2),
            "note": "two launches (slices of the positions, merge) replayed from a graph; "
                    "8 cache sets cycled (268 MB)"}
        del ga, kcs, vcs

        # one token through the whole stack of decoder layers (no embedding, no lm_head): per layer
        # norm+1/s -> Q,K,V in one launch -> attention at position 2047 -> o -> residual ->
        # norm+1/s -> gate,up in one launch -> silu*mul -> down -> residual
        if L >= 2:
            kcl = [torch.randn((Ha, La, Da), generator=gen, device=dev).to(torch.float16) for _ in range(L)]
            vcl = [torch.randn((Ha, La, Da), generator=gen, device=dev).to(torch.float16) for _ in range(L)]
            gam = torch.ones(4096, dtype=torch.float16, device=dev)
            hid = torch.randn((1, 4096), generator=gen, device=dev).to(torch.float16)
            xs1 = torch.empty_like(hid)
            act = torch.empty((1, 11008), dtype=torch.float16, device=dev)
            yq, yk, yv, yo, yg, yu, yd = (torch.empty((1, N), dtype=torch.float16, device=dev)
                                          for _, N, K in shapes)
            layer_calls = []
            for l in range(L):
                w = layers[l]
                layer_calls.append((
                    awq.prepare_linear_multi([(xs1, *w[0], yq, 4096), (xs1, *w[1], yk, 4096),
                                              (xs1, *w[2], yv, 4096)]),
                    awq.prepare_linear(outa.view(1, 4096), *w[3], yo, 4096),
                    awq.prepare_linear_multi([(xs1, *w[4], yg, 11008), (xs1, *w[5], yu, 11008)]),
                    awq.prepare_linear(act, *w[6], yd, 4096)))

            def token_pass():
                for l in range(L):
                    qkv, o, gu, down = layer_calls[l]
                    awq.awq_rmsnorm_inv_scale(hid, gam, s_by_k[4096], out=xs1)
                    qkv()
                    awq.awq_decode_attention(yq.view(Ha, Da), yk.view(Ha, Da), yv.view(Ha, Da),
                                             kcl[l], vcl[l], La - 1, out=outa, workspace=wsa)
                    o()
                    hid.add_(yo)
                    awq.awq_rmsnorm_inv_scale(hid, gam, s_by_k[4096], out=xs1)
                    gu()
                    awq.awq_silu_mul(yg, yu, out=act)
                    down()
                    hid.add_(yd)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                token_pass()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            gt = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gt):
                token_pass()
            gt.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(20):
                hid.normal_(generator=gen)
                gt.replay()
            e1.record()
            torch.cuda.synchronize()
            mst = e0.elapsed_time(e1) / 20
            bt = L * (step_bytes(1) + ba)
            extras[f"token_step_{L}_decoder_layers_context_2048"] = {
                "ms_per_token": round(mst, 4), "us_per_layer": round(mst * 1e3 / L, 2),
                "tokens_per_s": round(1e3 / mst, 1), "GB/s": gbs(bt, mst),
                "finite": bool(torch.isfinite(hid.float()).all().item()),
                "note": "11 launches per layer replayed from one graph; the two residual additions are "
                        "torch element-wise kernels, every other step is this library's; embedding, "
                        "final norm and lm_head are not included"}
            # the same token step with the normalisations and residual additions inside the
            # linears' launches (awq_w4a16_linear_fused_multi): 7 launches per layer
            wnorm = (gam.float() / s_by_k[4096]).to(torch.float16)
            fused_calls = []
            for l in range(L):
                w = layers[l]
                def lin(x, p, y, N, **kw):
                    return dict(x=x, qweight=w[p][0], scales=w[p][1], zeros=w[p][2], y=y, N=N, **kw)
                fused_calls.append((
                    awq.prepare_linear_fused_multi([lin(hid, 0, yq, 4096, norm=wnorm), lin(hid, 1, yk, 4096, norm=wnorm),
                                                    lin(hid, 2, yv, 4096, norm=wnorm)]),
                    awq.prepare_linear_fused_multi([lin(outa.view(1, 4096), 3, hid, 4096, residual=hid)]),
                    awq.prepare_linear_fused_multi([lin(hid, 4, yg, 11008, norm=wnorm), lin(hid, 5, yu, 11008, norm=wnorm)]),
                    awq.prepare_linear_fused_multi([lin(act, 6, hid, 4096, residual=hid)])))

            def token_pass_fused():
                for l in range(L):
                    qkv, o, gu, down = fused_calls[l]
                    qkv()
                    awq.awq_decode_attention(yq.view(Ha, Da), yk.view(Ha, Da), yv.view(Ha, Da),
                                             kcl[l], vcl[l], La - 1, out=outa, workspace=wsa)
                    o()
                    gu()
                    awq.awq_silu_mul(yg, yu, out=act)
                    down()
            # both forms from the same hidden state: the results must agree to fp16 rounding
            h0 = torch.randn((1, 4096), generator=gen, device=dev).to(torch.float16)
            hid.copy_(h0)
            token_pass()
            h_plain = hid.float().clone()
            hid.copy_(h0)
            token_pass_fused()
            h_fused = hid.float().clone()
            torch.cuda.synchronize()
            agree = float((h_plain - h_fused).abs().max() / h_plain.abs().max())
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                token_pass_fused()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            gf = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gf):
                token_pass_fused()
            gf.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(20):
                hid.normal_(generator=gen)
                gf.replay()
            e1.record()
            torch.cuda.synchronize()
            msf = e0.elapsed_time(e1) / 20
            extras[f"token_step_{L}_decoder_layers_context_2048_fused_norm_residual"] = {
                "ms_per_token": round(msf, 4), "us_per_layer": round(msf * 1e3 / L, 2),
                "tokens_per_s": round(1e3 / msf, 1), "GB/s": gbs(bt, msf),
                "max_difference_from_unfused_over_max": agree,
                "note": "7 launches per layer: the RMS normalisations run in the prologue and the residual "
                        "additions in the epilogue of the linears' launches"}
            del gt, gf, kcl, vcl

        # scale search (Eq. 4-5): 20 grid points on one 4096 x 4096 linear with 2048 cached rows
        name, N, K = shapes[0]
        out = workloads.outlier_channels(K, 1, 0, 0)
        Xs = torch.from_numpy(workloads.activations(M, K, 1, 1, 0, workloads.ROLE_CALIB, out)).to(dev)
        Ws = torch.from_numpy(W0[0]).to(dev)
        alphas = [i / 20 for i in range(20)]
        need = awq.load().awq_search_scale_workspace_bytes(M, N, K, len(alphas), 128)
        wsp = torch.empty(need, dtype=torch.uint8, device=dev)
        awq.awq_search_scale(Ws, Xs, alphas, workspace=wsp)
        torch.cuda.synchronize()
        reps = 5
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            best, losses, s_best = awq.awq_search_scale(Ws, Xs, alphas, workspace=wsp)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        fl = (len(alphas) + 1) * workloads.flops(M, N, K)
        extras["search_scale"] = {"shape": f"{N}x{K}, T={M}, {len(alphas)} grid points", "ms": round(ms, 3),
                                  "alpha_best": alphas[int(best.item())],
                                  "loss_best_over_rtn": round(float(losses[int(best.item())] / losses[0]), 4),
                                  "TFLOP/s": round(fl / (ms * 1e-3) / 1e12, 1),
                                  "pct_of_mfma_peak": round(100 * fl / (ms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 2)}
        del wsp, Ws, Xs
        torch.cuda.empty_cache()

        # steps a0 and a0' at the calibration size of configs[4] (128 sequences x 512 tokens per distinct
        # layer input): s = mean|X|^0.5 and x / s, two buffers cycled (1 GB and more: nothing stays cached)
        prep = {}
        T4 = 128 * 512
        for Kc in (4096, 11008):
            Xc = [torch.randn((T4, Kc), device=dev, dtype=torch.float16) for _ in range(2)]
            sc_ = torch.empty(Kc, dtype=torch.float32, device=dev)
            yc = torch.empty_like(Xc[0])
            for name, fn, nbytes in (("act_scale", lambda i: awq.awq_act_scale(Xc[i & 1], 0.5, out=sc_), 2 * T4 * Kc),
                                     ("apply_inv_scale", lambda i: awq.awq_apply_inv_scale(Xc[i & 1], sc_, out=yc), 4 * T4 * Kc)):
                for i in range(4):
                    fn(i)
                torch.cuda.synchronize()
                e0.record()
                for i in range(10):
                    fn(i)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) / 10 * 1e3
                prep[f"{name}_{T4}x{Kc}"] = {"us": round(us, 1), "GB/s": round(nbytes / us / 1e3, 1),
                                             "pct_of_hbm_peak": round(100 * nbytes / us / 1e3 / HBM_PEAK_GBS, 2)}
            del Xc, yc
            torch.cuda.empty_cache()
        # the four distinct inputs of a decoder layer (q/k/v share one, o, gate/up share one: K = 4096; down:
        # K = 11008) in one awq_act_scale_multi call, two sets cycled
        sets = []
        for _ in range(2):
            Xl = [torch.randn((T4, Kc), device=dev, dtype=torch.float16) for Kc in (4096, 4096, 4096, 11008)]
            sets.append(awq.prepare_act_scale_multi(
                [(X, torch.empty(X.shape[1], dtype=torch.float32, device=dev)) for X in Xl], 0.5))
        for i in range(4):
            sets[i & 1]()
        torch.cuda.synchronize()
        e0.record()
        for i in range(10):
            sets[i & 1]()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 10 * 1e3
        nb = 2 * T4 * (3 * 4096 + 11008)
        prep["act_scale_multi_one_layer_4_inputs"] = {"us": round(us, 1), "GB/s": round(nb / us / 1e3, 1),
                                                      "pct_of_hbm_peak": round(100 * nb / us / 1e3 / HBM_PEAK_GBS, 2)}
        del sets, Xl
        torch.cuda.empty_cache()
        extras["calibration_steps_configs4_size"] = prep
        result["extras"] = extras

    if args.copy_probe:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        result["copy_probe"] = {"kernel": "torch elementwise add (vectorized_elementwise_kernel)",
                                "bytes_read": src.numel() * 4, "bytes_written": dst.numel() * 4, "launches": 5}

    if not args.skip_cpu:
        result["cpu_baseline"] = cpu_baseline(W0, calib_by_k, x_by_k, shapes)
    print(json.dumps(result), flush=True)


def cpu_baseline(W0, calib_by_k, x_by_k, shapes):
    """The oracle as it stands, on the host cores: one decode step (7 linears, M = 1) from the
    packed arrays (unpack -> dequantize -> matmul), repeated for a bounded time."""
    import numpy as np
    import oracle
    import workloads

    cores = len(os.sched_getaffinity(0))
    packed = []
    for p, (name, N, K) in enumerate(shapes):
        s = oracle.act_scale(calib_by_k[K], 0.5).astype(np.float32)
        c, sc, z = oracle.quantize(W0[p], s)
        packed.append(oracle.pack(c, sc, z))
    xs = {K: x_by_k[K][:1].cpu().numpy() for K in x_by_k}
    bytes_step = sum(workloads.algorithmic_bytes(1, N, K) for _, N, K in shapes)
    reps, t_total = 0, 0.0
    while reps < 2 or (t_total < 10.0 and reps < 200):
        t0 = time.perf_counter()
        for p, (name, N, K) in enumerate(shapes):
            c, sc, z = oracle.unpack(*packed[p], N, K)
            oracle.matmul(xs[K], oracle.dequant(c, sc, z))
        t_total += time.perf_counter() - t0
        reps += 1
    omp = int(os.environ.get("OMP_NUM_THREADS", cores))
    also = {}
    try:
        # quantize + pack of each distinct shape (all cores)
        dq = {}
        for p in (0, 4, 6):
            name, N, K = shapes[p]
            sK = oracle.act_scale(calib_by_k[K], 0.5).astype(np.float32)
            t0 = time.perf_counter()
            c, sc, z = oracle.quantize(W0[p], sK)
            oracle.pack(c, sc, z)
            tq = time.perf_counter() - t0
            also[f"quantize_pack_{N}x{K}_GB/s"] = round((2 * N * K + N * K * 0.51953125) / tq / 1e9, 3)
            also[f"quantize_pack_{N}x{K}_s"] = round(tq, 3)
            dq[p] = oracle.dequant(c, sc, z)
        # the linear on already dequantized weights at M = 1 and M = 16 per distinct shape (fp64 matmul)
        for p in (0, 4, 6):
            name, N, K = shapes[p]
            x16 = x_by_k[K][:16].cpu().numpy()
            for M in (1, 16):
                t0 = time.perf_counter()
                oracle.matmul(x16[:M], dq[p])
                also[f"matmul_m{M}_{N}x{K}_ms"] = round((time.perf_counter() - t0) * 1e3, 2)
        # configs[2] (M = 2048) and configs[4] (224 matrices, 128 steps): never run in full on the
        # host; measured sample x scale factor, labelled as extrapolated
        t64 = 0.0
        x64 = {K: x_by_k[K][:64].cpu().numpy() for K in x_by_k}
        for p in (0, 4, 6):
            t0 = time.perf_counter()
            oracle.matmul(x64[shapes[p][2]], dq[p])
            t64 += time.perf_counter() - t0
        also["configs2_prefill_m2048_three_shapes_s_extrapolated"] = round(t64 * 2048 / 64, 2)
        also["configs2_extrapolated_from"] = "64 of the 2048 rows per shape x 32"
        tq_layer = sum(also[f"quantize_pack_{shapes[p][1]}x{shapes[p][2]}_s"] * c for p, c in ((0, 4), (4, 2), (6, 1)))
        also["configs4_quantize_pack_224_matrices_s_extrapolated"] = round(tq_layer * 32, 1)
        also["configs4_decode_128_steps_s_extrapolated"] = round(t_total / reps * 32 * 128, 1)
        also["configs4_extrapolated_from"] = ("one layer's quantize_pack x 32; one layer's decode step (above) "
                                              "x 32 layers x 128 steps")
        del dq
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        t0 = time.perf_counter()
        for p, (name, N, K) in enumerate(shapes):
            c, sc, z = oracle.unpack(*packed[p], N, K)
            oracle.matmul(xs[K], oracle.dequant(c, sc, z))
        also["decode_step_one_thread_GB/s"] = round(bytes_step / (time.perf_counter() - t0) / 1e9, 3)
        gomp.omp_set_num_threads(min(cores, omp))
    except Exception as exc:
        also["error"] = type(exc).__name__
    return {
        "also": also,
        "value": round(bytes_step * reps / t_total / 1e9, 3),
        "unit": "GB/s",
        "cores": min(cores, omp),
        "kind": "oracle",
        "sample": f"{reps} decode steps (7 projections of layer 0, M=1): unpack (1 thread) + "
                  f"dequantize + fp64 matmul (OpenMP), {t_total:.1f} s of CPU time",
    }


if __name__ == "__main__":
    main()
