#!/usr/bin/env python3
"""Benchmark of the decode step's weight stream: 3.5-bit fused dequant-GEMV on Llama-2-7B-shaped layers, batch 1.

A "step" is one pass of the hot path over one decoder layer's seven linears (q, k, v, o 4096x4096; gate, up
11008x4096; down 4096x11008): seven iflow_qgemv launches that stream 96.5 MiB of packed 3.5-bit weights once.
Successive steps walk a ring of distinct layers (> 1 GiB of packed weights) so that no launch finds its
weights in the 256 MB Infinity Cache or in L2: the figure is an HBM figure.  Weights are seeded synthetic
Gaussians (sigma 0.02) quantized on the GPU by iflow_quantize before the timed region; activations are seeded
N(0,1) fp16.  Launches are captured once into a HIP graph (one graph = one trip round the ring) and replayed;
the timed region is bracketed by HIP events on the launch stream and by device synchronisation.

Prints ONE JSON line.  `value` = algorithmic bytes per step / time per step, in GB/s (weights incl. block
headers + activations + outputs).  `roofline` prices the GEMV kernel against 8 TB/s; `cpu_baseline` is the
CPU oracle timed on a bounded sample of the same workload on this host.
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

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
SIGMA = 0.02


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1600)
    ap.add_argument("--warmup", type=int, default=160)
    ap.add_argument("--ring", type=int, default=32, help="distinct layers in the weight ring (32 = a whole 7B-shaped stack, 3.0 GiB packed)")
    ap.add_argument("--format", default="Q3H_B64")
    ap.add_argument("--launches", type=int, default=1, choices=(1, 4, 7),
                    help="launches per layer: 7 = one per matrix; 4 = q,k,v in one iflow_qgemv_multi launch, o, gate+up in one, down")
    ap.add_argument("--layers-per-launch", type=int, default=32,
                    help="with --launches 1: chain this many layers into one launch (the next layer's q/k/v read down's output); "
                         "32 = the whole stack, one decode step's weight stream in one launch")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--context", type=int, default=0,
                    help="with --fused: also run iflow_attn_decode (32 heads of 128) over a cache of this many positions per layer, "
                         "between the q,k,v and the o launch - a whole decoder layer, position embedding aside")
    ap.add_argument("--fused", action="store_true",
                    help="with --launches 4: rms normalization, silu-gated input and residuals fused into the four launches of a layer "
                         "(iflow_qgemv_fused), each launch reading the previous one's output")
    ap.add_argument("--separate-gate", action="store_true",
                    help="with --fused: store gate and up and apply silu(gate)*up in front of the down product (iflow_qgemv_fused "
                         "with IFLOW_X_SILU_MUL) instead of producing the gated vector in the gate/up launch (iflow_qgemv_gated)")
    ap.add_argument("--large-shapes", action="store_true",
                    help="also time one and eight activation vectors on 70B-shaped matrices (8192x8192, 28672x8192, 8192x28672) in the "
                         "3.5-, 4- and 8-bit formats (other_paths.large_shapes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the context figures for batches > 1 and the cache-hot case")
    ap.add_argument("--steady-state", action="store_true",
                    help="instead of the decoder layers: one chained launch of four independent 98304 x 4096 products (a wavefront's "
                         "step loop runs 16 steps per phase: what the kernel streams when phases are long), with the clock the launch ran at")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies before the timed region (reference for HBM counters)")
    return ap.parse_args()


def algorithmic_bytes(rows, cols, bits_per_weight, batch=1):
    """What the method must move once: packed weights incl. headers, activations in, outputs out."""
    return rows * cols * bits_per_weight / 8.0 + 2.0 * batch * cols + 2.0 * batch * rows


def cpu_baseline(fmt_name: str, reps: int = 3):
    """The oracle, as it stands, on a bounded sample: one layer's seven linears (202 M weights), `reps` times."""
    import numpy as np
    from oracle import oracle
    from paper_2401_08294_amd import synth
    ofmt = oracle.FORMATS[fmt_name]
    bpw = oracle.packed_bytes(ofmt, 64, 64) * 8 / 4096.0
    threads = max(1, min(16, os.cpu_count() or 1))
    total_bytes, total_s, used = 0.0, 0.0, 1
    for i, (_, rows, cols) in enumerate(synth.LLAMA2_7B_LAYER):
        w = synth.weights(rows, cols, SIGMA, synth.BASE_SEED + 900 + i)
        x = synth.activations(1, cols, synth.BASE_SEED + 950 + i)
        q, s, o = oracle.quantize(ofmt, w)
        rec = oracle.pack_canonical(ofmt, q, s, o)
        del w, q
        for _ in range(reps):
            t0 = time.perf_counter()
            _, used = oracle.qgemm_canonical(ofmt, rec, rows, cols, x.view(np.uint16), threads=threads)
            total_s += time.perf_counter() - t0
            total_bytes += algorithmic_bytes(rows, cols, bpw)
    # the same oracle on one thread, one 4096 x 4096 matrix (context for the core count)
    _, rows, cols = synth.LLAMA2_7B_LAYER[0]
    w = synth.weights(rows, cols, SIGMA, synth.BASE_SEED + 900)
    x = synth.activations(1, cols, synth.BASE_SEED + 950)
    q, s, o = oracle.quantize(ofmt, w)
    rec = oracle.pack_canonical(ofmt, q, s, o)
    t0 = time.perf_counter()
    oracle.qgemm_canonical(ofmt, rec, rows, cols, x.view(np.uint16), threads=1)
    single = algorithmic_bytes(rows, cols, bpw) / (time.perf_counter() - t0) / 1e9
    return {"value": round(total_bytes / total_s / 1e9, 4), "unit": "GB/s", "cores": int(used), "host_cores": os.cpu_count(),
            "threads": int(used), "kind": "oracle",
            "single_thread_value": round(single, 4),
            "sample": f"unpack + dequantize + fp64 GEMV of one layer's seven linears, {reps} passes "
                      f"({total_bytes / 1e6:.0f} MB of packed weights in {total_s:.1f} s); the multiply is row-parallel "
                      f"over {used} threads, unpack and dequantize are serial"}


def log_environment(torch):
    """Device, clocks and software versions to stderr (the JSON line on stdout stays alone).  The clocks come from
    the driver's sysfs files: a process that holds the GPU starts no other program."""
    import glob
    p = torch.cuda.get_device_properties(0)
    print(f"[bench] device: {p.name}, {p.multi_processor_count} CUs, {p.total_memory / 2**30:.0f} GiB, "
          f"torch {torch.__version__}, HIP {getattr(torch.version, 'hip', None)}", file=sys.stderr)
    for dev in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        try:
            if open(dev + "/vendor").read().strip() != "0x1002":
                continue
            for name in ("pp_dpm_sclk", "pp_dpm_mclk", "power_dpm_force_performance_level"):
                try:
                    text = open(f"{dev}/{name}").read().split("\n")
                except OSError:
                    continue
                cur = [l.strip() for l in text if l.strip().endswith("*")] or [l.strip() for l in text if l.strip()][:1]
                print(f"[bench]   {dev.split('/')[4]} {name}: {' '.join(cur)}", file=sys.stderr)
        except OSError as e:              # sysfs may be hidden on the box
            print(f"[bench]   {dev}: {e}", file=sys.stderr)


def chain_clock_mhz(torch, iflow, ws):
    """The shader clock a chained launch ran at, from the stamps its first workgroup leaves in the workspace header (the
    shader clock counter and the 100 MHz counter at its start and its end, low words); the launch must have ended."""
    w = [int(v) & 0xFFFFFFFF for v in ws.view(torch.int32)[iflow.CHAIN_WS_CLOCKS:iflow.CHAIN_WS_CLOCKS + 4].cpu().tolist()]
    cycles, ticks = (w[2] - w[0]) & 0xFFFFFFFF, (w[3] - w[1]) & 0xFFFFFFFF
    return round(100.0 * cycles / ticks, 1) if ticks else None


def steady_state(torch, iflow, dev, fmt, format_name, gen):
    """One chained launch over four independent products of 98304 x 4096 (201 MB packed each in the 3.5-bit format; every
    wavefront runs 16 steps per phase, so phase entries and hand-overs are a few per cent): the rate of the step loop itself,
    and the shader clock during the launch.  Built with IFLOW_HIPCC_DEFINES=-DIFLOW_CHAIN_ABL=1 (loads only) or =2 (decode
    only) the same command times the two halves of the loop apart."""
    rows, cols, nph = 98304, 4096, 4
    n = iflow.packed_bytes(fmt, rows, cols)
    mats = []
    for _ in range(nph):
        w = torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * SIGMA
        pk = torch.empty(n, dtype=torch.uint8, device=dev)
        iflow.quantize(fmt, w, rows, cols, pk, n)
        mats.append(pk)
        del w
    x = torch.randn((cols,), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
    ys = [torch.empty((rows,), dtype=torch.float16, device=dev) for _ in range(nph)]
    phases = [(cols, x, [(mats[i], rows, ys[i])]) for i in range(nph)]
    wsb = iflow.qgemv_chain_workspace_bytes([rows] * nph)
    pb = iflow.qgemv_chain_plan_bytes(phases)
    ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    plan = torch.empty(pb, dtype=torch.uint8, device=dev)
    chain = iflow.qgemv_chain_plan(fmt, phases, plan, pb, ws, wsb)
    for _ in range(3):
        iflow.qgemv_chain_launch(chain)
    torch.cuda.synchronize()
    times = []
    for _ in range(7):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            iflow.qgemv_chain_launch(chain)
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) / 5)
    iflow.qgemv_chain_check(chain)
    us = sorted(times)[len(times) // 2] * 1e3
    gbps = n * nph / us / 1e3
    return {"steady_state": {"what": f"{format_name}, one chained launch of {nph} independent products of {rows} x {cols} "
                                     f"({n * nph / 1e6:.0f} MB packed), eager launches, median of 7 x 5",
                             "us_per_launch": round(us, 1), "GB/s": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
                             "shader_clock_mhz": chain_clock_mhz(torch, iflow, ws)}}


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); nothing was run", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2401_08294_amd import iflow, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    iflow.lib()
    dev = torch.device("cuda:0")
    fmt = iflow.FORMATS[args.format]
    bpw = iflow.BITS_PER_WEIGHT[fmt]
    shapes = synth.LLAMA2_7B_LAYER

    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 2)
    if args.steady_state:
        print(json.dumps(steady_state(torch, iflow, dev, fmt, args.format, gen)))
        return

    # ---- build the ring of quantized layers (untimed) --------------------------------------------------
    ring = []
    for layer in range(args.ring):
        mats = []
        for name, rows, cols in shapes:
            w = torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * SIGMA
            n = iflow.packed_bytes(fmt, rows, cols)
            packed = torch.empty(n, dtype=torch.uint8, device=dev)
            iflow.quantize(fmt, w, rows, cols, packed, n)
            mats.append((rows, cols, packed))
            del w
        ring.append(mats)
    xs = {cols: torch.randn((cols,), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
          for cols in {c for _, _, c in shapes}}
    ys = [torch.empty((rows,), dtype=torch.float16, device=dev) for _, rows, _ in shapes]
    torch.cuda.synchronize()

    if args.calibrate_copy:      # a plain copy of known size: 1 GiB read + 1 GiB written per launch (far beyond the caches)
        src = torch.ones(256 * 2**20, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            iflow.calibration_copy(src, dst, src.numel() * 4)
        torch.cuda.synchronize()
        del src, dst

    step_bytes = sum(algorithmic_bytes(r, c, bpw) for _, r, c in shapes)
    if args.launches != 1:
        args.layers_per_launch = 1

    stream = torch.cuda.Stream()
    raw = stream.cuda_stream

    # projections that read the same activation vector and may share a launch: (q, k, v) and (gate, up)
    groups = [[0, 1, 2], [3], [4, 5], [6]] if args.launches in (1, 4) else [[i] for i in range(len(shapes))]
    if args.launches == 1:       # chained launches: o reads q's output, gate/up read o's, down reads gate's, the next layer's q/k/v read down's
        assert args.format in iflow.FORMATS, "unknown format"
        args.layers_per_launch = max(1, min(args.layers_per_launch, args.ring))
        lpl = args.layers_per_launch
        # all outputs of the chain as views of one allocation
        per_layer = sum((r + 127) // 128 * 128 for _, r, _ in shapes)
        y_arena = torch.empty((lpl * per_layer,), dtype=torch.float16, device=dev)
        ys_l, cursor = [], 0
        for _ in range(lpl):
            row = []
            for _, r, _ in shapes:
                row.append(y_arena[cursor:cursor + r])
                cursor += (r + 127) // 128 * 128
            ys_l.append(row)
        ys = ys_l[0]
        if lpl > 1:                      # no norms between the products here: start small so that fp16 holds the growth
            xs[shapes[0][2]].mul_(2.0 ** -10)            # (each layer grows the values about 4.4-fold; the chain saturates harmlessly after that)
        chains = {}

    launch_count = [0]

    def chain_for(layer, count):
        """The compiled chain for `count` consecutive layers starting at ring position `layer` (compiled once, outside the timed region)."""
        key = (layer, count)
        if key not in chains:
            phases = []
            for l in range(count):
                m_l, y_l = ring[(layer + l) % args.ring], ys_l[l]
                x_l = [xs[shapes[0][2]] if l == 0 else ys_l[l - 1][6], y_l[0], y_l[3], y_l[4]]
                phases += [(m_l[g[0]][1], x_l[i], [(m_l[j][2], m_l[j][0], y_l[j]) for j in g]) for i, g in enumerate(groups)]
            ws_bytes = iflow.qgemv_chain_workspace_bytes([m[1] for ph in phases for m in ph[2]])
            plan_bytes = iflow.qgemv_chain_plan_bytes(phases)
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
            plan = torch.empty(plan_bytes, dtype=torch.uint8, device=dev)
            t0 = time.perf_counter()
            chain = iflow.qgemv_chain_plan(fmt, phases, plan, plan_bytes, ws, ws_bytes, stream=raw)
            chains[key] = (chain, plan, ws, time.perf_counter() - t0)
        return chains[key][0]

    def chain_launch(layer, count):
        """One launch for `count` consecutive layers starting at ring position `layer`."""
        iflow.qgemv_chain_launch(chain_for(layer, count), stream=raw)
        launch_count[0] += 1

    if args.fused:
        assert args.launches == 4, "--fused goes with --launches 4"
        hidden_state = xs[shapes[0][2]].clone()               # the residual stream, updated in place by the o and down launches
        gains = [(1.0 + 0.1 * torch.randn((shapes[0][2],), generator=gen, device=dev, dtype=torch.float32)).to(torch.float16) for _ in range(2)]
        attn_out = torch.empty_like(ys[0])
        if args.context > 0:                                  # a key/value cache per ring layer (never appended to: the lengths stay fixed)
            caches = [(torch.randn((32, args.context, 128), generator=gen, device=dev, dtype=torch.float32).to(torch.float16),
                       torch.randn((32, args.context, 128), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)) for _ in range(args.ring)]
            attn_ws_bytes = iflow.attn_decode_workspace_bytes(32)
            attn_ws = torch.empty((attn_ws_bytes,), dtype=torch.uint8, device=dev)

    def fused_step(layer):
        """One decoder layer in four launches: norm -> q,k,v | o + residual | norm -> silu(gate)*up | down + residual
        (--separate-gate: norm -> gate,up | silu(gate)*up -> down + residual).
        (q's output stands in for the attention output, which is not part of this library.)"""
        m = ring[layer]
        h = hidden_state
        iflow.qgemv_fused(fmt, [m[i][2] for i in (0, 1, 2)], [m[i][0] for i in (0, 1, 2)], m[0][1], h, [ys[0], ys[1], ys[2]],
                          iflow.X_RMS_GAIN, gains[0], 1e-5, stream=raw)
        o_in = ys[0]
        if args.context > 0:
            kc, vc = caches[layer]
            iflow.attn_decode(ys[0], kc, vc, 32, 32, 128, args.context, args.context, 128 ** -0.5, attn_out, attn_ws, attn_ws_bytes, stream=raw)
            o_in = attn_out
        iflow.qgemv_fused(fmt, [m[3][2]], [m[3][0]], m[3][1], o_in, [h], residual_list=[h], stream=raw)
        if args.separate_gate:
            iflow.qgemv_fused(fmt, [m[4][2], m[5][2]], [m[4][0], m[5][0]], m[4][1], h, [ys[4], ys[5]], iflow.X_RMS_GAIN, gains[1], 1e-5, stream=raw)
            iflow.qgemv_fused(fmt, [m[6][2]], [m[6][0]], m[6][1], ys[4], [h], iflow.X_SILU_MUL, ys[5], 0.0, residual_list=[h], stream=raw)
        else:
            iflow.qgemv_gated(fmt, m[4][2], m[5][2], m[4][0], m[4][1], h, ys[4], iflow.X_RMS_GAIN, gains[1], 1e-5, stream=raw)
            iflow.qgemv_fused(fmt, [m[6][2]], [m[6][0]], m[6][1], ys[4], [h], residual_list=[h], stream=raw)
        launch_count[0] += 4

    def one_step(layer):
        if args.fused:
            return fused_step(layer)
        mats = ring[layer]
        for g in groups:
            cols = mats[g[0]][1]
            if len(g) == 1:
                rows, _, packed = mats[g[0]]
                iflow.qgemv(fmt, packed, rows, cols, xs[cols], ys[g[0]], stream=raw)
            else:
                iflow.qgemv_multi(fmt, [mats[i][2] for i in g], [mats[i][0] for i in g], cols, xs[cols],
                                  [ys[i] for i in g], stream=raw)
            launch_count[0] += 1

    def advance(layer, budget):
        """Run at most `budget` steps (layers) starting at ring position `layer`; returns how many were run."""
        if args.launches == 1:
            count = min(args.layers_per_launch, budget)
            chain_launch(layer, count)
            return count
        one_step(layer)
        return 1

    graph = None
    graph_launches = 0
    with torch.cuda.stream(stream):
        layer = 0
        while layer < (args.ring if args.launches == 1 else min(2, args.ring)):      # load code objects (and compile every chain) before capture
            layer += advance(layer, args.ring - layer)
        stream.synchronize()
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            launch_count[0] = 0
            with torch.cuda.graph(graph, stream=stream):
                layer = 0
                while layer < args.ring:
                    layer += advance(layer, args.ring - layer)
            graph_launches = launch_count[0]

        def run(nsteps, start_layer=0):
            """Exactly nsteps steps: whole ring trips by graph replay, the rest by direct launches."""
            done, layer = 0, start_layer
            while done < nsteps:
                if graph is not None and layer == 0 and nsteps - done >= args.ring:
                    graph.replay()
                    launch_count[0] += graph_launches
                    done += args.ring
                else:
                    n = advance(layer, min(nsteps - done, args.ring - layer))
                    done += n
                    layer = (layer + n) % args.ring
            return layer

        # The timed region is repeated (eleven times when it is shorter than eight trips round the ring, else three times)
        # and the median is reported; the first,
        # untimed repeat also compiles every chain the region needs (iflow_qgemv_chain_plan stays outside the timing).
        repeats = 11 if args.steps < 8 * args.ring else 3
        # Untimed steps in front of every timed region: the --warmup steps, and never fewer than sixteen trips round the ring (12 ms)
        # (with a handful of steps the part has not reached its steady state: a 20-step region measured 26.3 us per step
        # after 5 warm-up steps and 24.9 after 64, 640 or 3200).  The line reports both numbers.
        settle = max(0, 16 * args.ring - args.warmup) if args.launches == 1 else 0
        region = None                                    # a timed region of several launches as one graph of its own: one host call
        if args.launches == 1:                           # instead of one per launch between the two events
            end = run(args.warmup, run(settle))
            launch_count[0] = 0
            run(args.steps, end)
            stream.synchronize()
            # (a region of one or two launches is issued directly: its launches then sit right behind the first event in the
            # stream, where a graph's submission leaves a gap of its own - 462-467 against 470-474 us for a 20-layer launch)
            if repeats > 1 and graph is not None and launch_count[0] > 2:
                region = torch.cuda.CUDAGraph()
                launch_count[0] = 0
                with torch.cuda.graph(region, stream=stream):
                    run_direct = graph
                    graph = None                         # (no replay of the ring's graph inside a capture: direct launches only)
                    run(args.steps, end)
                    graph = run_direct
                region_launches = launch_count[0]
                region.replay()
                stream.synchronize()
        times = []
        for rep_i in range(repeats):
            end = run(args.warmup, run(settle))
            stream.synchronize()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            launch_count[0] = 0
            if region is not None:
                region.replay()
                launch_count[0] = region_launches
            else:
                run(args.steps, end)
            e1.record(stream)
            e1.synchronize()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        ms = sorted(times)[len(times) // 2]

        # spread: every ring trip of a short extra pass timed on its own (the events cost a little, so this pass is
        # not the headline), and the attainable ceiling: a kernel that only reads the same packed weights
        spread = None
        if graph is not None:
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(41)]
            evs[0].record(stream)
            for i in range(40):
                graph.replay()
                evs[i + 1].record(stream)
            evs[-1].synchronize()
            per = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 / args.ring for i in range(40))
            spread = {"per_layer_us_min": round(per[0], 3), "per_layer_us_median": round(per[len(per) // 2], 3),
                      "per_layer_us_max": round(per[-1], 3), "ring_trips": 40}
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        def read_ring():
            for mats in ring:
                for _, _, packed in mats:
                    iflow.calibration_read(packed, packed.numel() // 16 * 16, sink, stream=raw)
        read_ring()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        r0.record(stream)
        for _ in range(10):
            read_ring()
        r1.record(stream)
        r1.synchronize()
        read_gbps = 10 * args.ring * sum(p.numel() // 16 * 16 for _, _, p in ring[0]) / (r0.elapsed_time(r1) * 1e-3) / 1e9
        big = torch.empty(2**30, dtype=torch.uint8, device=dev)          # and one launch over 1 GiB: the asymptote
        iflow.calibration_read(big, big.numel(), sink, stream=raw)
        r0.record(stream)
        for _ in range(5):
            iflow.calibration_read(big, big.numel(), sink, stream=raw)
        r1.record(stream)
        r1.synchronize()
        read_big_gbps = 5 * big.numel() / (r0.elapsed_time(r1) * 1e-3) / 1e9
        del big

        # context figures for the other paths of the library (never the headline): batches 2..16 and 512 over a ring of
        # the 16 distinct gate matrices (344 MiB packed, beyond the caches), and the small parity case that stays cache-hot
        other = None
        if not args.no_extras:
            gate = [mats[4] for mats in ring]
            g_rows, g_cols = gate[0][0], gate[0][1]
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

            def time_gemm(mats, rows, cols, batch, reps):
                X = torch.randn((batch, cols), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
                Y = torch.empty((batch, rows), dtype=torch.float16, device=dev)
                for _, _, packed in mats[:2]:
                    iflow.qgemm(fmt, packed, rows, cols, X, batch, Y, stream=raw)
                t0.record(stream)
                for _ in range(reps):
                    for _, _, packed in mats:
                        iflow.qgemm(fmt, packed, rows, cols, X, batch, Y, stream=raw)
                t1.record(stream)
                t1.synchronize()
                return t0.elapsed_time(t1) * 1e3 / (reps * len(mats))            # us per product

            other = {"what": f"{args.format}, {g_rows}x{g_cols}, ring of {len(gate)} matrices, eager launches, us per product", "batch": {}}
            for batch in (1, 2, 4, 8, 16):
                us = time_gemm(gate, g_rows, g_cols, batch, 12)
                nbytes = g_rows * g_cols * bpw / 8 + 2 * batch * (g_rows + g_cols)
                other["batch"][str(batch)] = {"us": round(us, 2), "GB/s": round(nbytes / us / 1e3, 1)}
            us = time_gemm(gate, g_rows, g_cols, 512, 4)
            tf = 2.0 * 512 * g_rows * g_cols / us / 1e6
            other["batch"]["512"] = {"us": round(us, 2), "TFLOP/s": round(tf, 1), "frac_of_f16_mfma_peak": round(tf / 2500.0, 4)}
            # decode-step attention over an fp16 key/value cache: 7B-shaped (32 heads, 32 kv heads) and 70B-shaped (64 / 8)
            other["attention_decode"] = {"what": "iflow_attn_decode, ring of caches beyond the on-chip caches, eager launches, us per call and "
                                                 "GB/s of key/value bytes; heads / key-value heads x head dimension", "cases": {}}
            # (7B: 32/32 x 128; 70B: 64/8 x 128; Falcon-40B-shaped: 128/8 x 64, sixteen query heads per key/value head; multi-query: 71/1 x 64)
            for n_heads, n_kv, hd, T in ((32, 32, 128, 1024), (32, 32, 128, 4096), (64, 8, 128, 4096), (128, 8, 64, 4096), (71, 1, 64, 16384)):
                kv_bytes = 2 * n_kv * T * hd * 2
                nring = max(4, min(32, (768 * 2**20) // kv_bytes))
                caches = [(torch.randn((n_kv, T, hd), generator=gen, device=dev, dtype=torch.float32).to(torch.float16),
                           torch.randn((n_kv, T, hd), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)) for _ in range(nring)]
                qv = torch.randn((n_heads, hd), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
                ov = torch.empty((n_heads, hd), dtype=torch.float16, device=dev)
                awb = iflow.attn_decode_workspace_bytes(n_heads)
                aws = torch.empty((awb,), dtype=torch.uint8, device=dev)
                for kc, vc in caches[:2]:
                    iflow.attn_decode(qv, kc, vc, n_heads, n_kv, hd, T, T, hd ** -0.5, ov, aws, awb, stream=raw)
                t0.record(stream)
                for _ in range(6):
                    for kc, vc in caches:
                        iflow.attn_decode(qv, kc, vc, n_heads, n_kv, hd, T, T, hd ** -0.5, ov, aws, awb, stream=raw)
                t1.record(stream)
                t1.synchronize()
                us = t0.elapsed_time(t1) * 1e3 / (6 * nring)
                other["attention_decode"]["cases"][f"{n_heads}/{n_kv} heads x {hd}, {T} positions"] = {"us": round(us, 2), "GB/s": round(kv_bytes / us / 1e3, 1)}
                del caches
            # a whole decode step per layer: normalization, gate and residuals fused into the four launches, attention over 1024
            # cached positions in between (HIP-graph replay over the ring; key/value bytes are not counted in the GB/s)
            if args.format == "Q3H_B64" and not args.fused:
                ctx = 1024
                hs = xs[shapes[0][2]].clone()
                gn = [(1.0 + 0.1 * torch.randn((shapes[0][2],), generator=gen, device=dev, dtype=torch.float32)).to(torch.float16) for _ in range(2)]
                ao = torch.empty_like(ys[0])
                kvs = [(torch.randn((32, ctx, 128), generator=gen, device=dev, dtype=torch.float32).to(torch.float16),
                        torch.randn((32, ctx, 128), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)) for _ in range(args.ring)]
                awb2 = iflow.attn_decode_workspace_bytes(32)
                aws2 = torch.empty((awb2,), dtype=torch.uint8, device=dev)

                def decode_layer(layer):
                    m = ring[layer]
                    iflow.qgemv_fused(fmt, [m[i][2] for i in (0, 1, 2)], [m[i][0] for i in (0, 1, 2)], m[0][1], hs, [ys[0], ys[1], ys[2]],
                                      iflow.X_RMS_GAIN, gn[0], 1e-5, stream=raw)
                    iflow.rope_append(ys[0], ys[1], ys[2], 32, 32, 128, ctx - 1, ctx, 10000.0, iflow.ROPE_HALVES, kvs[layer][0], kvs[layer][1],
                                      stream=raw)
                    iflow.attn_decode(ys[0], kvs[layer][0], kvs[layer][1], 32, 32, 128, ctx, ctx, 128 ** -0.5, ao, aws2, awb2, stream=raw)
                    iflow.qgemv_fused(fmt, [m[3][2]], [m[3][0]], m[3][1], ao, [hs], residual_list=[hs], stream=raw)
                    iflow.qgemv_gated(fmt, m[4][2], m[5][2], m[4][0], m[4][1], hs, ys[4], iflow.X_RMS_GAIN, gn[1], 1e-5, stream=raw)
                    iflow.qgemv_fused(fmt, [m[6][2]], [m[6][0]], m[6][1], ys[4], [hs], residual_list=[hs], stream=raw)

                for layer in range(2):
                    decode_layer(layer)
                stream.synchronize()
                dgraph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(dgraph, stream=stream):
                    for layer in range(args.ring):
                        decode_layer(layer)
                for _ in range(3):
                    dgraph.replay()
                t0.record(stream)
                for _ in range(20):
                    dgraph.replay()
                t1.record(stream)
                t1.synchronize()
                us_layer = t0.elapsed_time(t1) * 1e3 / (20 * args.ring)
                other["decode_step_with_attention"] = {
                    "what": "per decoder layer: rms-norm + q,k,v | rotary embedding + cache append | attention over 1024 cached positions "
                            "(32 heads) | o + residual | rms-norm + silu(gate)*up | down + residual: 4 fused launches + rope_append "
                            "+ attention, HIP-graph replay over the ring",
                    "us_per_layer": round(us_layer, 2), "weight_GB/s": round(step_bytes / us_layer / 1e3, 1),
                    "tokens_per_s_32_layers": round(1e6 / (32 * us_layer), 1)}
                # the same decode step with the layer's products and modules in ONE chained launch per layer:
                # [attention output] -> o + residual -> rms-norm + silu(gate)*up -> down + residual -> rms-norm + the NEXT layer's q,k,v;
                # per layer: rope_append, attention, one chained launch (HIP-graph replay over the ring)
                hid, ffn_rows = shapes[0][2], shapes[4][1]
                hsA, hsB = hs.clone(), torch.empty_like(hs)
                h1b = torch.empty_like(hs)
                ab = torch.empty((ffn_rows,), dtype=torch.float16, device=dev)
                qb, kb, vb = torch.empty_like(hs), torch.empty_like(hs), torch.empty_like(hs)
                layer_chains = []
                for layer in range(args.ring):
                    m, mn = ring[layer], ring[(layer + 1) % args.ring]
                    h_in, h_out = (hsA, hsB) if layer % 2 == 0 else (hsB, hsA)
                    phs = [(m[3][1], ao, [(m[3][2], m[3][0], h1b, h_in)], {}),
                           (m[4][1], h1b, [(m[4][2], m[4][0], ab), (m[5][2], m[5][0], None)],
                            {"x_op": iflow.X_RMS_GAIN, "aux": gn[1], "eps": 1e-5, "gated": True}),
                           (m[6][1], ab, [(m[6][2], m[6][0], h_out, h1b)], {}),
                           (mn[0][1], h_out, [(mn[0][2], mn[0][0], qb), (mn[1][2], mn[1][0], kb), (mn[2][2], mn[2][0], vb)],
                            {"x_op": iflow.X_RMS_GAIN, "aux": gn[0], "eps": 1e-5})]
                    wsb = iflow.qgemv_chain_workspace_bytes([mm[1] for ph in phs for mm in ph[2]])
                    plb = iflow.qgemv_chain_plan_bytes(phs)
                    wst = torch.empty(wsb, dtype=torch.uint8, device=dev)
                    plt = torch.empty(plb, dtype=torch.uint8, device=dev)
                    layer_chains.append((iflow.qgemv_chain_plan_fused(fmt, phs, plt, plb, wst, wsb, stream=raw), plt, wst))

                def decode_layer_chained(layer):
                    iflow.rope_append(qb, kb, vb, 32, 32, 128, ctx - 1, ctx, 10000.0, iflow.ROPE_HALVES, kvs[layer][0], kvs[layer][1], stream=raw)
                    iflow.attn_decode(qb, kvs[layer][0], kvs[layer][1], 32, 32, 128, ctx, ctx, 128 ** -0.5, ao, aws2, awb2, stream=raw)
                    iflow.qgemv_chain_launch(layer_chains[layer][0], stream=raw)

                m0 = ring[0]
                iflow.qgemv_fused(fmt, [m0[i][2] for i in (0, 1, 2)], [m0[i][0] for i in (0, 1, 2)], m0[0][1], hsA, [qb, kb, vb],
                                  iflow.X_RMS_GAIN, gn[0], 1e-5, stream=raw)      # the first layer's q,k,v
                for layer in range(2):
                    decode_layer_chained(layer)
                stream.synchronize()
                cgraph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(cgraph, stream=stream):
                    for layer in range(args.ring):
                        decode_layer_chained(layer)
                for _ in range(3):
                    cgraph.replay()
                t0.record(stream)
                for _ in range(20):
                    cgraph.replay()
                t1.record(stream)
                t1.synchronize()
                for ch, _, _ in layer_chains:
                    iflow.qgemv_chain_check(ch, stream=raw)
                us_layer_c = t0.elapsed_time(t1) * 1e3 / (20 * args.ring)
                other["decode_step_with_attention_chained"] = {
                    "what": "per decoder layer: rotary embedding + cache append | attention over 1024 cached positions (32 heads) | ONE chained "
                            "launch: o + residual -> rms-norm + silu(gate)*up -> down + residual -> rms-norm + the next layer's q,k,v "
                            "(iflow_qgemv_chain_plan_fused); HIP-graph replay over the ring",
                    "us_per_layer": round(us_layer_c, 2), "weight_GB/s": round(step_bytes / us_layer_c / 1e3, 1),
                    "tokens_per_s_32_layers": round(1e6 / (32 * us_layer_c), 1)}
                # and without the attention: the whole stack, modules included, in one launch (q's output stands in for the attention's)
                arena2 = torch.empty((args.ring * (5 * hid + ffn_rows + 6 * 128),), dtype=torch.float16, device=dev)
                cur2 = [0]

                def take2(nrows):
                    v = arena2[cur2[0]:cur2[0] + nrows]
                    cur2[0] += (nrows + 127) // 128 * 128
                    return v

                phs_all, hcur = [], hsA
                for layer in range(args.ring):
                    m = ring[layer]
                    q_l, k_l, v_l, h1_l, a_l, h2_l = take2(hid), take2(hid), take2(hid), take2(hid), take2(ffn_rows), take2(hid)
                    phs_all += [(m[0][1], hcur, [(m[0][2], m[0][0], q_l), (m[1][2], m[1][0], k_l), (m[2][2], m[2][0], v_l)],
                                 {"x_op": iflow.X_RMS_GAIN, "aux": gn[0], "eps": 1e-5}),
                                (m[3][1], q_l, [(m[3][2], m[3][0], h1_l, hcur)], {}),
                                (m[4][1], h1_l, [(m[4][2], m[4][0], a_l), (m[5][2], m[5][0], None)],
                                 {"x_op": iflow.X_RMS_GAIN, "aux": gn[1], "eps": 1e-5, "gated": True}),
                                (m[6][1], a_l, [(m[6][2], m[6][0], h2_l, h1_l)], {})]
                    hcur = h2_l
                wsb = iflow.qgemv_chain_workspace_bytes([mm[1] for ph in phs_all for mm in ph[2]])
                plb = iflow.qgemv_chain_plan_bytes(phs_all)
                wst = torch.empty(wsb, dtype=torch.uint8, device=dev)
                plt = torch.empty(plb, dtype=torch.uint8, device=dev)
                all_chain = iflow.qgemv_chain_plan_fused(fmt, phs_all, plt, plb, wst, wsb, stream=raw)
                for _ in range(2):
                    iflow.qgemv_chain_launch(all_chain, stream=raw)
                t0.record(stream)
                for _ in range(10):
                    iflow.qgemv_chain_launch(all_chain, stream=raw)
                t1.record(stream)
                t1.synchronize()
                iflow.qgemv_chain_check(all_chain, stream=raw)
                us_layer_f = t0.elapsed_time(t1) * 1e3 / (10 * args.ring)
                other["fused_stack_in_one_launch"] = {
                    "what": f"{args.ring} decoder layers in ONE chained launch with their modules (rms-norm + q,k,v | o + residual | rms-norm + "
                            "silu(gate)*up | down + residual; q's output stands in for the attention's), eager launches",
                    "us_per_layer": round(us_layer_f, 2), "weight_GB/s": round(step_bytes / us_layer_f / 1e3, 1),
                    "frac_of_hbm_peak": round(step_bytes / us_layer_f / 1e3 / HBM_PEAK_GBPS, 4)}
                # the whole decode step, attention included, in ONE launch (iflow_decode_stack_plan)
                names = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
                stack_layers = []
                for layer in range(args.ring):
                    ly = {n: ring[layer][i][2] for i, n in enumerate(names)}
                    ly.update(norm1=gn[0], norm2=gn[1], k_cache=kvs[layer][0], v_cache=kvs[layer][1])
                    stack_layers.append(ly)
                h_out_s = torch.empty_like(hs)
                stack_args = (fmt, hid, ffn_rows, 32, 32, ctx, 1e-5, 10000.0, iflow.ROPE_HALVES)
                sb, plb, wsb = iflow.decode_stack_sizes(iflow.decode_stack(*stack_args, n_layers=args.ring))
                scr = torch.empty((sb // 2,), dtype=torch.float16, device=dev)
                plt_s = torch.empty(plb, dtype=torch.uint8, device=dev)
                wst_s = torch.empty(wsb, dtype=torch.uint8, device=dev)
                stack = iflow.decode_stack_plan(iflow.decode_stack(*stack_args, layers=stack_layers, h_in=hsA, h_out=h_out_s, scratch=scr),
                                                plt_s, plb, wst_s, wsb, stream=raw)
                for _ in range(2):
                    iflow.decode_stack_launch(stack, ctx - 1, stream=raw)
                t0.record(stream)
                for _ in range(10):
                    iflow.decode_stack_launch(stack, ctx - 1, stream=raw)
                t1.record(stream)
                t1.synchronize()
                iflow.qgemv_chain_check(stack, stream=raw)
                us_layer_s = t0.elapsed_time(t1) * 1e3 / (10 * args.ring)
                other["decode_step_in_one_launch"] = {
                    "what": f"{args.ring} decoder layers of the decode step in ONE launch, attention included (rms-norm + q,k,v | rotary "
                            "embedding + cache append + attention over 1024 cached positions, 32 heads, as two phases | o + residual | "
                            "rms-norm + silu(gate)*up | down + residual), eager launches",
                    "us_per_layer": round(us_layer_s, 2), "weight_GB/s": round(step_bytes / us_layer_s / 1e3, 1),
                    "tokens_per_s_32_layers": round(1e6 / (32 * us_layer_s), 1)}
                # the same launch at other context lengths (the caches hold 1024 rows: positions below that)
                by_ctx = {}
                for pos in (0, 255, 511):
                    for _ in range(2):
                        iflow.decode_stack_launch(stack, pos, stream=raw)
                    t0.record(stream)
                    for _ in range(10):
                        iflow.decode_stack_launch(stack, pos, stream=raw)
                    t1.record(stream)
                    t1.synchronize()
                    by_ctx[str(pos + 1)] = round(t0.elapsed_time(t1) * 1e3 / (10 * args.ring), 2)
                iflow.qgemv_chain_check(stack, stream=raw)
                by_ctx[str(ctx)] = round(us_layer_s, 2)
                other["decode_step_in_one_launch"]["us_per_layer_by_cached_positions"] = by_ctx
                del kvs
            # the other block formats of Table 3 (and the 2-bit one) on the same matrix shape, 1 to 16 activation vectors:
            # copies of one packed matrix at 16 distinct addresses
            other["other_formats"] = {"what": f"{g_rows}x{g_cols}, ring of 16 packed copies, eager launches; per format and number of "
                                              "activation vectors: us per product, GB/s of packed bytes", "formats": {}}
            wg = torch.randn((g_rows, g_cols), generator=gen, device=dev, dtype=torch.float32) * SIGMA
            for oname in ("Q8_B64", "Q6_B64", "Q5_B64", "Q4_B64", "Q3_B32", "Q2_B32"):
                ofmt = iflow.FORMATS[oname]
                nb_o = iflow.packed_bytes(ofmt, g_rows, g_cols)
                first = torch.empty(nb_o, dtype=torch.uint8, device=dev)
                iflow.quantize(ofmt, wg, g_rows, g_cols, first, nb_o, stream=raw)
                copies = [first] + [first.clone() for _ in range(15)]
                per_batch = {}
                for ob in (1, 2, 4, 8, 16):
                    Xo = torch.randn((ob, g_cols), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
                    Yo = torch.empty((ob, g_rows), dtype=torch.float16, device=dev)
                    for pk in copies[:2]:
                        iflow.qgemm(ofmt, pk, g_rows, g_cols, Xo, ob, Yo, stream=raw)
                    t0.record(stream)
                    for _ in range(8):
                        for pk in copies:
                            iflow.qgemm(ofmt, pk, g_rows, g_cols, Xo, ob, Yo, stream=raw)
                    t1.record(stream)
                    t1.synchronize()
                    us = t0.elapsed_time(t1) * 1e3 / (8 * 16)
                    per_batch[str(ob)] = {"us": round(us, 2), "GB/s": round(nb_o / us / 1e3, 1)}
                other["other_formats"]["formats"][oname] = per_batch
                del copies, first
            del wg
            # config 3's other two formats, and the bit-plane formats, through the chained launch: 8 distinct 7B-shaped layers per format, one launch per
            # pass over them (every product reading its predecessor's output), eager launches of ~0.3 ms each
            if args.format == "Q3H_B64" and not args.fused:
                other["formats_chained"] = {"what": "q+k+v -> o -> gate+up -> down -> next layer's q+k+v ..., 8 distinct 7B-shaped layers in ONE chained "
                                                    "launch, eager; us per layer, GB/s of the format's algorithmic bytes, fraction of the HBM peak", "formats": {}}
                for oname in ("Q4_B64", "Q8_B64", "Q6_B64", "Q5_B64", "Q3_B32", "Q2_B32"):
                    ofmt = iflow.FORMATS[oname]
                    nl = 8
                    ring_o = []
                    for _ in range(nl):
                        mats_o = []
                        for _, rows, cols in shapes:
                            w = torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * SIGMA
                            nb_o = iflow.packed_bytes(ofmt, rows, cols)
                            pk = torch.empty(nb_o, dtype=torch.uint8, device=dev)
                            iflow.quantize(ofmt, w, rows, cols, pk, nb_o, stream=raw)
                            mats_o.append((rows, cols, pk))
                            del w
                        ring_o.append(mats_o)
                    layer_bytes = sum(m[2].numel() + 2 * m[1] + 2 * m[0] for m in ring_o[0])
                    per_l = sum((r + 127) // 128 * 128 for _, r, _ in shapes)
                    ya = torch.empty((nl * per_l,), dtype=torch.float16, device=dev)
                    yl, cur = [], 0
                    for _ in range(nl):
                        row = []
                        for _, r, _ in shapes:
                            row.append(ya[cur:cur + r])
                            cur += (r + 127) // 128 * 128
                        yl.append(row)
                    # (no norms between the products: start small so that fp16 holds the growth over eight layers)
                    x_first = (torch.randn((shapes[0][2],), generator=gen, device=dev, dtype=torch.float32) * 2.0 ** -10).to(torch.float16)
                    phs = []
                    for l in range(nl):
                        m_l, y_l = ring_o[l], yl[l]
                        x_l = [x_first if l == 0 else yl[l - 1][6], y_l[0], y_l[3], y_l[4]]
                        phs += [(m_l[g[0]][1], x_l[i], [(m_l[j][2], m_l[j][0], y_l[j]) for j in g]) for i, g in enumerate([[0, 1, 2], [3], [4, 5], [6]])]
                    wsb = iflow.qgemv_chain_workspace_bytes([m[1] for ph in phs for m in ph[2]])
                    plb = iflow.qgemv_chain_plan_bytes(phs)
                    wst = torch.empty(wsb, dtype=torch.uint8, device=dev)
                    plt = torch.empty(plb, dtype=torch.uint8, device=dev)
                    ch = iflow.qgemv_chain_plan(ofmt, phs, plt, plb, wst, wsb, stream=raw)
                    for _ in range(3):
                        iflow.qgemv_chain_launch(ch, stream=raw)
                    t0.record(stream)
                    for _ in range(20):
                        iflow.qgemv_chain_launch(ch, stream=raw)
                    t1.record(stream)
                    t1.synchronize()
                    iflow.qgemv_chain_check(ch, stream=raw)
                    us_l = t0.elapsed_time(t1) * 1e3 / (20 * nl)
                    other["formats_chained"]["formats"][oname] = {"us_per_layer": round(us_l, 2), "GB/s": round(layer_bytes / us_l / 1e3, 1),
                                                                  "frac_of_hbm_peak": round(layer_bytes / us_l / 1e3 / HBM_PEAK_GBPS, 4)}
                    del ring_o, phs, ch, wst, plt, ya
            # 70B-shaped matrices (one and eight activation vectors): launches long enough not to be bound by their own
            # start-up; copies of one packed matrix, at least 1.2 GB of them, replayed from a HIP graph
            if args.large_shapes:
                other["large_shapes"] = {"what": "70B-shaped matrices, sigma 0.015, copies of one packed matrix (>= 1.2 GB in all), HIP-graph "
                                             "replay; per format, shape and number of activation vectors: us per product, GB/s of packed "
                                             "bytes, fraction of the HBM peak", "formats": {}}
            for oname in (("Q3H_B64", "Q4_B64", "Q8_B64") if args.large_shapes else ()):
                ofmt = iflow.FORMATS[oname]
                per_shape = {}
                for l_rows, l_cols in ((8192, 8192), (28672, 8192), (8192, 28672)):
                    wl = torch.randn((l_rows, l_cols), generator=gen, device=dev, dtype=torch.float32) * 0.015
                    nb_l = iflow.packed_bytes(ofmt, l_rows, l_cols)
                    first = torch.empty(nb_l, dtype=torch.uint8, device=dev)
                    iflow.quantize(ofmt, wl, l_rows, l_cols, first, nb_l, stream=raw)
                    del wl
                    copies = [first] + [first.clone() for _ in range(max(1, int(1.2e9 // nb_l)))]
                    per_batch = {}
                    for ob in (1, 8):
                        Xl = torch.randn((ob, l_cols), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
                        Yl = torch.empty((ob, l_rows), dtype=torch.float16, device=dev)
                        for pk in copies[:2]:
                            iflow.qgemm(ofmt, pk, l_rows, l_cols, Xl, ob, Yl, stream=raw)
                        stream.synchronize()
                        lgraph = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(lgraph, stream=stream):
                            for pk in copies:
                                iflow.qgemm(ofmt, pk, l_rows, l_cols, Xl, ob, Yl, stream=raw)
                        lgraph.replay()
                        t0.record(stream)
                        for _ in range(6):
                            lgraph.replay()
                        t1.record(stream)
                        t1.synchronize()
                        us = t0.elapsed_time(t1) * 1e3 / (6 * len(copies))
                        per_batch[str(ob)] = {"us": round(us, 2), "GB/s": round(nb_l / us / 1e3, 1),
                                              "frac_of_hbm_peak": round(nb_l / us / 1e3 / HBM_PEAK_GBPS, 4)}
                        del lgraph
                    per_shape[f"{l_rows}x{l_cols}"] = per_batch
                    del copies, first
                other["large_shapes"]["formats"][oname] = per_shape
            w1 = torch.randn((1024, 1024), generator=gen, device=dev, dtype=torch.float32) * SIGMA
            n1 = iflow.packed_bytes(fmt, 1024, 1024)
            p1 = torch.empty(n1, dtype=torch.uint8, device=dev)
            iflow.quantize(fmt, w1, 1024, 1024, p1, n1)
            us = time_gemm([(1024, 1024, p1)], 1024, 1024, 1, 400)
            other["cache_hot_1024x1024_batch1"] = {"us": round(us, 2), "GB/s": round((n1 + 4096) / us / 1e3, 1),
                                                   "note": "0.5 MiB of codes, resident in cache: launch-bound, not an HBM figure"}

    ms_per_step = ms / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    launches_per_step = launch_count[0] / args.steps            # a chained launch covers several layers (steps)
    us_per_launch = ms_per_step * 1e3 / launches_per_step
    bytes_per_launch = step_bytes / launches_per_step
    achieved = bytes_per_launch / (us_per_launch * 1e-6) / 1e9

    # HBM bytes from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE, calibrated), if present.  The summary
    # gives bytes per LAYER of the profiled launch; `traffic` is that figure times the layers of this run's average launch,
    # so that traffic / algorithmic_bytes_per_launch is the measured ratio whatever --steps is.  The kernel-trace average
    # of the same profiled command is copied next to it (per layer), as a second source for the roofline fraction.
    traffic, trace_us_per_layer = None, None
    layers_per_launch_avg = 1.0 / launches_per_step
    tfile = os.path.join(ROOT, "profiles", "q3h_chain_7b_layers_hbm_traffic.txt" if args.launches == 1
                         else "q3h_gemv_7b_layer_hbm_traffic.txt" if args.launches == 4 else "none")
    kfile = os.path.join(ROOT, "profiles", "q3h_chain_7b_layers_kernel_stats.txt" if args.launches == 1 else "none")

    def summary_value(path, key):
        if args.format != "Q3H_B64" or not os.path.exists(path):
            return None
        for line in open(path):
            if line.startswith(key):
                try:
                    return float(line.split("=")[1].split()[0])
                except (ValueError, IndexError):
                    return None
        return None

    per_layer = summary_value(tfile, "hbm_bytes_per_layer")
    if per_layer is not None:
        traffic = int(per_layer * layers_per_launch_avg)
    trace_us_per_layer = summary_value(kfile, "kernel_us_per_layer")

    out = {
        "metric": "achieved HBM GB/s (% of peak) of 3.5-bit fused dequant-GEMV, 7B shapes, batch 1" if args.format == "Q3H_B64"
                  else f"achieved HBM GB/s (% of peak) of {args.format} fused dequant-GEMV, 7B shapes, batch 1 (context; the headline is the 3.5-bit format)",
        "value": round(value, 1), "unit": "GB/s", "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "untimed_settling_steps": settle, "ms_per_step": round(ms_per_step, 5), "timed_repeats": repeats,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 x u7-pair codes, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "llama2-7b decoder-layer linears (q,k,v,o 4096x4096; gate,up 11008x4096; down 4096x11008), "
                               f"{args.format}, batch 1, ring of {args.ring} distinct layers "
                               f"({args.ring * step_bytes / 2**30:.2f} GiB packed), "
                               + ("HIP-graph replay" if graph is not None else "eager launches")
                               + (f", median of {repeats} repeats of the timed region" if repeats > 1 else "")
                               + {1: f", 1 chained launch per {args.layers_per_launch} layer(s) (q+k+v -> o -> gate+up -> down -> next layer's q+k+v ..., "
                                     "each phase reading the previous one's output)",
                                  4: ", 4 launches per layer (q+k+v, o, gate+up, down)"
                                     + (", rms normalization, silu gate and residuals fused in, each launch reading the previous one's output" if args.fused else "")
                                     + (f", attention over {args.context} cached positions per layer in between (its {2 * 32 * args.context * 128 * 2} "
                                        "key/value bytes per layer are NOT counted in the value)" if args.fused and args.context > 0 else ""),
                                  7: ", 7 launches per layer"}[args.launches],
                   "format": args.format, "batch": 1, "bytes_per_step": int(step_bytes), "launches_per_step": round(launches_per_step, 4)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "frac_source": "HIP events on the launch stream around the timed region of this run (launch gaps included)",
                     "kernel": "iflow::q3h_gemv_kernel<1, 2, false|true, -1>", "avg_launch_us": round(us_per_launch, 3),
                     "layers_per_launch": round(layers_per_launch_avg, 4),
                     "algorithmic_bytes_per_launch": int(bytes_per_launch),
                     "kernel_trace_us_per_layer": trace_us_per_layer,
                     "frac_from_kernel_trace": (round(step_bytes / (trace_us_per_layer * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)
                                                if trace_us_per_layer else None),
                     "kernel_trace_source": "profiles/q3h_chain_7b_layers_kernel_stats.txt (rocprofv3 --kernel-trace --stats of this command)"
                                            if trace_us_per_layer else None},
    }
    out["spread"] = spread
    out["stream_read_ceiling"] = {"value": round(read_gbps, 1), "unit": "GB/s", "frac_of_peak": round(read_gbps / HBM_PEAK_GBPS, 4),
                                  "what": "iflow_calibration_read over the same packed matrices, one launch per matrix (7 per layer), eager",
                                  "one_launch_over_1GiB": round(read_big_gbps, 1)}
    out["other_paths"] = other
    log_environment(torch)
    if args.launches == 1:
        for chain, _, _, _ in chains.values():
            iflow.qgemv_chain_check(chain, stream=raw)         # raises if a wait inside a launch ever gave up
        out["roofline"]["kernel"] = f"iflow::chain_kernel<2, false, {fmt}, false>"
        # the clock the last launch of the longest chain ran at (the part lowers it under load: a launch's cycles are
        # what the kernel decides, its clock is the power management's)
        longest = max(chains, key=lambda k: k[1])
        out["roofline"]["shader_clock_mhz_during_launch"] = chain_clock_mhz(torch, iflow, chains[longest][2])
        out["config"]["chain_plans"] = {f"{k[1]} layers from ring position {k[0]}": {"plan_MB": round(v[1].numel() / 1e6, 1),
                                                                                      "plan_call_s": round(v[3], 2)} for k, v in chains.items()}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.format)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
