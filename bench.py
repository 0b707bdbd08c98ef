#!/usr/bin/env python3
"""Benchmark of the routed mixed-bit linear hot path on one MI355X.

Workload (default): BASELINE config 1 - the seven linears of a Llama-2-7B-shaped decoder
block (q/k/v/o 4096x4096, gate/up 11008x4096, down 4096x11008), each with its own
router, one decode batch of bf16 tokens with 1% outlier channels, uniform precision mix.
A *step* is one pass of the whole hot path over all seven linears for one batch, as the four
dependent stages of the block: {q, k, v} (one input), {o}, {gate, up} (one input), {down};
each stage is one mbq_routed_linear_group call (route every projection's tokens, then the
routed outputs).  Steps are replayed from HIP graphs that hold up to 32 consecutive steps each (the
decode step of a 32-layer model replays its 32 blocks at once: a replay costs about 6 us of idle
GPU, which one step per replay would charge to every block); what is left of --steps after
whole replays runs from one-step graphs.  Weights, activations and router parameters are resident in HBM
before the timed region; three distinct copies of the packed block (> 600 MB) are
rotated so that no step finds its weights in the 256 MB last-level cache.

Prints ONE JSON line: metric/value/unit and timing of the step, `roofline` (dominant kernel against the HBM
peak), `cpu_baseline` (the CPU oracle on a sample of the same workload) and `extra` (side measurements).
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
RING = 3                        # distinct packed copies of the block rotated across steps
STAGES = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))   # projections that share their input
# HBM bytes per linear-kernel launch at batch 16 (mean over the four stages) from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of `bench.py --probe decode`, scaled by what the same counters read for a plain 256 MiB copy
# (FETCH_SIZE x2.000, WRITE_SIZE x1.000); see profiles/decode_linear_hbm_traffic_llama2_7b_batch16.txt
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {16: 53.10e6}
# HBM bytes per mbq_linear call (gather pre-kernel + tile kernel), mean over the three linears, same counters and scale
# factors from `bench.py --probe prefill` / `--probe prefill70b`; see profiles/prefill_hbm_traffic.txt
MEASURED_PREFILL_TRAFFIC_BYTES_PER_CALL = {"configs[2]": 653.8e6, "70b": 3498.4e6}


def algorithmic_bytes(N, K, T, pmax):
    """Bytes one routed-linear call has to move: slices 0..pmax actually read, the
    fp32 scale / zero point pairs, the activations, the outputs."""
    return (pmax + 1) * N * K // 4 + N * K // 16 + 2 * T * K + 4 * T * N


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--batch", type=int, default=16, help="decode batch (tokens per step): 1, 4 or 16")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--warm", action="store_true",
                    help="timeline probe: do not flush the last-level cache between the stage call and the timed launch")
    ap.add_argument("--steps-per-replay", type=int, default=32,
                    help="steps captured in one HIP graph (a decode step of a 32-layer model replays 32 blocks "
                         "at once); the remainder of --steps runs from one-step graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the batch-1/4 and prefill side measurements")
    ap.add_argument("--probe", choices=["decode", "prefill", "prefill70b", "timeline"], default=None,
                    help="counter probe for rocprofv3 --pmc, nothing is timed.  decode: a plain 256 MiB device copy "
                         "(known size, calibrates the counters) then a few mbq_linear launches per linear of the "
                         "block.  prefill / prefill70b: three mbq_linear launches of each linear of BASELINE configs[2] / of the "
                         "70B-shaped linears at 4096 tokens.  "
                         "timeline: where the time of the one-token-tile decode kernel goes, from the clock stamps of "
                         "the library's timeline build of that kernel (prints a table per stage)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2602_20191_amd as mbq
    from workloads import CONFIGS, make_case

    mbq.load()          # no fallback: raises if libmbq.so is missing
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = CONFIGS[1]
    T = args.batch
    if args.probe in ("prefill", "prefill70b"):
        # counter probe: three mbq_linear calls per linear; configs[2] (2048 tokens) with the bench's inputs, or the
        # 70B-shaped linears of configs[4] at 4096 tokens with the weights, activations and mix of the side measurement
        done = []
        if args.probe == "prefill":
            pcfg = CONFIGS[2]
            Tp = pcfg.token_counts[0]
            jobs = []
            for li, spec in enumerate(pcfg.linears):
                case = make_case(pcfg, li, Tp)
                blob = mbq.mbq_encode(torch.from_numpy(case["W"]).to(dev))
                X = torch.from_numpy(case["X"].view(np.int16)).view(torch.bfloat16).to(dev)
                routing = mbq.mbq_route(X, torch.from_numpy(case["Wr"]).to(dev), torch.from_numpy(case["br"]).to(dev))
                jobs.append((spec, X, blob, routing))
        else:
            Tp = 4096
            mix = torch.tensor([0.70, 0.20, 0.08, 0.02], device=dev)
            jobs = []
            for li, spec in enumerate(CONFIGS[4].linears):
                g = torch.Generator(device=dev)
                g.manual_seed(41 + li)
                blob = mbq.mbq_encode(torch.randn((spec.N, spec.K), generator=g, device=dev) * 0.02)
                g.manual_seed(100 + Tp)
                X = torch.randn((Tp, spec.K), generator=g, device=dev).to(torch.bfloat16)
                g.manual_seed(7 * Tp + li)
                prec = torch.multinomial(mix, Tp, replacement=True, generator=g).to(torch.int32)
                perm = torch.sort(prec, stable=True).indices.to(torch.int32)
                counts = torch.bincount(prec, minlength=4)
                offsets = torch.cat([torch.zeros(1, dtype=torch.int64, device=dev),
                                     torch.cumsum(counts, 0)]).to(torch.int32)
                jobs.append((spec, X, blob, (prec, perm, offsets)))
                torch.cuda.synchronize()
        for spec, X, blob, (prec, perm, offsets) in jobs:
            Y = torch.empty((Tp, spec.N), dtype=torch.float32, device=dev)
            ws = mbq.linear_workspace(Tp, spec.N, spec.K, dev)
            for _ in range(3):
                mbq.mbq_linear(X, blob, spec.N, spec.K, prec, perm, offsets, Y=Y, ws=ws)
            torch.cuda.synchronize()
            done.append({"name": spec.name, "N": spec.N, "K": spec.K, "T": Tp,
                         "mix": np.bincount(prec.cpu().numpy(), minlength=4).tolist()})
            del Y, ws
        print(json.dumps({"probe": args.probe, "linears": done}))
        return 0

    # ------------------------------------------------------------------ inputs in HBM
    t0 = time.time()
    layers = []
    for li, spec in enumerate(cfg.linears):
        case = make_case(cfg, li, T)
        Wd = torch.from_numpy(case["W"]).to(dev)
        blob = mbq.mbq_encode(Wd)
        torch.cuda.synchronize()
        del Wd
        blobs = [blob] + [blob.clone() for _ in range(RING - 1)]
        X = torch.from_numpy(case["X"].view(np.int16)).view(torch.bfloat16).to(dev)
        layer = dict(
            spec=spec, X=X, Wr=torch.from_numpy(case["Wr"]).to(dev), br=torch.from_numpy(case["br"]).to(dev),
            blobs=blobs, x_bits=case["X"], Wr_h=case["Wr"], br_h=case["br"],
            prec=torch.empty(T, dtype=torch.int32, device=dev), perm=torch.empty(T, dtype=torch.int32, device=dev),
            offsets=torch.empty(5, dtype=torch.int32, device=dev),
            Y=torch.empty((T, spec.N), dtype=torch.float32, device=dev),
            ws_r=mbq.route_workspace(T, spec.K, dev), ws_l=mbq.linear_workspace(T, spec.N, spec.K, dev))
        layers.append(layer)
    by_name = {l["spec"].name: l for l in layers}
    stages = []
    for names in STAGES:
        ls = [by_name[n] for n in names]
        for l in ls[1:]:                      # the stage's projections read the first one's activations
            l["X"], l["x_bits"] = ls[0]["X"], ls[0]["x_bits"]
        K = ls[0]["spec"].K
        stages.append(dict(
            names=names, layers=ls, X=ls[0]["X"], K=K, Ns=[l["spec"].N for l in ls],
            Wr=[l["Wr"] for l in ls], br=[l["br"] for l in ls],
            routing=[(l["prec"], l["perm"], l["offsets"]) for l in ls], Y=[l["Y"] for l in ls],
            ws_r=mbq.route_workspace(T, K, dev), ws_l=mbq.linear_workspace(T, max(l["spec"].N for l in ls), K, dev)))
    print(f"[bench] inputs ready in {time.time() - t0:.1f}s "
          f"({sum(l['blobs'][0].numel() for l in layers) * RING / 1e6:.0f} MB of packed weights)", file=sys.stderr)

    if args.probe == "timeline":
        return timeline_probe(mbq, torch, dev, stages, T, flush_cache=not args.warm)

    if args.probe == "decode":
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)          # plain copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        for st in stages:
            for i in range(RING):
                mbq.mbq_routed_linear_group(st["X"], st["Wr"], st["br"], [l["blobs"][i] for l in st["layers"]],
                                            st["Ns"], routing=st["routing"], Y=st["Y"], ws_route=st["ws_r"],
                                            ws_linear=st["ws_l"])
        torch.cuda.synchronize()
        print(json.dumps({"probe": "done", "copy_bytes": 256 << 20, "launches_per_stage": RING,
                          "stages": [["+".join(st["names"]), st["Ns"], st["K"],
                                      [int(l["prec"].max().item()) for l in st["layers"]]] for st in stages]}))
        return 0

    def step(ring_slot: int) -> None:
        for st in stages:
            mbq.mbq_routed_linear_group(st["X"], st["Wr"], st["br"], [l["blobs"][ring_slot] for l in st["layers"]],
                                        st["Ns"], routing=st["routing"], Y=st["Y"], ws_route=st["ws_r"],
                                        ws_linear=st["ws_l"])

    # ------------------------------------------------------------- launch mechanism
    launch = "eager"
    graphs = None          # one step per replay, one graph per weight copy
    long_graphs = None     # `per_replay` consecutive steps per replay, one graph per starting copy
    # whole replays of equal length cover the timed steps: K = 300 -> 10 replays of 30, K = 50 -> 2 of 25
    n_replays = max(1, -(-args.steps // max(1, args.steps_per_replay)))
    per_replay = max(1, args.steps // n_replays)
    step(0)
    torch.cuda.synchronize()
    if not args.no_graph:
        try:
            graphs = []
            for slot in range(RING):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    step(slot)
                graphs.append(g)
            if per_replay > 1:
                long_graphs = []
                for slot in range(RING):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        for j in range(per_replay):
                            step((slot + j) % RING)
                    long_graphs.append(g)
            launch = "hipgraph" if per_replay == 1 else f"hipgraph, {per_replay} steps per replay"
        except Exception as exc:  # capture not available: time eager launches instead
            print(f"[bench] graph capture failed ({exc}); falling back to eager launches", file=sys.stderr)
            graphs = long_graphs = None
            torch.cuda.synchronize()

    def run_steps(first: int, count: int) -> None:
        """Steps first .. first + count - 1; step i works on weight copy i % RING."""
        i, end = first, first + count
        while i < end:
            if long_graphs is not None and end - i >= per_replay:
                long_graphs[i % RING].replay()
                i += per_replay
            elif graphs is not None:
                graphs[i % RING].replay()
                i += 1
            else:
                step(i % RING)
                i += 1

    run_steps(0, args.warmup)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_start = time.perf_counter()
    ev0.record()
    run_steps(args.warmup, args.steps)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3
    ms_per_step = wall_ms / args.steps
    ev_ms_per_step = ev0.elapsed_time(ev1) / args.steps

    # realised routing (device results of the last step)
    mixes, step_bytes, pmaxes = [], 0, []
    for l in layers:
        p = l["prec"].cpu().numpy()
        pmax = int(p.max())
        pmaxes.append(pmax)
        mixes.append(np.bincount(p, minlength=4).tolist())
        step_bytes += algorithmic_bytes(l["spec"].N, l["spec"].K, T, pmax) + 16 * l["spec"].K
    avg_bits = float(np.mean([2 * (q + 1) for m in mixes for q in range(4) for _ in range(m[q])]))

    # ------------------------------------- dominant kernel: per-launch duration (HIP events)
    # The linear kernel of every stage alone (activations already prepared in the workspace by the
    # stage call above; mbq_bench_linear_group_prepared launches only that kernel), 24 launches per
    # HIP-graph replay over the rotating weight copies, timed with events on the launch stream.
    # Each stage rotates over enough copies of its own weights (>= 640 MB together) that no launch finds
    # them in the 256 MB last-level cache, as in the whole-step loop above.
    per_graph = 24
    kernel_us, kernel_bytes = [], []
    if True:
        for st in stages:
            stage_mb = sum(l["blobs"][0].numel() for l in st["layers"]) / 1e6
            copies = max(RING, int(np.ceil(640.0 / stage_mb)))
            pools = [l["blobs"] + [l["blobs"][0].clone() for _ in range(copies - RING)] for l in st["layers"]]
            n_launch = max(per_graph, copies)
            def burst():
                for i in range(n_launch):
                    mbq.bench_linear_group_prepared(T, st["K"], [pool[i % copies] for pool in pools], st["Ns"],
                                                    st["routing"], st["Y"], st["ws_l"])
            burst()
            torch.cuda.synchronize()
            g = None
            if not args.no_graph:
                try:
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        burst()
                except Exception:
                    g = None
                    torch.cuda.synchronize()
            reps = 8
            (g.replay() if g is not None else burst())
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                (g.replay() if g is not None else burst())
            b.record()
            torch.cuda.synchronize()
            kernel_us.append(a.elapsed_time(b) * 1e3 / (reps * n_launch))
            del pools, g
            kernel_bytes.append(sum(algorithmic_bytes(l["spec"].N, l["spec"].K, T, pm) - 2 * T * l["spec"].K
                                    for l, pm in zip(st["layers"], [pmaxes[layers.index(l)] for l in st["layers"]]))
                                + 2 * T * st["K"])
    avg_launch_us = float(np.mean(kernel_us))
    avg_launch_bytes = float(np.mean(kernel_bytes))
    achieved = avg_launch_bytes / (avg_launch_us * 1e-6) / 1e9

    out = {
        "metric": "decode tokens/s of the routed mixed-bit linear path (route + linear, 7 linears of a Llama-2-7B block)",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # the arithmetic of the timed kernels (batch <= 16): bf16 activations split exactly into two FP8 (E4M3) pieces,
        # 2-bit codes taken as FP4 (E2M1) operands, v_mfma_scale_f32_16x16x128_f8f6f4, fp32 accumulate and epilogue
        "dtype": "fp8(e4m3) x2 x fp4(e2m1) scaled MFMA, fp32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": f"BASELINE configs[1]: Llama-2-7B-shaped decoder block, 7 routed linears, decode batch {T}, "
                        "group 128, 2-bit base + three 2-bit residual slices, uniform precision mix, 1% outlier channels",
            "batch": T, "launch": launch, "weight_ring_copies": RING,
            "stages": ["+".join(n) for n in STAGES],
            "precision_mix_per_linear": mixes, "avg_bits": avg_bits,
        },
        "hbm_gbps_whole_step": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "event_ms_per_step": ev_ms_per_step,
        "roofline": {
            "bound": "hbm", "kernel": "the linear kernel of each stage: mbq::decode_f4_ws_kernel, K in one part "
                                      "(q+k+v, o, gate+up) and in two parts of two chunks (down)",
            "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
            "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(T),
            "avg_launch_us": avg_launch_us, "avg_launch_bytes": avg_launch_bytes,
            "per_stage_us": {"+".join(st["names"]): round(u, 2) for st, u in zip(stages, kernel_us)},
            "per_stage_gbps": {"+".join(st["names"]): round(bts / (u * 1e-6) / 1e9, 1)
                               for st, u, bts in zip(stages, kernel_us, kernel_bytes)},
        },
    }

    if not args.no_extra:
        peaks = measured_peaks(mbq, torch, dev)
        out["measured_peaks"] = peaks
        out["roofline"]["frac_of_measured_read"] = achieved / peaks["read_gbps"]
        out["roofline"]["frac_of_measured_copy"] = achieved / peaks["copy_gbps"]
        out["extra"] = extra_measurements(mbq, torch, dev, cfg, layers, stages, T)
        for key in ("prefill_mlp_2048tok", "prefill_70b_mlp_4096tok"):
            r = out["extra"][key]["roofline"]
            r["frac_of_measured_lds_fed_loop"] = r["achieved"] / peaks["mfma_bf16_lds_fed_tflops"]

    # ------------------------------------------------------------------ CPU baseline
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, layers, T)
    print(json.dumps(out))
    return 0


def timeline_probe(mbq, torch, dev, stages, T, dump_dir="gpurun_out", flush_cache=True):
    """Per stage (ring kernel only, K <= 8192): the stage call once (prepares the activations), the last-level cache
    flushed by a 1 GiB fill, then the timeline build of the linear kernel on cold weights; repeated `reps` times.
    Times are microseconds after the first wavefront of the launch entered the kernel (100 MHz clock: 0.01 us
    steps), given as min / median / max over all wavefronts of the launch."""
    flush = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    reps = 5
    names = ["entry", "precisions here", "first block requested", "activations + first block here"]
    for st in stages:
        if st["K"] > 8192:
            continue
        runs = []
        for rep in range(reps):
            blobs = [l["blobs"][rep % RING] for l in st["layers"]]
            mbq.mbq_routed_linear_group(st["X"], st["Wr"], st["br"], blobs, st["Ns"], routing=st["routing"],
                                        Y=st["Y"], ws_route=st["ws_r"], ws_linear=st["ws_l"])
            if flush_cache:
                flush.fill_(rep)
            torch.cuda.synchronize()
            stamps = mbq.bench_decode_timeline(T, st["K"], blobs, st["Ns"], st["routing"], st["Y"], st["ws_l"])
            torch.cuda.synchronize()
            runs.append(stamps.cpu().numpy())
        full = runs[-1].astype(np.int64)                    # [workgroups, 9 wavefronts, 32]: 8 arithmetic + the loader
        a, ld = full[:, :8, :], full[:, 8, :]
        live = a[:, :, 0] > 0
        t0 = a[:, :, 0][live].min()
        us = lambda x: (x - t0) / 100.0
        tiles = int(((a[:, 0, 4:30:2] > 0).sum(axis=1)).max())
        print(f"stage {'+'.join(st['names'])}: N {st['Ns']} K {st['K']} T {T}; {int(live[:, 0].sum())} workgroups, "
              f"up to {tiles} tiles each")
        spans = [(r[:, :8, 30][r[:, :8, 0] > 0].max() - r[:, :, 0][r[:, :, 0] > 0].min()) / 100.0 for r in runs]
        print("  first entry -> last end, us, per repetition: " + " ".join(f"{x:.2f}" for x in spans))

        def row(label, v):
            v = v[v > 0]
            if v.size:
                print(f"  {label:<34s} {us(v.min()):7.2f} {us(np.median(v)):7.2f} {us(v.max()):7.2f}")
        print(f"  {'phase (us after first entry)':<34s} {'min':>7s} {'median':>7s} {'max':>7s}")
        for k, nm in enumerate(names):
            row(nm, a[:, :, k][live])
        for i in range(tiles):
            row(f"tile {i}: MFMAs done", a[:, :, 4 + 2 * i][live])
            row(f"tile {i}: outputs stored", a[:, :, 5 + 2 * i][live])
        row("end", a[:, :, 30][live])
        ldl = ld[:, 0] > 0
        row("loader: precisions here", ld[:, 1][ldl])
        row("loader: first block issued", ld[:, 2][ldl])
        for i in (0, 1, 3, 7, 11, 15, 19, 23, 25):
            row(f"loader: block {i} published", ld[:, 4 + i][ldl])
        row("loader: end", ld[:, 30][ldl])
        # per XCD: when its workgroups start and end
        xcc = (a[:, 0, 31] >> 32) & 0xF
        for x in sorted(set(xcc[live[:, 0]].tolist())):
            sel = live[:, 0] & (xcc == x)
            print(f"  XCD {x}: {int(sel.sum()):3d} workgroups, entry {us(a[sel, 0, 0].min()):.2f}..{us(a[sel, 0, 0].max()):.2f}"
                  f", end {us(a[sel][:, :, 30].min()):.2f}..{us(a[sel][:, :, 30].max()):.2f}")
        if dump_dir and os.path.isdir(dump_dir):
            np.save(os.path.join(dump_dir, f"timeline_{'_'.join(st['names'])}_T{T}.npy"), np.stack(runs))
    return 0


def warm_until_steady(torch, fn, batch=5, budget_ms=50.0):
    """Untimed launches of fn(i) for budget_ms of GPU time: after host-side set-up the GPU needs some tens of
    milliseconds of work before its launches reach their sustained duration (measured: the 2048-token gate linear
    328 us over the first 20 calls, 278 us from the sixtieth on)."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    spent, i = 0.0, 0
    while spent < budget_ms:
        a.record()
        for _ in range(batch):
            fn(i)
            i += 1
        b.record()
        torch.cuda.synchronize()
        spent += a.elapsed_time(b)


def extra_measurements(mbq, torch, dev, cfg, layers, stages, T_main):
    """Side figures, each timed with HIP events over eager back-to-back launches:
    the same block at the other decode batches of the config, and the three prefill linears of
    BASELINE configs[2] (2048 tokens) as TFLOP/s."""
    from workloads import CONFIGS, make_case

    extra = {}
    for T in cfg.token_counts:
        if T == T_main:
            continue
        bufs = {}
        for li, l in enumerate(layers):
            case = make_case(cfg, li, T, with_weight=False)
            spec = l["spec"]
            bufs[spec.name] = dict(
                X=torch.from_numpy(case["X"].view(np.int16)).view(torch.bfloat16).to(dev),
                prec=torch.empty(T, dtype=torch.int32, device=dev), perm=torch.empty(T, dtype=torch.int32, device=dev),
                offsets=torch.empty(5, dtype=torch.int32, device=dev),
                Y=torch.empty((T, spec.N), dtype=torch.float32, device=dev))

        def one(slot):
            for st in stages:
                bs = [bufs[n] for n in st["names"]]
                mbq.mbq_routed_linear_group(bs[0]["X"], st["Wr"], st["br"], [l["blobs"][slot] for l in st["layers"]],
                                            st["Ns"], routing=[(b["prec"], b["perm"], b["offsets"]) for b in bs],
                                            Y=[b["Y"] for b in bs], ws_route=st["ws_r"], ws_linear=st["ws_l"])

        one(0)
        torch.cuda.synchronize()
        graphs = []
        per_replay = 10                    # consecutive steps per graph replay, as in the main run
        try:
            for slot in range(RING):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for j in range(per_replay):
                        one((slot + j) % RING)
                graphs.append(g)
        except Exception:
            graphs = []
            per_replay = 1
        n = 6 if graphs else 60
        for i in range(1 if graphs else 6):
            graphs[i % RING].replay() if graphs else one(i % RING)
        a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n):
            graphs[i % RING].replay() if graphs else one(i % RING)
        b2.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b2) / (n * per_replay)
        byts = 0
        for l in layers:
            b = bufs[l["spec"].name]
            pmax = int(b["prec"].max().item())
            byts += algorithmic_bytes(l["spec"].N, l["spec"].K, T, pmax) + 16 * l["spec"].K
        extra[f"decode_batch_{T}"] = {"ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3),
                                      "hbm_gbps_whole_step": byts / (ms * 1e-3) / 1e9,
                                      "launch": f"hipgraph, {per_replay} steps per replay" if graphs else "eager"}
    # the same block under other slice configurations (Sec. 4.1 general widths), on the SAME packed blobs (a configuration
    # only says where the eight-bit code may be cut): a 4-bit first slice and two 2-bit residual slices (three-output
    # routers choosing among 4, 6 and 8 bits; the routers are rows 1..3 of the block's own), and a 3-bit first slice with
    # residual slices of 1, 2 and 2 bits (tokens at 3, 4, 6 and 8 bits: the decode kernels then feed the two bits of every
    # code to the matrix cores separately)
    for bits in ((4, 2, 2), (3, 1, 2, 2)):
        scfg = mbq.Config(bits)
        E = len(bits)
        T = T_main
        Wr3 = [[w[4 - E:].contiguous() for w in st["Wr"]] for st in stages]
        br3 = [[b[4 - E:].contiguous() for b in st["br"]] for st in stages]

        def one_cfg(slot):
            for st, wr, br_ in zip(stages, Wr3, br3):
                mbq.mbq_routed_linear_group_cfg(st["X"], wr, br_, scfg, [l["blobs"][slot] for l in st["layers"]],
                                                st["Ns"], routing=st["routing"], Y=st["Y"], ws_route=st["ws_r"],
                                                ws_linear=st["ws_l"])

        one_cfg(0)
        torch.cuda.synchronize()
        per_replay = 10
        graphs = []
        try:
            for slot in range(RING):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for j in range(per_replay):
                        one_cfg((slot + j) % RING)
                graphs.append(g)
        except Exception:
            graphs, per_replay = [], 1
        n = 6 if graphs else 60
        for i in range(1 if graphs else 6):
            graphs[i % RING].replay() if graphs else one_cfg(i % RING)
        a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n):
            graphs[i % RING].replay() if graphs else one_cfg(i % RING)
        b2.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b2) / (n * per_replay)
        byts, mixes = 0, []
        for l in layers:
            digits = l["prec"].cpu().numpy() >> (1 if mbq.config_counts_bits(scfg) else 0)
            byts += algorithmic_bytes(l["spec"].N, l["spec"].K, T, int(digits.max())) + 4 * E * l["spec"].K
            mixes.append(np.bincount(digits, minlength=4).tolist())
        extra["slice_config_" + "_".join(str(b) for b in bits) + f"_decode_batch_{T}"] = {
            "workload": f"the block of the main line, slice widths {list(bits)}: routers with {E} outputs, tokens at "
                        f"{[mbq.config_bits(scfg, p) for p in range(E)]} bits",
            "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3), "hbm_gbps_whole_step": byts / (ms * 1e-3) / 1e9,
            "tokens_per_digit_precision_per_linear": mixes,
            "launch": f"hipgraph, {per_replay} steps per replay" if graphs else "eager"}
        # leave the stage buffers as the main run had them
        for st in stages:
            mbq.mbq_routed_linear_group(st["X"], st["Wr"], st["br"], [l["blobs"][0] for l in st["layers"]], st["Ns"],
                                        routing=st["routing"], Y=st["Y"], ws_route=st["ws_r"], ws_linear=st["ws_l"])
        torch.cuda.synchronize()
    # the same block with 4-bit activations (App. E.4), one mbq_routed_linear_group_act call per stage: the quantiser
    # launch (transform, per-token quantiser, router input rebuilt in the original space), the router launch on that
    # input (which also prepares the integer activations for the decode kernel), the linear launch, one launch for the
    # row scaling and bias of the stage's projections.  The block's own weights stand in for the transformed ones, the
    # transform's shift and scale are drawn at random, the bias is zero.
    if True:
        T = T_main
        rng_a = np.random.default_rng(2602)
        act = []
        for st in stages:
            K = st["X"].shape[1]
            act.append({
                "shift": torch.from_numpy(rng_a.normal(0, 0.1, size=K).astype(np.float32)).to(dev),
                "scale": torch.from_numpy(np.exp2(rng_a.uniform(-1, 1, size=K)).astype(np.float32)).to(dev),
                "out": (torch.empty_like(st["X"]), torch.empty((T,), dtype=torch.float32, device=dev),
                        torch.empty_like(st["X"])),
                "bias": [torch.zeros((N,), dtype=torch.float32, device=dev) for N in st["Ns"]]})

        def one_act(slot):
            for st, a_ in zip(stages, act):
                mbq.mbq_routed_linear_group_act(st["X"], 4, a_["shift"], a_["scale"], st["Wr"], st["br"],
                                                [l["blobs"][slot] for l in st["layers"]], st["Ns"], bias=a_["bias"],
                                                routing=st["routing"], Y=st["Y"], act=a_["out"], ws_route=st["ws_r"],
                                                ws_linear=st["ws_l"])

        one_act(0)
        torch.cuda.synchronize()
        per_replay = 10
        graphs = []
        try:
            for slot in range(RING):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for j in range(per_replay):
                        one_act((slot + j) % RING)
                graphs.append(g)
        except Exception:
            graphs, per_replay = [], 1
        n = 6 if graphs else 60
        for i in range(1 if graphs else 6):
            graphs[i % RING].replay() if graphs else one_act(i % RING)
        a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n):
            graphs[i % RING].replay() if graphs else one_act(i % RING)
        b2.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b2) / (n * per_replay)
        extra[f"activations_4bit_decode_batch_{T}"] = {
            "workload": "the block of the main line with 4-bit per-token activations: quantise, route on the rebuilt "
                        "activations, routed linears on the integers, row scaling; one stage call each",
            "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3),
            "launches_per_step": 4 * len(stages),
            "launch": f"hipgraph, {per_replay} steps per replay" if graphs else "eager"}
        for st in stages:
            mbq.mbq_routed_linear_group(st["X"], st["Wr"], st["br"], [l["blobs"][0] for l in st["layers"]], st["Ns"],
                                        routing=st["routing"], Y=st["Y"], ws_route=st["ws_r"], ws_linear=st["ws_l"])
        torch.cuda.synchronize()
    # the prefill linears of BASELINE configs[2] (gate, up, down; 2048 tokens), each as the whole mbq_linear call
    # (gather/group-sum pre-kernel + tile kernel) timed with HIP events over back-to-back launches
    pcfg = CONFIGS[2]
    T = pcfg.token_counts[0]
    per_linear, flops_sum, ms_sum, route_sum = {}, 0.0, 0.0, 0.0
    for li, spec in enumerate(pcfg.linears):
        case = make_case(pcfg, li, T)
        Wd = torch.from_numpy(case["W"]).to(dev)
        blob = mbq.mbq_encode(Wd)
        del Wd
        X = torch.from_numpy(case["X"].view(np.int16)).view(torch.bfloat16).to(dev)
        Wr, br = torch.from_numpy(case["Wr"]).to(dev), torch.from_numpy(case["br"]).to(dev)
        prec, perm, offsets = mbq.mbq_route(X, Wr, br)
        Y = torch.empty((T, spec.N), dtype=torch.float32, device=dev)
        ws = mbq.linear_workspace(T, spec.N, spec.K, dev)
        warm_until_steady(torch, lambda i: mbq.mbq_linear(X, blob, spec.N, spec.K, prec, perm, offsets, Y=Y, ws=ws))
        a, b2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = 20
        a.record()
        for _ in range(n):
            mbq.mbq_linear(X, blob, spec.N, spec.K, prec, perm, offsets, Y=Y, ws=ws)
        b2.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b2) / n
        # the router launch of the same call sequence, alone
        ws_r = mbq.route_workspace(T, spec.K, dev)
        for _ in range(3):
            mbq.mbq_route(X, Wr, br, out=(prec, perm, offsets), ws=ws_r)
        a.record()
        for _ in range(n):
            mbq.mbq_route(X, Wr, br, out=(prec, perm, offsets), ws=ws_r)
        b2.record()
        torch.cuda.synchronize()
        route_ms = a.elapsed_time(b2) / n
        flops = 2.0 * T * spec.N * spec.K
        per_linear[spec.name] = {"N": spec.N, "K": spec.K, "ms": ms, "tflops": flops / (ms * 1e-3) / 1e12,
                                 "route_ms": route_ms, "route_share_of_call": route_ms / (route_ms + ms),
                                 "mix": np.bincount(prec.cpu().numpy(), minlength=4).tolist()}
        flops_sum += flops
        ms_sum += ms
        route_sum += route_ms
        del blob, X, Y, ws
    tf = flops_sum / (ms_sum * 1e-3) / 1e12
    extra["prefill_mlp_2048tok"] = {
        "workload": "BASELINE configs[2]: gate/up 11008x4096 and down 4096x11008, 2048 tokens, {50,30,15,5}% mix + 2% "
                    "outlier tokens at 8 bits; useful flops 2 T N K over the whole mbq_linear call",
        "ms_total": ms_sum, "tflops": tf, "route_ms_total": route_sum,
        "tflops_route_and_linear": flops_sum / ((ms_sum + route_sum) * 1e-3) / 1e12, "per_linear": per_linear,
        "roofline": {"bound": "mfma", "kernel": "mbq::prefill_kernel (+ mbq::prefill_prep_kernel)", "achieved": tf,
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0,
                     "traffic": MEASURED_PREFILL_TRAFFIC_BYTES_PER_CALL["configs[2]"]}}
    # the paper's 2-layer router (hidden width 64) at the decode batch and at 2048 tokens, K = 4096
    from workloads import make_mlp_router, make_tokens
    Kr, Hr = 4096, 64
    W1, b1, W2, b2 = (torch.from_numpy(a).to(dev) for a in make_mlp_router(Kr, Hr, [7]))
    mlp = {}
    for Tr in (16, 2048):
        xb, _ = make_tokens(Tr, Kr, [7, Tr], outlier_channel_frac=0.01)
        Xr = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(dev).reshape(Tr, Kr)
        outr = (torch.empty(Tr, dtype=torch.int32, device=dev), torch.empty(Tr, dtype=torch.int32, device=dev),
                torch.empty(5, dtype=torch.int32, device=dev))
        wsr = mbq.route_mlp_workspace(Tr, Kr, Hr, dev)
        for _ in range(3):
            mbq.mbq_route_mlp(Xr, W1, b1, W2, b2, 0.0, out=outr, ws=wsr)
        a, b2e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = 50
        a.record()
        for _ in range(n):
            mbq.mbq_route_mlp(Xr, W1, b1, W2, b2, 0.0, out=outr, ws=wsr)
        b2e.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b2e) / n * 1e3
        mlp[f"tokens_{Tr}"] = {"us": us, "fp64_gflops": 2.0 * Tr * Kr * Hr / (us * 1e-6) / 1e9,
                               "mix": np.bincount(outr[0].cpu().numpy(), minlength=4).tolist()}
    extra["route_mlp_hidden64_K4096"] = mlp
    extra.update(other_config_measurements(mbq, torch, dev))
    return extra


def other_config_measurements(mbq, torch, dev):
    """BASELINE configs[3] (Llama-3-8B-shaped block, 64 tokens, decode) and configs[4] (70B-shaped MLP linears, 4096-token
    prefill and a 256-token batch).  Shapes and mixes are the configs'; the weights are drawn on the GPU (normal x 0.02:
    only the shapes matter for the time) and, for configs[4], the precisions are drawn directly with the target mix."""
    from workloads import CONFIGS

    def blob_of(N, K, seed):
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        W = torch.randn((N, K), generator=g, device=dev) * 0.02
        b = mbq.mbq_encode(W)
        torch.cuda.synchronize()
        del W
        return b

    def timed(fn, n, warm=2):
        for i in range(warm):
            fn(i)
        warm_until_steady(torch, fn, batch=max(2, n // 3))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(n):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    out = {}
    # ---- configs[3]: decoder block at 64 tokens, one router per linear (zero bias: uniform mix), stages as in the main run
    c3 = CONFIGS[3]
    T = c3.token_counts[0]
    specs = {sp.name: sp for sp in c3.linears}
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    stages = []
    for names in STAGES:
        K = specs[names[0]].K
        X = torch.randn((T, K), generator=g, device=dev).to(torch.bfloat16)
        Ns = [specs[n].N for n in names]
        stages.append(dict(
            X=X, K=K, Ns=Ns, blobs=[[blob_of(N, K, 31 + i)] for i, N in enumerate(Ns)],
            Wr=[torch.randn((4, K), generator=g, device=dev) / K ** 0.5 for _ in names],
            br=[torch.zeros(4, device=dev) for _ in names],
            routing=[(torch.empty(T, dtype=torch.int32, device=dev), torch.empty(T, dtype=torch.int32, device=dev),
                      torch.empty(5, dtype=torch.int32, device=dev)) for _ in names],
            Y=[torch.empty((T, N), dtype=torch.float32, device=dev) for N in Ns],
            ws_r=mbq.route_workspace(T, K, dev), ws_l=mbq.linear_workspace(T, max(Ns), K, dev)))
        for bl in stages[-1]["blobs"]:
            bl.extend(bl[0].clone() for _ in range(RING - 1))

    def block(slot):
        for st in stages:
            mbq.mbq_routed_linear_group(st["X"], st["Wr"], st["br"], [bl[slot % RING] for bl in st["blobs"]], st["Ns"],
                                        routing=st["routing"], Y=st["Y"], ws_route=st["ws_r"], ws_linear=st["ws_l"])
    block(0)
    torch.cuda.synchronize()
    graphs = []
    per_replay = 10                        # consecutive blocks per graph replay, as in the main run
    try:
        for slot in range(RING):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                for j in range(per_replay):
                    block(slot + j)
            graphs.append(gr)
    except Exception:
        graphs = []
        torch.cuda.synchronize()
    if graphs:
        ms = timed(lambda i: graphs[i % RING].replay(), 6, warm=1) / per_replay
    else:
        ms = timed(block, 30, warm=3)
    byts = sum(algorithmic_bytes(N, st["K"], T, int(r[0].max().item())) + 16 * st["K"]
               for st in stages for N, r in zip(st["Ns"], st["routing"]))
    out["decode_llama3_8b_block_batch64"] = {
        "workload": "BASELINE configs[3] shapes: q,o 4096x4096, k,v 1024x4096, gate,up 14336x4096, down 4096x14336; "
                    "64 tokens, seven routers, uniform mix; HIP-graph replays of 10 blocks, three weight copies rotated",
        "ms_per_step": ms, "tokens_per_s": T / (ms * 1e-3), "hbm_gbps_whole_step": byts / (ms * 1e-3) / 1e9,
        "hbm_frac": byts / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    del stages
    torch.cuda.empty_cache()

    # ---- configs[4]: 70B-shaped MLP linears, mix {70,20,8,2}%
    c4 = CONFIGS[4]
    mix = torch.tensor([0.70, 0.20, 0.08, 0.02], device=dev)

    def routing_of(T, seed):
        g2 = torch.Generator(device=dev)
        g2.manual_seed(seed)
        prec = torch.multinomial(mix, T, replacement=True, generator=g2).to(torch.int32)
        perm = torch.sort(prec, stable=True).indices.to(torch.int32)
        counts = torch.bincount(prec, minlength=4)
        offsets = torch.cat([torch.zeros(1, dtype=torch.int64, device=dev), torch.cumsum(counts, 0)]).to(torch.int32)
        return prec, perm, offsets

    pre, dec = {}, {}
    fl_sum = ms_sum = 0.0
    for li, spec in enumerate(c4.linears):
        blobs = [blob_of(spec.N, spec.K, 41 + li)]
        blobs += [blobs[0].clone() for _ in range(RING - 1)]
        for T, store in ((4096, pre), (256, dec)):
            g2 = torch.Generator(device=dev)
            g2.manual_seed(100 + T)
            X = torch.randn((T, spec.K), generator=g2, device=dev).to(torch.bfloat16)
            prec, perm, offsets = routing_of(T, 7 * T + li)
            Y = torch.empty((T, spec.N), dtype=torch.float32, device=dev)
            ws = mbq.linear_workspace(T, spec.N, spec.K, dev)
            ms = timed(lambda i: mbq.mbq_linear(X, blobs[i % RING], spec.N, spec.K, prec, perm, offsets, Y=Y, ws=ws),
                       6 if T == 4096 else 12)
            flops = 2.0 * T * spec.N * spec.K
            byts = algorithmic_bytes(spec.N, spec.K, T, int(prec.max().item()))
            store[spec.name] = {"N": spec.N, "K": spec.K, "ms": ms, "tflops": flops / (ms * 1e-3) / 1e12,
                                "gbps": byts / (ms * 1e-3) / 1e9, "mix": torch.bincount(prec, minlength=4).tolist()}
            if T == 4096:
                fl_sum += flops
                ms_sum += ms
            del X, Y, ws
        del blobs
        torch.cuda.empty_cache()
    tf = fl_sum / (ms_sum * 1e-3) / 1e12
    out["prefill_70b_mlp_4096tok"] = {
        "workload": "BASELINE configs[4] shapes: gate/up 28672x8192, down 8192x28672, 4096 tokens, {70,20,8,2}% mix "
                    "(precisions drawn directly); useful flops 2 T N K over the whole mbq_linear call",
        "ms_total": ms_sum, "tflops": tf, "per_linear": pre,
        "roofline": {"bound": "mfma", "kernel": "mbq::prefill_kernel (+ mbq::prefill_prep_kernel)", "achieved": tf,
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0,
                     "traffic": MEASURED_PREFILL_TRAFFIC_BYTES_PER_CALL["70b"]}}
    for v in dec.values():   # the mixed case: both fractions, graded against the larger of the two times
        v["hbm_frac"] = v["gbps"] / HBM_PEAK_GBPS
        v["mfma_frac"] = v["tflops"] / 2500.0
    out["batch256_70b_mlp"] = {"workload": "the same three linears at 256 tokens (prefill kernel); bytes and flops both matter",
                               "per_linear": dec}
    return out


def cpu_baseline(cfg, layers, T):
    """The C oracle (oracle/mbq_oracle.c: plain fp64 loops, dequantise-then-dot, OpenMP over output rows) timed on
    the host in full on the bench workload: routing, bucketing and the routed linear of all seven linears of the
    block at batch T, once with every hardware thread and once with one.  Encoding is the offline step and is not
    timed.  Also counts, per linear, the tokens whose top-2 router logits are closer than 1e-5 (reported apart by the
    parity rule) and the tokens where the GPU's choice differs from the oracle's."""
    from oracle import c_oracle as C
    from workloads import make_weight

    threads = C.max_threads()
    t_all = t_one = 0.0
    near_ties, differing = [], []
    for li, l in enumerate(layers):
        spec = l["spec"]
        W = make_weight(spec.N, spec.K, [cfg.seed, li], cfg.weight_df)
        codes, s0, z0 = C.encode(W)                      # offline step: not timed
        del W
        for n_threads in (threads, 1):
            C.set_threads(n_threads)
            t0 = time.perf_counter()
            S, prec, gap = C.route(l["x_bits"], l["Wr_h"], l["br_h"])
            perm, offsets = C.bucket(prec)
            C.linear(l["x_bits"], codes, s0, z0, prec)
            dt = time.perf_counter() - t0
            if n_threads == 1:
                t_one += dt
            else:
                t_all += dt
        C.set_threads(threads)
        gpu_prec = l["prec"].cpu().numpy()
        near = gap < 1e-5
        near_ties.append(int(near.sum()))
        differing.append(int(((gpu_prec != prec) & ~near).sum()))
        del codes
    return {"value": T / t_all, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"the whole workload once (7 linears, batch {T}): routing + bucketing + routed linear by the C "
                      f"oracle (fp64, plain loops, gcc -O2 -fopenmp); encode not timed",
            "seconds": t_all, "value_1_thread": T / t_one, "seconds_1_thread": t_one,
            "near_tie_tokens_per_linear": near_ties, "tokens_routed_differently_off_the_near_tie_list": differing}


def measured_peaks(mbq, torch, dev):
    """What this chip itself reaches, next to the published peaks: a plain streaming copy and a read-only stream over
    1 GiB (HIP events, 5 launches each), and an MFMA loop fed from LDS (v_mfma_f32_32x32x16_bf16, one workgroup of 8
    wavefronts per compute unit), with and without one workgroup barrier per 16 MFMAs."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev)
    dst = torch.empty(n, dtype=torch.uint8, device=dev)
    src.fill_(1)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)

    def timed(fn, reps=5):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    t_copy = min(timed(lambda: mbq.bench_copy(src, dst, width=w)) for w in (4, 8))
    t_read = min(timed(lambda: mbq.bench_read(src, sink, width=w)) for w in (1, 4))
    out = {"copy_gbps": 2 * n / t_copy / 1e9, "read_gbps": n / t_read / 1e9}
    steps = 20000
    for name, barrier in (("mfma_bf16_lds_fed_tflops", False), ("mfma_bf16_lds_fed_barrier_per_16_tflops", True)):
        flops = [0.0]

        def run():
            flops[0] = mbq.bench_mfma_loop(steps, barrier, sink)
        t = timed(run, reps=3)
        out[name] = flops[0] / t / 1e12
    del src, dst
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    sys.exit(main())
