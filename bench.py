#!/usr/bin/env python3
"""Benchmark of the fused MBCI chain on one MI355X.

A step is one pass of the whole hot path (tile pick on the host, then the fused kernel:
A tile -> registers, B/D tiles -> LDS, GEMM 1, [softmax], GEMM 2, store E) over one batch of
synthetic input.  Inputs are resident in HBM before the timed region starts.  Because the
small workloads fit in the 256 MB memory-side cache, steps rotate over enough distinct
input/output sets (> 768 MiB in total) that every step's operands come from HBM.

Protocol (the same for every workload and for the ceilings):
  1. --warmup untimed steps (they also set kernel attributes before any capture);
  2. the --steps steps, rounded up to whole rotations over the buffer sets (a graph of 20 steps
     would replay the same 20 sets for ever, a third of which the memory-side cache can hold),
     are captured once into a HIP graph (each step is still one call of the C ABI on the
     capturing stream; the host-side tile pick runs at capture);
  3. an untimed clock ramp: the graph is replayed until at least RAMP_MS of device time have
     passed, whatever --warmup says (a cold engine clock makes a launch up to a third slower);
  4. the timed region is `replays` back-to-back replays of that graph, as many as it takes to
     fill MIN_REGION_MS, bracketed by synchronize on both sides.  `ms_per_step` and `value`
     come from the host clock around the region divided by the steps of the graph x replays;
     `us_per_launch_events` from HIP events on the launch stream around the same region.
--eager times plain calls instead of graph replays (the tile pick is then inside every step).

Prints ONE JSON line: the BASELINE metric (effective HBM GB/s on compulsory bytes) with a
`roofline` object for the chain kernel and a `cpu_baseline` object (the fp64 oracle timed on
this host's cores).  The metric is quoted per configuration: a default run also measures the
other four configurations after the timed region (one child process each, same protocol) and
reports them under `per_config`, each with its own roofline, parity and cpu_baseline; `value`
stays cfg2's.  --ceilings measures, with the same protocol, what bounds the kernel on this
machine: a streaming copy, a loop of MFMAs only and an empty kernel.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
MFMA_PEAK_TFLOPS = 2500.0  # dense fp16 / bf16
RAMP_MS = 150.0            # untimed launches before anything is timed
MIN_REGION_MS = 20.0       # the timed region is at least this long
CPU_SAMPLE_FLOPS = 2.0e10  # fp64 work given to the oracle per workload (a few seconds of the host's cores)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000, help="steps per captured graph (the timed region replays it)")
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="cfg2", help="cfg1..cfg5 (default: cfg2, the configuration the metric is quoted on), or a row of the "
                                                      "paper's shape tables: G1..G12, S1..S9")
    ap.add_argument("--tiles", default=None, help="mb,rg,ns,nj[,tl] to override the picker")
    ap.add_argument("--tune", action="store_true",
                    help="choose the tiles by the measured search (Alg. 1) before the warm-up instead of by the "
                         "model alone; candidates are timed as the timed region is (graph replay over the rotating sets)")
    ap.add_argument("--chain3", action="store_true",
                    help="append a third GEMM: G = E . F with F[b, L, L] (built for K = L in {64, 128}); bytes and "
                         "flops of the extra operand and GEMM are added to the figures")
    ap.add_argument("--eager", action="store_true", help="time plain calls instead of a HIP graph replay")
    ap.add_argument("--warm", action="store_true", help="reuse one buffer set (cache-resident operands)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="with the default workload the other four configurations are measured as well (child "
                         "processes, after the timed region) and reported under 'per_config'; this switches that off")
    ap.add_argument("--ceilings", action="store_true",
                    help="measure the machine's ceilings instead of the chain: device copy (16 MiB and 1 GiB of "
                         "traffic), MFMA-only loop, empty kernel; one JSON line")
    ap.add_argument("--copy-ref", type=int, default=0, metavar="MiB",
                    help="after the timed region also run one plain device copy of this many MiB (the "
                         "known-size kernel that calibrates the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--traffic", default=os.path.join(ROOT, "profiles", "traffic.json"),
                    help="JSON file with measured HBM bytes per launch (from the rocprofv3 --pmc runs)")
    return ap.parse_args()


class Timer:
    """The protocol of the module docstring around any `step(i)`."""

    def __init__(self, torch, steps, warmup, eager=False, rotate=1):
        # the graph holds whole rotations over the buffer sets: a short graph would only ever touch the
        # first few sets, which together may fit the 256 MB memory-side cache in front of HBM
        steps = (steps + rotate - 1) // rotate * rotate
        self.torch, self.steps, self.warmup, self.eager = torch, steps, warmup, eager

    def measure(self, step):
        torch = self.torch
        for i in range(max(self.warmup, 1)):
            step(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        graph = None
        if not self.eager:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):      # the binding launches on torch's current (capturing) stream
                for i in range(self.steps):
                    step(i)

        def once():
            if graph is not None:
                graph.replay()
            else:
                for i in range(self.steps):
                    step(i)
        # clock ramp: untimed passes, back to back, until RAMP_MS of device time have passed
        # (replays keep the device busy; plain calls from Python would leave it idle most of the time)
        ramp_launches, ramp_ms, passes = 0, 0.0, 1
        while ramp_ms < RAMP_MS:
            e0.record()
            for _ in range(passes):
                once()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            ramp_ms += ms
            ramp_launches += passes * self.steps
            once_ms = ms / passes
            passes = int(min(10000, max(1, 30.0 / max(once_ms, 1e-4))))       # aim at 30 ms between synchronisations
        replays = max(1, int(math.ceil(MIN_REGION_MS / max(once_ms, 1e-3))))
        # ---- timed region: `replays` x `steps` steps ---------------------------------------
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(replays):
            once()
        e1.record()
        torch.cuda.synchronize()
        wall_s = time.perf_counter() - t0
        dev_s = e0.elapsed_time(e1) * 1e-3
        n = self.steps * replays
        return {"t_step": wall_s / n, "t_kernel": dev_s / n, "replays": replays, "graph_steps": self.steps,
                "clock_ramp_launches": ramp_launches, "clock_ramp_ms": ramp_ms}


def run_ceilings(args, torch, mcf):
    """The machine's ceilings under the protocol of the chain: copy, MFMA-only, empty kernel."""
    out = {"kind": "ceilings", "steps": args.steps, "warmup": args.warmup}
    timer = Timer(torch, args.steps, args.warmup)

    def copy_case(total_bytes, rotate_bytes):
        half = total_bytes // 2                                 # read half, write half
        n_sets = max(2, min(64 if total_bytes >= 2**20 else 1024, rotate_bytes // total_bytes))
        srcs = [torch.full((half // 2,), 1.0, dtype=torch.float16, device="cuda") for _ in range(n_sets)]
        dsts = [torch.empty_like(s) for s in srcs]
        r = timer.measure(lambda i: mcf.probe_copy(dsts[i % n_sets], srcs[i % n_sets]))
        assert bool((dsts[0] == 1.0).all())
        return {"traffic_bytes": total_bytes, "buffer_sets": n_sets, "us_per_launch": r["t_kernel"] * 1e6,
                "gbs": total_bytes / r["t_kernel"] / 1e9, "frac_of_hbm_peak": total_bytes / r["t_kernel"] / 1e9 / HBM_PEAK_GBS,
                "replays": r["replays"]}

    out["copy_288KiB"] = copy_case(288 * 2**10, 1024 * 2**20)   # cfg1's compulsory bytes: what a load -> store chain costs a launch
    out["copy_10MiB"] = copy_case(10 * 2**20, 1024 * 2**20)     # cfg4's
    out["copy_16MiB"] = copy_case(16 * 2**20, 1024 * 2**20)     # cfg2's compulsory bytes, operands from HBM
    out["copy_24MiB"] = copy_case(24 * 2**20, 1024 * 2**20)     # cfg3's
    out["copy_1GiB"] = copy_case(2**30, 4 * 2**30)
    buf = torch.empty(2048 * 8 * 64, dtype=torch.float32, device="cuda")
    for waves, blocks in ((4, 256), (8, 256), (4, 512)):
        iters = 64
        r = timer.measure(lambda i: mcf.probe_mfma(buf, blocks, waves, iters))
        flops = blocks * waves * iters * 8 * 32768
        out[f"mfma_{blocks}x{waves}w"] = {"us_per_launch": r["t_kernel"] * 1e6, "flops": flops,
                                           "tflops": flops / r["t_kernel"] / 1e12,
                                           "frac_of_mfma_peak": flops / r["t_kernel"] / 1e12 / MFMA_PEAK_TFLOPS}
    # long loop: the launch is amortised, what remains is the sustained matrix rate
    iters = 4096
    r = Timer(torch, 50, 5).measure(lambda i: mcf.probe_mfma(buf, 256, 8, iters))
    flops = 256 * 8 * iters * 8 * 32768
    out["mfma_sustained"] = {"us_per_launch": r["t_kernel"] * 1e6, "flops": flops, "tflops": flops / r["t_kernel"] / 1e12,
                             "frac_of_mfma_peak": flops / r["t_kernel"] / 1e12 / MFMA_PEAK_TFLOPS}
    for blocks in (1, 256, 2048):
        r = timer.measure(lambda i: mcf.probe_empty(blocks))
        out[f"empty_{blocks}"] = {"us_per_launch": r["t_kernel"] * 1e6}
    print(json.dumps(out))
    return 0


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the fused chain shards over batch / row "
              "blocks with no exchange; no multi-GPU path is built). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import mcf_inputs as mi
    import paper_2506_22169_amd as mcf
    from paper_2506_22169_amd.binding import make_problem as c_problem

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    mcf.load_library()  # fail loudly if the HIP library is not built
    if args.ceilings:
        return run_ceilings(args, torch, mcf)

    w = mi.WORKLOADS[args.workload] if args.workload in mi.WORKLOADS else mi.PAPER_SHAPES[args.workload]
    tdt = torch.float16 if w.dtype == "f16" else torch.bfloat16
    tiles = tuple(int(v) for v in args.tiles.split(",")) if args.tiles else None

    # ---- inputs: set 0 is the seeded workload; the other sets are batch-rotations of it ----
    x = mi.make_inputs(w, values=False)

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(tdt).cuda()

    A0, B0s, D0 = dev(x["a_bits"]), dev(x["b_bits"]), dev(x["d_bits"])
    per_set, flops = w.compulsory_bytes, w.flops
    P = w.L
    if args.chain3:                       # F[b, L, P] read once; G[b, M, P] replaces E[b, M, L] (P = L)
        f_bits = mi.to_bits(mi.draw(w.seed, 4, (w.batch, w.L, P), w.dist), w.dtype)
        F0 = dev(f_bits)
        per_set += 2 * w.batch * w.L * P
        flops += 2 * w.batch * w.M * w.L * P
    n_sets = 1 if args.warm else max(2, min(64, math.ceil(768 * 2**20 / per_set)))
    if per_set * n_sets > 8 * 2**30:
        n_sets = max(2, (8 * 2**30) // per_set)
    sets = []
    for s in range(n_sets):
        sh = s % max(w.batch, 1)
        A = A0 if s == 0 else torch.roll(A0, sh, 0).contiguous()
        Bs = B0s if s == 0 else torch.roll(B0s, sh, 0).contiguous()
        D = D0 if s == 0 else torch.roll(D0, sh, 0).contiguous()
        B = Bs.transpose(1, 2) if w.softmax else Bs
        E = torch.empty((w.batch, w.M, w.L), dtype=tdt, device="cuda")
        F = None if not args.chain3 else (F0 if s == 0 else torch.roll(F0, sh, 0).contiguous())
        sets.append((A, B, D, E, F))

    def step(i):
        A, B, D, E, F = sets[i % n_sets]
        if args.chain3:
            mcf.gemm_chain3(A, B, D, F, scale=w.scale if w.softmax else None, out=E, tiles=tiles)
        elif w.softmax:
            mcf.softmax_gemm_chain(A, B, D, w.scale, out=E, tiles=tiles)
        else:
            mcf.gemm_chain(A, B, D, out=E, tiles=tiles)

    prob = c_problem(w.batch, w.M, w.K, w.N, w.L, w.dtype,
                     b_stride=(w.N * w.K, 1, w.K) if w.softmax else None)
    search = None
    if args.chain3 and tiles is None and not args.tune:
        try:
            t3 = mcf.pick_tiles3(prob, P, w.softmax)
        except mcf.McfError:
            print(f"bench.py: no three-GEMM kernels built for K={w.K} L={w.L} P={P}", file=sys.stderr)
            return 2
        tiles = (t3.mb, t3.rg, t3.ns, t3.nj)
    if args.tune and tiles is None:
        for i in range(max(args.warmup, 3000)):   # bring the clocks up before the first candidate is timed
            step(i)
        torch.cuda.synchronize()

        def measure(t):
            nonlocal tiles
            tiles = (t.mb, t.rg, t.ns, t.nj) if args.chain3 else (t.mb, t.rg, t.ns, t.nj, t.tl)
            reps = max(2 * n_sets, min(200, args.steps))
            for i in range(3):
                step(i)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for i in range(reps):
                    step(i)
            g.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e-3 / reps
        if args.chain3:
            try:
                best, rep = mcf.search_tiles3(prob, P, w.softmax, measure, seed=w.seed)
            except mcf.McfError:
                print(f"bench.py: no three-GEMM kernels built for K={w.K} L={w.L} P={P}", file=sys.stderr)
                return 2
        else:
            best, rep = mcf.search_tiles(prob, w.softmax, measure, seed=w.seed)
        tiles = (best.mb, best.rg, best.ns, best.nj) if args.chain3 else (best.mb, best.rg, best.ns, best.nj, best.tl)
        search = {"measured": rep.measured, "generations": rep.generations, "converged": bool(rep.converged),
                  "best_us": rep.best_t_s * 1e6,
                  "log": [[e.generation, e.mb, e.rg, e.ns, e.nj, e.tl, round(e.t_est_s * 1e6, 3), round(e.t_meas_s * 1e6, 3)]
                          for e in rep.entries()]}
    # the tile pick on the host (what a step does before its launch): timed on its own
    tp0 = time.perf_counter()
    for _ in range(200):
        picked_auto = mcf.pick_tiles(prob, w.softmax)
    pick_us = (time.perf_counter() - tp0) / 200 * 1e6
    picked = picked_auto if tiles is None else mcf.eval_tiles(prob, *tiles, softmax=w.softmax)

    m = Timer(torch, args.steps, args.warmup, args.eager, rotate=n_sets).measure(step)
    t_step, t_kernel = m["t_step"], m["t_kernel"]

    if args.copy_ref:
        n = args.copy_ref * 2**20 // 2
        src = torch.ones(n, dtype=torch.float16, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    gbs = per_set / t_step / 1e9
    tflops = flops / t_step / 1e12
    ai = flops / per_set
    bound = "hbm" if ai < MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9) else "mfma"
    if bound == "hbm":
        achieved, peak, unit = per_set / t_kernel / 1e9, HBM_PEAK_GBS, "GB/s"
    else:
        achieved, peak, unit = flops / t_kernel / 1e12, MFMA_PEAK_TFLOPS, "TFLOP/s"
    traffic = None
    if args.traffic and os.path.exists(args.traffic) and not args.chain3:
        traffic = json.load(open(args.traffic)).get(args.workload)

    # ---- parity of set 0 at the benchmarked configuration + oracle timing ------------------
    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        A, B, D, E, F = sets[0]
        step(0)
        torch.cuda.synchronize()
        full_flops = flops
        nb = w.batch if full_flops <= CPU_SAMPLE_FLOPS else max(1, int(w.batch * CPU_SAMPLE_FLOPS / full_flops))
        rows = None
        A64 = mi.from_bits(x["a_bits"][:nb], w.dtype)
        B64 = mi.from_bits(x["b_bits"][:nb], w.dtype)
        B64 = B64.transpose(0, 2, 1) if w.softmax else B64
        D64 = mi.from_bits(x["d_bits"][:nb], w.dtype)
        if full_flops > CPU_SAMPLE_FLOPS and not args.chain3:   # long-sequence workload: a bounded sample of rows of one head
            rng = np.random.default_rng(0)
            n_rows = max(64, int(CPU_SAMPLE_FLOPS / (2.0 * w.N * (w.K + w.L))))
            rows = np.stack([np.zeros(n_rows, dtype=np.int64), rng.integers(0, w.M, n_rows)], axis=1)
        tc = time.perf_counter()
        if rows is None:
            if args.chain3:
                ref, threads = oracle.chain3(A64, B64, D64, mi.from_bits(f_bits[:nb], w.dtype), softmax=w.softmax,
                                             scale=w.scale, return_threads=True)
            else:
                ref, threads = oracle.chain(A64, B64, D64, softmax=w.softmax, scale=w.scale, return_threads=True)
            got = mi.from_bits(E[:nb].contiguous().view(torch.int16).cpu().numpy().view(np.uint16), w.dtype)
            frac = nb / w.batch
            sample = f"all rows of {nb} of {w.batch} batches"
        else:
            ref = oracle.chain_rows(A64, B64, D64, rows, softmax=w.softmax, scale=w.scale)
            threads = os.cpu_count()
            got = mi.from_bits(E[0][torch.from_numpy(rows[:, 1]).cuda()].contiguous().view(torch.int16)
                               .cpu().numpy().view(np.uint16), w.dtype)
            frac = len(rows) / (w.batch * w.M)
            sample = f"{len(rows)} sampled rows of batch 0"
        cpu_s = time.perf_counter() - tc
        cpu_baseline = {"value": per_set * frac / cpu_s / 1e9, "unit": "GB/s", "cores": int(threads),
                        "kind": "oracle", "sample": sample, "seconds": cpu_s,
                        "gflops_fp64": flops * frac / cpu_s / 1e9}
        parity = {"max_abs_err": float(np.max(np.abs(got - ref))), "max_abs_ref": float(np.max(np.abs(ref))),
                  "tolerance": 1e-2, "checked": sample}
        parity["ok"] = bool(parity["max_abs_err"] <= 1e-2 * parity["max_abs_ref"])

    roofline = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak, "traffic": traffic}
    out = {
        "metric": "fused-chain effective HBM GB/s (% of peak) and TFLOP/s per config",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t_step * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: batch={w.batch} M={w.M} K={w.K} N={w.N} L={w.L} {w.dtype}"
                               f"{' softmax' if w.softmax else ''}{f' + third GEMM P={P}' if args.chain3 else ''}",
                   "tiles": {"mb": picked.mb, "rg": picked.rg, "ns": picked.ns, "nj": picked.nj, "tm": picked.tm,
                             "tn": picked.tn, "tk": picked.tk, "tl": picked.tl, "stages": picked.stages},
                   "buffer_sets": n_sets, "launch": "eager" if args.eager else "hip_graph",
                   "replays": m["replays"], "graph_steps": m["graph_steps"], "timed_steps": m["graph_steps"] * m["replays"],
                   "clock_ramp_launches": m["clock_ramp_launches"], "clock_ramp_ms": round(m["clock_ramp_ms"], 1),
                   "tile_choice": "search" if search else ("given" if args.tiles else "model"), "search": search},
        "pct_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS, "tflops": tflops,
        "pct_mfma_peak": 100.0 * tflops / MFMA_PEAK_TFLOPS,
        "us_per_launch_events": t_kernel * 1e6,
        "host_tile_pick_us": pick_us,
        "model_t_est_us": picked.t_est_s * 1e6,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    # ---- the metric is quoted per configuration: measure the other four as well (`value` is cfg2's) ----
    if (args.workload == "cfg2" and not args.no_per_config and not args.no_cpu_baseline
            and not (args.chain3 or args.tune or args.tiles or args.warm or args.eager)):
        import subprocess
        per = {"cfg2": {"us_per_launch": t_kernel * 1e6, "gbs": gbs, "tflops": tflops, "roofline": roofline,
                        "tiles": [picked.mb, picked.rg, picked.ns, picked.nj, picked.tl],
                        "cpu_baseline": cpu_baseline, "parity_ok": parity["ok"]}}
        del sets
        torch.cuda.empty_cache()
        for name in ("cfg1", "cfg3", "cfg4", "cfg5"):
            steps = 20 if name == "cfg5" else 1000    # graph length of the child; its timed region is sized by time
            try:
                r = subprocess.run([sys.executable, os.path.abspath(__file__), "--workload", name, "--steps", str(steps),
                                    "--warmup", str(min(args.warmup, 50)), "--no-per-config"],
                                   capture_output=True, text=True, timeout=300)
                d = json.loads(r.stdout.strip().splitlines()[-1])
                t = d["config"]["tiles"]
                per[name] = {"us_per_launch": d["us_per_launch_events"], "gbs": d["value"], "tflops": d["tflops"],
                             "roofline": d["roofline"], "tiles": [t["mb"], t["rg"], t["ns"], t["nj"], t["tl"]],
                             "cpu_baseline": d["cpu_baseline"], "parity_ok": d["parity"]["ok"]}
            except Exception as e:      # context only: never fail the benchmark line over it
                per[name] = {"error": str(e)[:200]}
        out["per_config"] = per
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
