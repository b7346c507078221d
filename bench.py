#!/usr/bin/env python3
"""Benchmark of the fused norm-test + AdamW step on one MI355X.

A "step" is one pass of the whole hot path (statistics, decision, fused AdamW: `normtest_step`) over
the headline workload: J=8 bfloat16 gradient rows of a flat d=1.5e9 vector with fp32 w, m, v, all
resident in HBM before the timed region.  Prints one JSON line; its `configs` array carries the other
workloads of the benchmark set (gpt2_small, fsdp_shard, per_sample, tiny), timed in the same run.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--mode full|stats|adamw|clipped|streams]
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
HEADLINE = "flat_1p5b"
METRIC = "norm-test+AdamW step: achieved HBM GB/s (% of peak), params/s at d=1.5B J=8"
OTHER_CONFIGS = ("gpt2_small", "fsdp_shard", "per_sample", "tiny")
KERNEL_SOURCE = os.path.join(ROOT, "paper_2412_21124_amd", "csrc", "normtest.hip")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def kernel_source_sha256(path: str = KERNEL_SOURCE) -> str:
    with open(path, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def traffic_from_profile(workload: str, mode: str, traffic_file: str = TRAFFIC_FILE, source: str = KERNEL_SOURCE):
    """HBM bytes per step that the tracked counter runs measured for this workload and mode (rocprofv3 --pmc
    FETCH_SIZE and WRITE_SIZE, scaled by the copy-kernel calibration; profiles/traffic.json records the runs), or
    None when there is no such run or when it was made with another version of the kernel source."""
    try:
        with open(traffic_file) as f:
            prof = json.load(f)
    except (OSError, ValueError):
        return None
    if prof.get("kernel_source_sha256") != kernel_source_sha256(source):
        return None
    entry = prof.get("entries", {}).get("%s/%s" % (workload, mode))
    return None if entry is None else float(entry["hbm_bytes_per_step"])


def make_workload(name: str, device: str, scale: float):
    import torch
    from paper_2412_21124_amd import synth
    if name == "flat_1p5b":
        return synth.flat_1p5b(d=int(1_500_000_000 * scale), device=device)
    if name == "gpt2_small":
        sizes = synth.gpt2_small_blocks()
        if scale != 1.0:
            sizes = synth.scaled_blocks(sizes, int(sum(sizes) * scale), 8)
        return synth.gpt2_small(1.0, block_sizes=sizes, device=device)
    if name == "fsdp_shard":
        return synth.fsdp_shard(3, d_shard=int(875_000_000 * scale), device=device)
    if name == "per_sample":
        return synth.per_sample(d=max(64, int((1 << 24) * scale) // 64 * 64), device=device)
    if name == "tiny":
        return synth.tiny(1e-2, device=device)
    if name.startswith("rows:"):
        # rows:J:d[:f32] -- J bf16 (fp32) rows of a flat d-coordinate vector with the headline's distribution
        # (row-count sweeps)
        parts = name.split(":")
        if len(parts) not in (3, 4) or (len(parts) == 4 and parts[3] not in ("f32", "bf16")):
            raise SystemExit("workload rows:J:d[:f32|:bf16], got %r" % name)
        J, d = int(parts[1]), int(parts[2])
        wl = synth.flat_1p5b(d=int(d * scale), J=J, device=device)
        wl.name = "rows_J%d" % J
        if len(parts) == 4 and parts[3] == "f32":
            ref = wl.hyper
            wl = synth.make("rows_J%d_f32" % J, J, int(d * scale), gdtype=torch.float32, sigma=1e-2, mu="normal",
                            mu_scale=1e-2, hyper=ref, seed=0, device=device)
        return wl
    if name in ("paper_300m", "paper_1.1b", "paper_3.4b"):
        which = name.split("_")[1]
        wl = synth.paper_model(which, device=device)
        return wl if scale == 1.0 else synth.paper_model(which, device=device, d=int(wl.d * scale))
    raise SystemExit("unknown workload %r" % name)


def cpu_baseline(wl, sample_coords: int):
    """The oracle, as it stands, on the host cores over the first `sample_coords` coordinates."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    from paper_2412_21124_amd import synth

    n = min(wl.d, sample_coords)
    cores = os.cpu_count() or 1
    threads = max(1, min(16, cores))     # the machine's CPU share for one GPU
    chunk = 1 << 22
    h = wl.hyper
    G = synth.grads_as_numpy(wl.grads, 0, n)
    w, m, v = (t[:n].cpu().numpy() for t in (wl.w, wl.m, wl.v))
    ranges = [(lo, min(n, lo + chunk)) for lo in range(0, n, chunk)]

    def work(r):
        lo, hi = r
        part = oracle.stats(G[:, lo:hi])
        oracle.adamw(G[:, lo:hi], w[lo:hi], m[lo:hi], v[lo:hi], h.lr, h.beta1, h.beta2, h.eps,
                     h.weight_decay, h.step)
        return part

    t0 = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        parts = list(ex.map(work, ranges))
    A, Bv, C = oracle.combine_chunks(parts)
    oracle.decide(A, Bv, C, wl.J, h.eta, h.b_k, h.b_max, h.round_to, h.ddof)
    dt = time.perf_counter() - t0
    # the same on one core, over a sixteenth of the sample
    n1 = max(1, n // 16)
    t1 = time.perf_counter()
    for r in [(lo, min(n1, lo + chunk)) for lo in range(0, n1, chunk)]:
        work(r)
    dt1 = time.perf_counter() - t1
    bytes_per_param = wl.J * wl.grad_bytes + 24
    used = min(threads, len(ranges))
    return {
        "value": n * bytes_per_param / dt / 1e9,
        "unit": "GB/s",
        "params_per_s": n / dt,
        "cores": used,
        "host_cores": cores,
        "kind": "oracle",
        "seconds": dt,
        "one_core_params_per_s": n1 / dt1,
        "sample": "first %d coordinates of the same workload (J=%d), statistics + decision + AdamW in fp64 "
                  "(the C oracle called from %d Python threads; the host reports %d cores)" % (n, wl.J, used, cores),
    }


MODE_TEXT = {
    "full": "stats+decision+fused AdamW in one pass",
    "stats": "statistics and decision only",
    "adamw": "mean + AdamW only (test skipped)",
    "clipped": "two-phase gradient-clipped step (stats+gbar, then AdamW)",
}


def time_steps(wl, mode: str, steps: int, warmup: int, *, layers=0, graph=False, calib_copy_gib=0):
    """Run `warmup` + `steps` steps of one workload and mode; HIP events on the launch stream bracket every step."""
    import torch
    from paper_2412_21124_amd import binding as B

    dev = wl.grads.device
    h = wl.hyper
    flags = {"full": B.NT_DO_STATS | B.NT_DO_ADAMW, "stats": B.NT_DO_STATS, "adamw": B.NT_DO_ADAMW,
             "clipped": B.NT_DO_STATS | B.NT_DO_ADAMW}[mode]
    if wl.name == "fsdp_shard" and mode in ("full", "stats"):
        flags |= B.NT_PARTIAL
    # bytes per coordinate: J gradient reads; + read/write of w, m, v; the clipped variant also writes and re-reads gbar
    bytes_per_param = wl.J * wl.grad_bytes + {"full": 24, "stats": 0, "adamw": 24, "clipped": 32}[mode]
    gbar_buf = torch.empty(wl.d, dtype=torch.float32, device=dev) if mode == "clipped" else None
    hy = B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                      step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof, flags=flags)
    gdtype = B.NT_BF16 if wl.grad_bytes == 2 else B.NT_F32
    ws_flags = flags | (B.NT_WRITE_GBAR if mode == "clipped" else 0)
    ws_bytes = B.normtest_workspace_bytes_for(gdtype, wl.J, wl.d, ws_flags)
    workspace = torch.empty(max(ws_bytes, 8), dtype=torch.uint8, device=dev)
    result = torch.empty(B.RESULT_BYTES, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    layer_off = layer_out = None
    if layers and mode == "adamw":
        raise SystemExit("--layers needs a mode that computes the statistics")
    if layers:
        if layers < 0:
            if not wl.meta.get("block_sizes"):
                raise SystemExit("--layers -1 needs a workload with parameter blocks (gpt2_small, per_sample)")
            sizes = wl.meta["block_sizes"]
        else:
            # sizes proportional to 1, 2, ..., N with odd remainders so that no boundary is aligned
            tot = layers * (layers + 1) // 2
            sizes = [max(1, (wl.d * (i + 1) // tot) | 1) for i in range(layers)]
            sizes[-1] = wl.d - sum(sizes[:-1])
            if sizes[-1] < 1:
                raise SystemExit("--layers: too many layers for this d")
        offs = [0]
        for sz in sizes:
            offs.append(offs[-1] + sz)
        layer_off = torch.tensor(offs, dtype=torch.int64, device=dev)
        layer_out = torch.empty(len(sizes) * B.LAYER_BYTES, dtype=torch.uint8, device=dev)

    # a shard of a longer vector says so (the library cuts it into tiles the way it would cut the whole vector)
    shard = None
    if "d_global" in wl.meta:
        shard = B.nt_shard_info(wl.meta["shard_id"], wl.meta["num_shards"], wl.meta["shard_offset"], wl.meta["d_global"])

    def step():
        if mode == "clipped":
            B.normtest_step_clipped(wl.grads, wl.w, wl.m, wl.v, gbar_buf, 1.0, hy, shard=shard, workspace=workspace,
                                    result=result, stream=stream)
        else:
            B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy, shard=shard, workspace=workspace, result=result,
                            stream=stream)
        if layer_off is not None:
            B.normtest_layer_stats(wl.grads, layer_off, workspace, layers=layer_out, stream=stream)

    if calib_copy_gib > 0:
        src = torch.zeros(calib_copy_gib << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        B.normtest_calib_copy(dst, src, stream=stream)
        torch.cuda.synchronize()
        del src, dst
    if graph:
        # capture on a side stream (the library only enqueues kernels, so the step can be captured as it is)
        eager_step = step
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            stream = side
            eager_step()                       # warm-up outside the capture
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            eager_step()
        stream = torch.cuda.current_stream()
        step = g.replay
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: exactly `steps` steps back to back, nothing else on the stream, a synchronize on both sides
    t0 = time.perf_counter()
    for i in range(steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # a second pass of `steps` steps with a pair of HIP events around each one, for the per-step distribution and
    # the kernel-level figure (the event records cost a few microseconds of stream time per step, which is why
    # they stay out of the timed region: it matters for steps well under a millisecond)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    for i in range(steps):
        starts[i].record(stream)
        step()
        stops[i].record(stream)
    torch.cuda.synchronize()
    ev_ms = sorted(s.elapsed_time(e) for s, e in zip(starts, stops))
    res = B.read_result(result).as_dict()
    alg_bytes = wl.d * bytes_per_param
    ev_avg = sum(ev_ms) / len(ev_ms)
    return {
        "flags": flags, "bytes_per_param": bytes_per_param, "alg_bytes": alg_bytes,
        "wall_ms_per_step": wall * 1e3 / steps, "ev_avg": ev_avg, "ev_median": ev_ms[len(ev_ms) // 2],
        "ev_min": ev_ms[0], "ev_max": ev_ms[-1], "result": res, "workspace_bytes": ws_bytes,
        "layers": 0 if layer_off is None else layer_off.numel() - 1,
        "route": MODE_TEXT[mode],
    }


def config_entry(name: str, device: str, steps: int, warmup: int):
    """One of the other workloads of the benchmark set, timed like the headline (full step, inputs resident)."""
    import torch
    wl = make_workload(name, device, 1.0)
    t = time_steps(wl, "full", steps, warmup)
    gbs = lambda ms: t["alg_bytes"] / (ms * 1e-3) / 1e9
    entry = {
        "workload": name, "J": wl.J, "d": wl.d, "grad_dtype": "bf16" if wl.grad_bytes == 2 else "f32",
        "bytes_per_param": t["bytes_per_param"], "steps": steps, "warmup": warmup, "route": t["route"],
        "ms_per_step": t["wall_ms_per_step"], "GBps": gbs(t["wall_ms_per_step"]),
        "frac": gbs(t["wall_ms_per_step"]) / HBM_PEAK_GBS,
        "params_per_s": wl.d / (t["wall_ms_per_step"] * 1e-3),
        "event_ms": {"avg": t["ev_avg"], "median": t["ev_median"], "min": t["ev_min"], "max": t["ev_max"]},
        "GBps_event_range": [gbs(t["ev_max"]), gbs(t["ev_min"])],
        "result": {k: t["result"][k] for k in ("T", "pass", "next_b", "status")},
    }
    del wl
    torch.cuda.empty_cache()
    return entry


STREAM_MATRIX = ([(0, r, w, False) for r in (0, 1, 2, 4, 8, 11) for w in (0, 1, 2, 3) if r + w > 0]
                 + [(0, 0, 1, True), (0, 0, 3, True)]
                 + [(4, 0, 0, False), (8, 0, 0, False), (16, 0, 0, False), (8, 0, 1, False), (8, 3, 3, False),
                    (4, 0, 3, True), (8, 0, 3, True), (16, 0, 3, True)])


def run_streams(args):
    """The library's stream-mix yardstick (normtest_calib_streams): what HBM gives for R read and W written
    streams walked in step with the step kernel's access widths and no arithmetic.  One JSON line."""
    import torch
    from paper_2412_21124_amd import binding as B
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU: the library has no CPU path")
    dev = "cuda:0"
    torch.cuda.set_device(0)
    coords = args.coords // 4 * 4
    mixes = STREAM_MATRIX if args.matrix else [(args.row_reads, args.reads, args.writes, args.rmw)]
    lc = args.launch_coords
    buf = torch.empty(max(B.calib_streams_bytes(coords, a, r, w) for a, r, w, _ in mixes), dtype=torch.uint8, device=dev)
    buf.zero_()
    stream = torch.cuda.current_stream()
    rows = []
    for a, r, w, rmw in mixes:
        nbytes = coords * (2 * a + 4 * r + (8 if rmw else 4) * w)
        for _ in range(args.warmup):
            B.normtest_calib_streams(buf, coords, a, r, w, rmw, launch_coords=lc, stream=stream)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        torch.cuda.synchronize()
        for e0, e1 in ev:
            e0.record(stream)
            B.normtest_calib_streams(buf, coords, a, r, w, rmw, launch_coords=lc, stream=stream)
            e1.record(stream)
        torch.cuda.synchronize()
        ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
        med = ms[len(ms) // 2]
        rows.append({"row_reads": a, "reads": r, "writes": w, "rmw": bool(rmw), "bytes": nbytes, "ms_median": med,
                     "ms_min": ms[0], "GBps": nbytes / (med * 1e-3) / 1e9, "frac": nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS})
        print("# row_reads %2d reads %2d writes %d rmw %d: %8.3f ms  %6.0f GB/s" % (a, r, w, rmw, med, rows[-1]["GBps"]),
              file=sys.stderr, flush=True)
    print(json.dumps({"metric": "stream-mix yardstick (no arithmetic): HBM GB/s", "unit": "GB/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "coords_per_stream": coords,
                      "coords_per_launch": lc if lc > 0 else coords, "peak": HBM_PEAK_GBS,
                      "mixes": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink d (debugging only; the result is then not the headline)")
    ap.add_argument("--mode", default="full", choices=["full", "stats", "adamw", "clipped", "streams"],
                    help="full: the fused step (headline); stats / adamw: one half only; clipped: two-phase variant; "
                         "streams: the stream-mix yardstick (see --row-reads, --reads, --writes, --rmw, --matrix)")
    ap.add_argument("--row-reads", type=int, default=8, help="streams mode: read streams of 2 bytes per coordinate")
    ap.add_argument("--reads", type=int, default=0, help="streams mode: read streams of 4 bytes per coordinate")
    ap.add_argument("--writes", type=int, default=3, help="streams mode: written streams of 4 bytes per coordinate")
    ap.add_argument("--rmw", action="store_true", help="streams mode: written streams are read first (in-place update)")
    ap.add_argument("--matrix", action="store_true", help="streams mode: every supported mix in one run")
    ap.add_argument("--coords", type=int, default=402_653_184,
                    help="streams mode: coordinates per stream (default 1.5 GiB per fp32 stream)")
    ap.add_argument("--launch-coords", type=int, default=0,
                    help="streams mode: coordinates per kernel launch (0: one launch), e.g. 134217728 = what the fused "
                         "step uses for up to 16 rows")
    ap.add_argument("--layers", type=int, default=0,
                    help="also produce the per-layer table each step: -1 = the workload's own parameter blocks, "
                         "N > 0 = N layers of uneven, unaligned sizes")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (removes launch gaps; matters for small d)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other workloads of the benchmark set (they run after the headline by default)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 29)
    ap.add_argument("--calib-copy-gib", type=int, default=0,
                    help="also run the library's plain copy kernel once on this many GiB (known traffic for scaling byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    if args.mode == "streams":
        return run_streams(args)

    import torch

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU: the library has no CPU path")
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = make_workload(args.workload, dev, args.scale)
    t = time_steps(wl, args.mode, args.steps, args.warmup, layers=args.layers,
                   graph=args.graph, calib_copy_gib=args.calib_copy_gib)
    headline = (args.workload == HEADLINE and args.mode == "full" and args.scale == 1.0 and not args.layers
                and not args.graph)
    ms_per_step = t["wall_ms_per_step"]
    value = t["alg_bytes"] / (ms_per_step * 1e-3) / 1e9
    achieved = t["alg_bytes"] / (t["ev_avg"] * 1e-3) / 1e9
    grad_dtype = "bf16" if wl.grad_bytes == 2 else "f32"
    out = {
        "metric": METRIC if headline else METRIC + " [this run: %s, mode %s%s]" % (
            wl.name, args.mode, "" if args.scale == 1.0 else ", d scaled by %g" % args.scale),
        "value": value,
        "unit": "GB/s",
        "pct_of_peak": 100.0 * value / HBM_PEAK_GBS,
        "params_per_s": wl.d / (ms_per_step * 1e-3),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "dtype_note": "arithmetic type: fp32 per coordinate, fp64 accumulation; gradients are stored as %s, w/m/v as fp32" % grad_dtype,
        "data": "synthetic",
        "config": {
            "workload": "%s: J=%d %s gradient rows, d=%d, fp32 w/m/v, %s" % (
                wl.name, wl.J, "bf16" if wl.grad_bytes == 2 else "fp32", wl.d, t["route"]),
            "mode": args.mode,
            "J": wl.J, "d": wl.d, "grad_dtype": grad_dtype,
            "bytes_per_param": t["bytes_per_param"], "flags": t["flags"],
            "layers": t["layers"],
            "graph_replay": bool(args.graph),
        },
        "result": {k: t["result"][k] for k in ("T", "pass", "next_b", "status")},
        "roofline": {
            "bound": "hbm",
            "kernel": "k_step (the fused streaming kernel; a long vector takes several launches of it, each over a run of "
                      "consecutive tiles; the HIP events bracket the whole step: every k_step launch, the gaps between "
                      "them and the reduction kernels)",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "launch_ms_avg": t["ev_avg"],
            "launch_ms_median": t["ev_median"],
            "launch_ms_min": t["ev_min"],
            "algorithmic_bytes": t["alg_bytes"],
            # counter-measured HBM bytes per step, quoted from the tracked profile of this kernel source (null if the
            # source has changed since that run, or if this is not a profiled configuration)
            "traffic": (traffic_from_profile(wl.name, args.mode)
                        if (args.scale == 1.0 and not args.layers) else None),
        },
    }
    if not args.no_cpu_baseline and args.mode == "full":
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample)
    if headline and not args.no_configs:
        del wl
        torch.cuda.empty_cache()
        out["configs"] = [config_entry(name, dev, 200 if name == "tiny" else 20, 5) for name in OTHER_CONFIGS]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
