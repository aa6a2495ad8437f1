#!/usr/bin/env python3
"""LOOKAT decode benchmark on one MI355X.

A "step" is one pass of the decode hot path over every layer of the workload: per layer,
encode the new token's key into the code cache, build the query's lookup tables, attend over
the coded cache.  `--path fused` (the default where the shape has a fused instance) does the
three in ONE kernel per layer (lookat_decode_step); `--path calls` makes the three library
calls (lookat_encode_keys, lookat_build_lut, lookat_attend_decode).  The step is captured in a
HIP graph and every replay is compared with the eager result; `--mode auto` (default) then times a
few untimed steps both ways, replayed from the graph and as plain C-ABI calls, and runs the warm-up
and the timed steps the faster way (`config.launch` says which; `--mode graph|eager` force one).
Inputs are seeded and synthetic (lookat_inputs), resident in HBM before the timed region;
codebooks come from the library's own Lloyd iterations on seeded calibration keys.
`--workload C4` times the prefill block instead (encode, table build, causal scoring).

Prints ONE JSON line: whole-step throughput in keys scored per second, the HBM roofline
of the decode kernel (algorithmic code+value bytes / average launch duration, measured
with HIP events on the launch stream, plus counted HBM traffic) and the CPU oracle timed on a
bounded sample.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

# HBM traffic per launch of the dominant kernel, from hardware counters (they cannot be read
# inside this process: two separate `rocprofv3 --pmc` runs of this script, FETCH_SIZE then
# WRITE_SIZE, recorded in the counter summaries under profiles/).  Entry: (FETCH_SIZE per dispatch,
# FETCH_SIZE of lookat::stream_read_kernel in the same run, KiB that kernel reads, WRITE_SIZE
# per dispatch in KiB).  bytes = (fetch * known_KiB / stream_fetch + write) * 1024.
COUNTED_TRAFFIC = {
    # key: (workload, fused step?) -> (FETCH_SIZE, stream FETCH_SIZE, stream KiB, WRITE_SIZE KiB, launch shape counted)
    # launch shape: "fused" = the 512-thread fused-step instance, one range per (b,h); "fused, paired" = its 1024-thread
    # form that serves two batch entries of a head per workgroup; else (ranges, wavefronts) of
    # lookat_attend_decode as lookat_attend_decode_launch_shape reports them.
    ("C1", True): (1249.5, 776.004, 1536.0, 3.375, "fused"),
    ("C1", False): (826.5, 776.004, 1536.0, 3.0, (1, 4)),
    ("C2", True): (26394.5, 24586.0, 49152.0, 108.0, "fused, paired"),
    ("C2", False): (26144.5, 24584.0, 49152.0, 96.0, (1, 4)),
    ("C3", True): (1.0838e6, 1.04858e6, 2097152.0, 136.0, "fused"),
    ("C3", False): (1.08264e6, 1.04858e6, 2097152.0, 268.0, (2, 16)),
    ("C4", "score_prefill"): (37033.6, 1.0, 2.0, 2.10989e6, None),   # lookup-and-sum kernel; FETCH_SIZE at 2 KiB per count (calibration of the 2 GiB read)
    ("C4", "score_prefill_dense"): (41175.7, 1.0, 2.0, 2.09782e6, None),   # matrix-core kernel
}


def counted_traffic(key, launch_shape=None):
    """HBM bytes per launch from the stored counter readings, or None when there is no reading for this
    workload or the launch shape timed now is not the one the counters were read on (a stale reading)."""
    if key not in COUNTED_TRAFFIC:
        return None
    fetch, stream_fetch, known_kib, write_kib, counted_shape = COUNTED_TRAFFIC[key]
    if counted_shape is not None and launch_shape != counted_shape:
        return None
    return int(round((fetch * known_kib / stream_fetch + write_kib) * 1024.0))


def per_launch_stats(torch, fn, layers, n_launch, batches=24):
    """Back-to-back launches timed in `batches` batches (a HIP event between batches only: an event between
    every two launches costs the GPU about 3 us and would measure itself): per-launch mean of every batch;
    returns the median, minimum and maximum over the batches (us per launch)."""
    per = max(len(layers), n_launch // batches // len(layers) * len(layers))   # whole rotations over the layers' caches
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(batches + 1)]
    for ly in layers:
        fn(ly)
    torch.cuda.synchronize()
    ev[0].record()
    for b in range(batches):
        for i in range(per):
            fn(layers[i % len(layers)])
        ev[b + 1].record()
    torch.cuda.synchronize()
    t = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 / per for i in range(batches))
    return {"median": t[len(t) // 2], "min": t[0], "max": t[-1], "launches_per_batch": per, "batches": batches}


def pick_launch_mode(mode, step, replay, trial_steps=10):
    """The way the steps are launched: `step` (plain C-ABI calls) or `replay` (the captured graph).
    With mode "auto", both run `trial_steps` untimed-region steps and the faster is taken (a graph
    node costs the GPU about half a microsecond more than a queued launch; plain calls cost host time
    per launch, which only matters when a step has many short kernels)."""
    import torch
    if mode == "eager" or replay is None:
        return step, "eager"
    if mode == "graph":
        return replay, "graph"
    took = {}
    for name, fn in (("graph", replay), ("eager", step)):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(trial_steps):
            fn()
        torch.cuda.synchronize()
        took[name] = (time.perf_counter() - t0) / trial_steps
    name = "graph" if took["graph"] <= took["eager"] else "eager"
    other = "eager" if name == "graph" else "graph"
    return (replay if name == "graph" else step), f"{name} (auto; {other}: {took[other] * 1e3:.4f} ms/step in the trial)"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4"],
                    help="C1..C3: decode step (C2 is the configuration the metric is quoted on); C4: prefill block")
    ap.add_argument("--mode", default="auto", choices=["auto", "graph", "eager"],
                    help="graph: one step captured in a HIP graph and replayed; eager: one C-ABI call at a time; "
                         "auto: whichever of the two runs a few untimed steps faster")
    ap.add_argument("--path", default="auto", choices=["auto", "fused", "calls"],
                    help="fused: one lookat_decode_step per layer; calls: encode_keys + build_lut + attend_decode; "
                         "auto: fused wherever the library has a fused kernel for the shape")
    ap.add_argument("--batch", type=int, default=0,
                    help="override the workload's batch size (e.g. --workload C3 --batch 1: single-user long context; "
                         "the fused step is then cut into ranges, lookat_decode_step_split)")
    ap.add_argument("--group", type=int, default=1, choices=[1, 2, 4, 8],
                    help="decode workloads: query heads per key/value head (grouped-query attention): the workload's H "
                         "query heads share H/group key/value heads; times lookat_attend_decode_gqa")
    ap.add_argument("--codes", default="encoded", choices=["encoded", "uniform"],
                    help="encoded: the cache holds the codes lookat_encode_keys gives the seeded keys (skewed, correlated "
                         "histograms, as real caches have); uniform: independent uniform random bytes, the worst case for "
                         "LDS bank conflicts of the table gathers")
    ap.add_argument("--kmeans-iters", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle leg")
    ap.add_argument("--probes", action="store_true",
                    help="also time the measurement aids on this workload's buffers and add them as \"probes\": the launch "
                         "interval of an empty kernel, the read stream in a sweep of launch shapes, and attention with the "
                         "in-kernel ticket merge (include/lookat_probe.h)")
    return ap.parse_args()


class Layer:
    """Device state of one attention layer: codebooks, code cache, value cache, query, new key."""

    def __init__(self, lk, li, cfg, device, index, kmeans_iters):
        import torch
        case = li.torch_case(cfg, device, layer=index)
        self.cb = lk.lookat_kmeans(case["calib"], case["cb_init"], kmeans_iters)
        self.codes = lk.lookat_encode_keys(case["keys"], self.cb)           # [B,H,L,m] code cache
        self.new_key = case["keys"][:, :, cfg.L - 1:cfg.L].contiguous()      # the step's new token
        # the fused step takes q and the new key in one dtype (fp16 -> fp32 widening is exact)
        self.q_step = case["q"][:, :, 0].to(self.new_key.dtype).contiguous()
        self.k_step = self.new_key[:, :, 0].contiguous()
        self.values = case["values"]
        self.q = case["q"]
        self.lut = torch.empty((cfg.B, cfg.H, 1, cfg.m, cfg.K), dtype=torch.float32, device=device)
        self.out = torch.empty((cfg.B, cfg.H, cfg.d_k), dtype=torch.float32, device=device)
        del case


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import lookat_inputs as li
    import paper_2601_10155_amd as lk

    if not torch.cuda.is_available():
        print("bench.py needs an MI355X; no GPU is visible", file=sys.stderr)
        sys.exit(1)
    lk.load_library()   # raises if liblookat.so is not built: there is no fallback path
    device = torch.device("cuda:0")
    torch.cuda.set_device(0)

    cfg = li.CONFIGS[args.workload]
    if args.batch:
        cfg = li.shrink(cfg, B=args.batch)
    if cfg.T > 1:
        prefill_main(args, cfg, lk, li, torch, device)
        return
    if args.group > 1:
        gqa_main(args, cfg, lk, li, torch, device)
        return
    scale = 1.0 / math.sqrt(cfg.d_k)
    layers = [Layer(lk, li, cfg, device, i, args.kmeans_iters) for i in range(cfg.layers)]
    if args.codes == "uniform":
        gen = torch.Generator(device=device)
        gen.manual_seed(li.BASE_SEED + 4242)
        for ly in layers:
            ly.codes.copy_(torch.randint(0, 256, ly.codes.shape, generator=gen, device=device, dtype=torch.uint8))
    splits = lk.attend_decode_auto_splits(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L)
    ws_bytes = lk.attend_decode_workspace_bytes(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L, splits)
    workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=device)
    torch.cuda.synchronize()

    def decode_only(ly):
        lk.lookat_attend_decode(ly.lut.view(cfg.B, cfg.H, cfg.m, cfg.K), ly.codes, ly.values, scale,
                                num_splits=splits, workspace=workspace, out=ly.out)

    # auto: the fused step wherever the library has one for the shape (one workgroup per (b,h) when that
    # fills the chip's 256 compute units or the unfused call would not cut the sequence either; else cut
    # into ranges, lookat_decode_step_split)
    fused = args.path == "fused" or (args.path == "auto" and cfg.d_k in (64, 128) and cfg.m in (2, 4, 8, 16))

    # the fused step is cut into ranges when one workgroup per (b,h) would leave the chip idle
    fused_split = fused and splits > 1 and cfg.B * cfg.H < 256

    def fused_only(ly):
        if fused_split:
            lk.lookat_decode_step_split(ly.q_step, ly.k_step, ly.cb, ly.codes, ly.values, scale, num_splits=splits,
                                        workspace=workspace, out=ly.out)
        else:
            lk.lookat_decode_step(ly.q_step, ly.k_step, ly.cb, ly.codes, ly.values, scale, out=ly.out)

    def step():
        for ly in layers:
            if fused:
                fused_only(ly)
            else:
                lk.lookat_encode_keys(ly.new_key, ly.cb, cache=ly.codes, position=cfg.L - 1)
                lk.lookat_build_lut(ly.q, ly.cb, lut_out=ly.lut)
                decode_only(ly)

    # ---- one eager step: its outputs are the reference for the graph replays ----------
    step()
    torch.cuda.synchronize()
    eager_out = [ly.out.clone() for ly in layers]

    graph = None
    if args.mode != "eager":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                      # warm the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(2):              # replays must reproduce the eager step exactly
            for ly in layers:
                ly.out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            for ly, ref in zip(layers, eager_out):
                if not torch.equal(ly.out, ref):
                    raise RuntimeError("graph replay differs from the eager step")

    run_step, launch = pick_launch_mode(args.mode, step, graph.replay if graph is not None else None)

    # ---- timed region: W warm-up steps, then exactly K steps ----------------------------
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    keys_per_step = cfg.layers * cfg.B * cfg.H * cfg.L
    value = keys_per_step * args.steps / elapsed
    ms_per_step = elapsed * 1e3 / args.steps

    # ---- roofline of the dominant kernel: decode launches alone, back to back, rotating over
    #      the layers' distinct caches (so no launch re-reads what the last-level cache holds) ----
    bytes_per_launch = cfg.B * cfg.H * cfg.L * (cfg.m + 2 * cfg.d_k)
    n_launch = max(args.steps, 20) * cfg.layers
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def time_launches(fn):
        for ly in layers:
            fn(ly)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n_launch):
            fn(layers[i % cfg.layers])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n_launch

    for ly in layers:                     # the tables must exist for the stand-alone decode launches
        lk.lookat_build_lut(ly.q, ly.cb, lut_out=ly.lut)
    us_decode_alone = time_launches(decode_only)
    us_per_launch = time_launches(fused_only) if fused else us_decode_alone
    achieved = bytes_per_launch / us_per_launch / 1e3   # GB/s
    stats = per_launch_stats(torch, fused_only if fused else decode_only, layers, n_launch)
    stats_alone = per_launch_stats(torch, decode_only, layers, n_launch) if fused else stats
    paired = fused and not fused_split and lk.decode_step_entries_per_workgroup(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L) == 2
    launch_shape = ("fused, paired" if paired else "fused") if (fused and not fused_split) else \
        (None if fused else lk.attend_decode_launch_shape(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L, splits))

    # plain read stream over the same value caches: what the HBM read path delivers here
    sink = torch.zeros(4, dtype=torch.int32, device=device)
    for ly in layers:
        lk.lookat_probe_stream_read(ly.values, sink)
    torch.cuda.synchronize()
    e0.record()
    for i in range(n_launch):
        lk.lookat_probe_stream_read(layers[i % cfg.layers].values, sink)
    e1.record()
    torch.cuda.synchronize()
    stream_us = e0.elapsed_time(e1) * 1e3 / n_launch
    stream_gbs = layers[0].values.numel() * 2 / stream_us / 1e3

    probes = None
    if args.probes:
        probes = run_probes(torch, lk, cfg, layers, scale, sink, time_launches, n_launch)

    result = {
        "metric": "LUT-attention decode keys scored/sec/GPU; achieved HBM GB/s vs peak",
        "value": value,
        "unit": "keys/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: B={cfg.B} H={cfg.H} L={cfg.L} d_k={cfg.d_k} m={cfg.m} K={cfg.K} "
                        f"layers={cfg.layers}; per layer encode(1 new key) + build_lut + attend_decode",
            "path": ("lookat_decode_step_split (fused ranges + merge per layer)" if fused_split
                     else "lookat_decode_step (one fused kernel per layer)") if fused
                    else "lookat_encode_keys + lookat_build_lut + lookat_attend_decode",
            "values": "fp16", "codes": "u8 (" + args.codes + ")", "lut": "f32", "launch": launch, "num_splits": splits,
            "codebooks": f"{args.kmeans_iters} Lloyd iterations (lookat_kmeans_step) on {cfg.n_calib} seeded "
                         "calibration keys per head",
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "lookat::decode_split_kernel" + ((" (fused step instance, two batch entries of a head per workgroup)"
                                                         if paired else " (fused step instance)") if fused else ""),
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if args.batch else counted_traffic((cfg.name, fused), launch_shape),
            "bytes_per_launch": bytes_per_launch,
            "us_per_launch": us_per_launch,
            "us_per_launch_median": stats["median"],
            "us_per_launch_min": stats["min"],
            "us_per_launch_max": stats["max"],
            "median_min_max_over": f"{stats['batches']} batches of {stats['launches_per_batch']} back-to-back launches",
            "launches_timed": n_launch,
            "attend_decode_alone_us": us_decode_alone,
            "attend_decode_alone_us_median": stats_alone["median"],
            "attend_decode_alone_us_min": stats_alone["min"],
            "attend_decode_alone_GBs": bytes_per_launch / us_decode_alone / 1e3,
            "read_stream_GBs": stream_gbs,
            "frac_of_read_stream": achieved / stream_gbs,
        },
    }

    if probes is not None:
        result["probes"] = probes
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, layers, scale, args.cpu_seconds)
    print(json.dumps(result), flush=True)


def run_probes(torch, lk, cfg, layers, scale, sink, time_launches, n_launch):
    """The measurement aids on this workload's buffers (per-launch microseconds, back to back on one stream)."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def loop(fn, n):
        fn(0)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n

    out = {"empty_launch_us": {f"{wg}x{th}": loop(lambda i: lk.lookat_probe_empty_launch(wg, th), 2000)
                               for wg, th in ((1, 256), (cfg.B * cfg.H, 256), (4 * cfg.B * cfg.H, 256))}}
    vbytes = layers[0].values.numel() * 2
    shapes = [(256, 2, 0, False), (256, 1, 0, False), (256, 4, 0, False), (512, 2, 0, False), (128, 2, 0, False),
              (256, 8, 768, False), (256, 8, 1536, False), (512, 8, 512, False), (1024, 8, 256, False), (1024, 4, 256, False),
              (256, 8, 768, True), (512, 8, 512, True), (1024, 8, 256, True), (256, 16, 768, False)]
    sweep = {}
    for th, loads, wgs, contig in shapes:
        us = loop(lambda i: lk.lookat_probe_stream_read_shaped(layers[i % len(layers)].values, sink, th, loads, wgs, contig, True),
                  n_launch // 4)
        sweep[f"{th} threads x {loads} loads, " + (f"{wgs} persistent workgroups" + (", contiguous shares" if contig else ", grid-strided")
                                                    if wgs else "one round")] = round(vbytes / us / 1e3, 1)
    out["read_stream_GBs_by_launch_shape"] = sweep
    out["read_stream_best_GBs"] = max(sweep.values())
    # the same bare read in the launch geometries of the decode kernels (contiguous shares, 8 loads in flight per
    # thread): what those geometries cost before any attention arithmetic
    BH = cfg.B * cfg.H
    geoms = [(f"{BH} x 256 threads (lookat_attend_decode: one (b,h) per workgroup)", 256, BH),
             (f"{BH} x 512 threads (fused step, one (b,h) per workgroup)", 512, BH),
             (f"{2 * BH} x 256 threads (two shares per (b,h))", 256, 2 * BH),
             (f"{4 * BH} x 256 threads (four shares per (b,h))", 256, 4 * BH)]
    if BH % 2 == 0:
        geoms.insert(2, (f"{BH // 2} x 1024 threads (fused step, two batch entries per workgroup)", 1024, BH // 2))
    out["read_stream_us_in_kernel_geometries"] = {
        name: round(loop(lambda i: lk.lookat_probe_stream_read_shaped(layers[i % len(layers)].values, sink, th, 8, wgs, True, True),
                         n_launch // 4), 2)
        for name, th, wgs in geoms}
    # attention with the in-kernel ticket merge against the two-launch path, ranges chosen by each
    ws = torch.zeros(max(16, lk.probe_attend_decode_ticket_workspace_bytes(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L, 0)),
                     dtype=torch.uint8, device=layers[0].values.device)
    pieces = {}

    def ticket(ly, splits=0):
        _, pieces[splits] = lk.lookat_probe_attend_decode_ticket(ly.lut.view(cfg.B, cfg.H, cfg.m, cfg.K), ly.codes, ly.values,
                                                                  scale, num_splits=splits, workspace=ws, out=ly.out)

    ref = lk.lookat_attend_decode(layers[0].lut.view(cfg.B, cfg.H, cfg.m, cfg.K), layers[0].codes, layers[0].values, scale).clone()
    ticket(layers[0])
    torch.cuda.synchronize()
    out["ticket_merge"] = {
        "us_per_launch_equal_shares": time_launches(ticket),
        "pieces_per_bh_equal_shares": pieces[0],
        "max_abs_diff_vs_lookat_attend_decode": float((layers[0].out - ref).abs().max()),
    }
    if cfg.B * cfg.H >= 256:   # the same kernel with one whole (b,h) per workgroup: nothing to merge
        out["ticket_merge"]["us_per_launch_one_range"] = time_launches(lambda ly: ticket(ly, 1))
    # the fused step with one and with two batch entries of a head per workgroup (two: the codebook is fetched
    # once per pair); lookat_decode_step takes `library_choice` of them
    if cfg.B % 2 == 0 and ((cfg.d_k == 64 and cfg.m in (2, 4, 8, 16)) or (cfg.d_k == 128 and cfg.m in (4, 8, 16))) \
            and hasattr(layers[0], "q_step"):
        ly0 = layers[0]
        one = lk.lookat_probe_decode_step_entries(1, ly0.q_step, ly0.k_step, ly0.cb, ly0.codes, ly0.values, scale).clone()
        two = lk.lookat_probe_decode_step_entries(2, ly0.q_step, ly0.k_step, ly0.cb, ly0.codes, ly0.values, scale)
        torch.cuda.synchronize()
        out["decode_step_entries_per_workgroup"] = {
            "library_choice": lk.decode_step_entries_per_workgroup(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L),
            "us_per_launch_one": time_launches(lambda ly: lk.lookat_probe_decode_step_entries(
                1, ly.q_step, ly.k_step, ly.cb, ly.codes, ly.values, scale, out=ly.out)),
            "us_per_launch_two": time_launches(lambda ly: lk.lookat_probe_decode_step_entries(
                2, ly.q_step, ly.k_step, ly.cb, ly.codes, ly.values, scale, out=ly.out)),
            "max_abs_diff_two_vs_one": float((two - one).abs().max()),
        }
    return out


def gqa_main(args, cfg, lk, li, torch, device):
    """Decode step with grouped queries: the workload's H query heads share H/group key/value heads.
    Per layer: encode the new key of every key/value head, build the tables of every query head
    (against its key/value head's codebooks), lookat_attend_decode_gqa.  One JSON line; the roofline
    is the grouped decode kernel against the key/value bytes it streams (once for the whole group)."""
    g = args.group
    if cfg.H % g:
        raise SystemExit(f"--group {g} does not divide the workload's {cfg.H} heads")
    kv = li.shrink(cfg, H=cfg.H // g)
    scale = 1.0 / math.sqrt(cfg.d_k)
    gen = torch.Generator(device=device)
    gen.manual_seed(li.BASE_SEED + 977)
    layers = []
    for i in range(cfg.layers):
        ly = Layer(lk, li, kv, device, i, args.kmeans_iters)
        ly.cb_q = ly.cb.repeat_interleave(g, dim=0).contiguous()     # codebooks as each query head sees them
        ly.q = (torch.randn((cfg.B, cfg.H, 1, cfg.d_k), generator=gen, device=device) / 8).to(ly.q.dtype)
        ly.lut = torch.empty((cfg.B, cfg.H, 1, cfg.m, cfg.K), dtype=torch.float32, device=device)
        ly.out = torch.empty((cfg.B, cfg.H, cfg.d_k), dtype=torch.float32, device=device)
        layers.append(ly)
    splits = 0   # the library's choice for grouped queries
    ws = torch.empty(max(16, lk.attend_decode_gqa_workspace_bytes(kv.B, kv.H, g, kv.d_k, kv.m, kv.L, 0)),
                     dtype=torch.uint8, device=device)

    def decode_only(ly):
        lk.lookat_attend_decode_gqa(ly.lut.view(cfg.B, cfg.H, cfg.m, cfg.K), ly.codes, ly.values, scale,
                                    num_splits=splits, workspace=ws, out=ly.out)

    fused = args.path != "calls"
    for ly in layers:
        ly.q_step = ly.q[:, :, 0].to(ly.k_step.dtype).contiguous()

    def fused_only(ly):
        lk.lookat_decode_step_gqa(ly.q_step, ly.k_step, ly.cb, ly.codes, ly.values, scale, num_splits=0,
                                  workspace=ws, out=ly.out)

    def step():
        for ly in layers:
            if fused:
                fused_only(ly)
            else:
                lk.lookat_encode_keys(ly.new_key, ly.cb, cache=ly.codes, position=cfg.L - 1)
                lk.lookat_build_lut(ly.q, ly.cb_q, lut_out=ly.lut)
                decode_only(ly)

    step()
    for ly in layers:   # (the fused step keeps its tables on chip; the checks and the unfused loop below need them)
        lk.lookat_build_lut(ly.q, ly.cb_q, lut_out=ly.lut)
    torch.cuda.synchronize()
    # the grouped kernel against the plain kernel on caches repeated per query head (layer 0)
    ly = layers[0]
    ref = lk.lookat_attend_decode(ly.lut.view(cfg.B, cfg.H, cfg.m, cfg.K),
                                  ly.codes.repeat_interleave(g, dim=1).contiguous(),
                                  ly.values.repeat_interleave(g, dim=1).contiguous(), scale)
    max_diff = float((ref - ly.out).abs().max())
    del ref
    graph = None
    if args.mode != "eager":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
    run_step, launch = pick_launch_mode(args.mode, step, graph.replay if graph is not None else None)
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_launch = max(args.steps, 20) * cfg.layers

    def time_launches(fn):
        for ly in layers:
            fn(ly)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n_launch):
            fn(layers[i % cfg.layers])
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n_launch

    us_unfused = time_launches(decode_only)
    us = time_launches(fused_only) if fused else us_unfused
    kv_bytes = kv.B * kv.H * kv.L * (kv.m + 2 * kv.d_k)
    scores_per_step = cfg.layers * cfg.B * cfg.H * cfg.L
    print(json.dumps({
        "metric": "LUT-attention decode with grouped queries: (query head, key) scores/sec/GPU; achieved HBM GB/s vs peak",
        "value": scores_per_step * args.steps / elapsed, "unit": "keys/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": elapsed * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name} with grouped queries: B={cfg.B} query heads={cfg.H} key/value heads={kv.H} "
                               f"(group={g}) L={cfg.L} d_k={cfg.d_k} m={cfg.m} layers={cfg.layers}; per layer "
                               "encode(1 new key) + build_lut + attend_decode_gqa",
                   "path": "lookat_decode_step_gqa (fused ranges + merge per layer)" if fused
                           else "lookat_encode_keys + lookat_build_lut + lookat_attend_decode_gqa",
                   "launch": launch, "num_splits": "library choice"},
        "roofline": {"bound": "hbm", "kernel": f"lookat::decode_split_kernel (group of {g} query heads"
                                               + (", fused step)" if fused else ")"),
                     "achieved": kv_bytes / us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": kv_bytes / us / 1e3 / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": kv_bytes,
                     "us_per_launch": us, "launches_timed": n_launch,
                     "attend_decode_gqa_alone_us": us_unfused,
                     "query_head_bytes_equivalent_GBs": kv_bytes * g / us / 1e3,
                     "max_abs_diff_vs_ungrouped_kernel": max_diff},
    }), flush=True)


def prefill_main(args, cfg, lk, li, torch, device):
    """Prefill block (configuration C4): a step = encode the block's keys, build every query's tables
    as a materialised array (matrix cores), score the causal block (the library's choice of kernel: for
    fp16 queries the dense product against the keys' centroids on the matrix cores).  One JSON line with
    the step rate and one roofline entry per kernel."""
    import numpy as np

    case = li.torch_case(cfg, device, layer=0)
    cb = lk.lookat_kmeans(case["calib"], case["cb_init"], args.kmeans_iters)
    keys, q = case["keys"], case["q"]
    codes = torch.empty((cfg.B, cfg.H, cfg.L, cfg.m), dtype=torch.uint8, device=device)
    lut = torch.empty((cfg.B, cfg.H, cfg.T, cfg.m, cfg.K), dtype=torch.float32, device=device)
    scores = torch.empty((cfg.B, cfg.H, cfg.T, cfg.L), dtype=torch.float32, device=device)
    calls = {
        "encode_keys": lambda: lk.lookat_encode_keys(keys, cb, codes_out=codes),
        "build_lut": lambda: lk.lookat_build_lut(q, cb, lut_out=lut),
        "score_prefill": lambda: lk.lookat_score_prefill(q, cb, codes, scores_out=scores),
    }
    # the lookup-and-sum scoring kernel on the same inputs (the library scores blocks of fp16 queries as a
    # dense product on the matrix cores): timed beside the step, not part of it
    extra_calls = {"score_prefill_lookup": lambda: lk.lookat_probe_score_prefill_lookup(q, cb, codes, scores_out=scores)}

    def step():
        for fn in calls.values():
            fn()

    for _ in range(max(1, args.warmup)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    us = {}
    for name, fn in list(calls.items()) + list(extra_calls.items()):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us[name] = e0.elapsed_time(e1) * 1e3 / args.steps

    # plain write stream over the table buffer: what the HBM write path delivers
    lk.lookat_probe_stream_write(lut, 0)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        lk.lookat_probe_stream_write(lut, 0)
    e1.record()
    torch.cuda.synchronize()
    write_stream_gbs = lut.numel() * 4 / (e0.elapsed_time(e1) * 1e3 / args.steps) / 1e3
    BH, nk = cfg.B * cfg.H, cfg.B * cfg.H * cfg.L
    pairs = BH * (cfg.T * (cfg.T + 1) // 2 + cfg.T * (cfg.L - cfg.T))        # visible (query, key) pairs
    enc_ops = nk * cfg.d_k * cfg.K * 3                                          # sub, mul, add in fp64 per (key, centroid, coordinate)
    lut_bytes = lut.numel() * 4
    lut_flops = BH * cfg.T * cfg.d_k * cfg.K * 2
    lds_bytes = pairs * cfg.m * 4                                               # 4 bytes of table per (query, key, subspace)
    score_bytes = scores.numel() * 4
    LDS_PEAK = 256 * 256 * 2.4e9 / 1e9                                          # 256 CUs x 256 B/clk (16-byte reads, measured 186) x 2.4 GHz, GB/s
    VALU_PEAK = 256 * 4 * 16 * 2.4e9 / 1e12                                     # single-operation fp32 lane-instructions, T/s
    cand = nk * cfg.m * cfg.K                                                   # candidates ranked by the encoder's filter
    d_sub = cfg.d_k // cfg.m
    result = {
        "metric": "LOOKAT prefill block: causal (query,key) pairs scored/sec/GPU",
        "value": pairs * args.steps / elapsed,
        "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B} H={cfg.H} T=L={cfg.L} d_k={cfg.d_k} m={cfg.m} K={cfg.K}; "
                               "encode_keys (fp16 keys) + build_lut (T queries per head, materialised) + score_prefill"},
        "roofline": {"bound": "hbm", "kernel": "lookat::score_prefill_dense_kernel (scores written; fp16 matrix cores on the "
                                               "keys' centroids)",
                     "achieved": score_bytes / us["score_prefill"] / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": score_bytes / us["score_prefill"] / 1e3 / HBM_PEAK_GBS,
                     "traffic": counted_traffic((cfg.name, "score_prefill_dense")),
                     "us_per_launch": us["score_prefill"], "bytes_per_launch": score_bytes,
                     "mfma_TFLOPs": pairs * cfg.d_k * 2 * 2 / us["score_prefill"] / 1e6,   # hi and lo term of every product
                     "mfma_peak_fp16_TFLOPs": 2500.0,
                     "write_stream_GBs": write_stream_gbs},
        "kernels": {
            "score_prefill_kernel (lookup-and-sum in LDS, forced; not part of the step)": {
                "bound": "hbm", "us": us["score_prefill_lookup"], "achieved": score_bytes / us["score_prefill_lookup"] / 1e3,
                "peak": HBM_PEAK_GBS, "unit": "GB/s (scores written)",
                "frac": score_bytes / us["score_prefill_lookup"] / 1e3 / HBM_PEAK_GBS,
                "traffic": counted_traffic((cfg.name, "score_prefill")),
                "lds_gather_GBs": lds_bytes / us["score_prefill_lookup"] / 1e3, "lds_peak_GBs": LDS_PEAK},
            "encode_filter_kernel": {"bound": "alu", "us": us["encode_keys"],
                                     "achieved": cand * 4 / us["encode_keys"] / 1e6, "peak": VALU_PEAK,
                                     "unit": "T lane-instructions/s (4 vector instructions per (key, subspace, centroid) "
                                             "candidate: compare, two selects, median; peak 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz)",
                                     "frac": cand * 4 / us["encode_keys"] / 1e6 / VALU_PEAK,
                                     "mfma_TFLOPs": cand * d_sub * 4 / us["encode_keys"] / 1e6,
                                     "mfma_peak_fp16_TFLOPs": 2500.0,
                                     "exact_fp64_scan_equivalent_Top_s": enc_ops / us["encode_keys"] / 1e6},
            "build_lut_mfma_kernel": {"bound": "hbm", "us": us["build_lut"], "achieved": lut_bytes / us["build_lut"] / 1e3,
                                      "peak": HBM_PEAK_GBS, "unit": "GB/s (table written)",
                                      "frac": lut_bytes / us["build_lut"] / 1e3 / HBM_PEAK_GBS,
                                      "mfma_TFLOPs": lut_flops / us["build_lut"] / 1e6, "mfma_peak_fp32_TFLOPs": 157.3},
        },
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = prefill_cpu_baseline(cfg, keys, q, cb, codes, scores, args.cpu_seconds)
    print(json.dumps(result), flush=True)


def prefill_cpu_baseline(cfg, keys, q, cb, codes, scores, budget_s):
    """The CPU oracle on one batch entry of the block, a few heads: encode, tables, causal scoring;
    checks the GPU's codes and scores of those heads against it."""
    import numpy as np

    import oracle

    nh = 2
    k = keys[0:1, :nh].cpu().numpy()
    qq = q[0:1, :nh].cpu().numpy()
    cbn = cb[:nh].cpu().numpy()
    t0 = time.perf_counter()
    c_ref = oracle.encode_keys(k, cbn)
    lut = oracle.build_lut(qq, cbn)
    s_ref = oracle.score_prefill(lut, c_ref)
    dt = time.perf_counter() - t0
    pairs = nh * (cfg.T * (cfg.T + 1) // 2 + cfg.T * (cfg.L - cfg.T))
    codes_ok = bool(np.array_equal(codes[0:1, :nh].cpu().numpy(), c_ref))
    got = scores[0:1, :nh].cpu().numpy()
    vis = np.isfinite(s_ref)
    err = float(np.max(np.abs(np.where(vis, got, 0.0) - np.where(vis, s_ref, 0.0))))
    return {"value": pairs / dt, "unit": "pairs/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"batch entry 0, heads 0..{nh - 1} of {cfg.H}: encode {cfg.L} keys, tables of {cfg.T} queries, "
                      "causal scoring; fp64, one pass",
            "codes_bit_exact_vs_oracle": codes_ok, "max_abs_score_diff_gpu_vs_oracle": err}


def cpu_baseline(cfg, layers, scale, budget_s):
    """The CPU oracle as it stands, on the same arrays the GPU consumed: the same three calls
    (encode the new key, build the tables, attend) on whole (b,h) slabs of the first layer, as many
    (b,h) pairs as fit the time budget, on all host cores (OpenMP over (b,h)) and on one thread.
    Also checks the GPU output on that sample."""
    import numpy as np

    import oracle

    ly = layers[0]
    BH = cfg.B * cfg.H
    threads = oracle.num_threads()
    cb = ly.cb.cpu().numpy()
    gpu_out = ly.out.cpu().numpy().reshape(BH, cfg.d_k)
    flat = lambda t: t.reshape((BH,) + tuple(t.shape[2:]))
    codes_d, values_d, q_d, key_d = flat(ly.codes), flat(ly.values), flat(ly.q), flat(ly.new_key)

    def slab(n):
        """Host copies of the first n (b,h) pairs (b-major: whole batch entries first), as [1, n, ...] arrays
        with the codebooks of their heads."""
        idx = np.arange(n)
        return (codes_d[:n].cpu().numpy()[None], values_d[:n].cpu().numpy()[None], q_d[:n].cpu().numpy()[None],
                key_d[:n].cpu().numpy()[None], np.ascontiguousarray(cb[idx % cfg.H]))

    def once(arrs):
        codes, values, q, new_key, cbn = arrs
        c = codes.copy()
        c[:, :, cfg.L - 1:cfg.L] = oracle.encode_keys(new_key, cbn)
        lut = oracle.build_lut(q, cbn)
        return oracle.attend_decode(lut[:, :, 0], c, values, scale)

    def timed(n, budget):
        arrs = slab(n)
        reps = 0
        t0 = time.perf_counter()
        while True:
            out = once(arrs)
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= budget or reps >= 50:
                return out, reps, dt

    # size the sample: time one (b,h) pair per thread, then take as many pairs as fit the budget
    probe = min(BH, threads)
    t0 = time.perf_counter()
    once(slab(probe))
    t1 = time.perf_counter() - t0
    n = int(max(probe, min(BH, probe * budget_s / max(t1, 1e-6) / 4)))
    out, reps, dt = timed(n, min(budget_s / 2, 2.0))
    err = float(np.max(np.abs(out[0] - gpu_out[:n])))
    # one thread: a share of the same sample sized to a few seconds
    n1 = int(max(1, min(n, n / max(threads, 1) * 2)))
    oracle.set_num_threads(1)
    try:
        _, reps1, dt1 = timed(n1, min(budget_s / 4, 2.0))
    finally:
        oracle.set_num_threads(threads)
    return {
        "value": reps * n * cfg.L / dt,
        "unit": "keys/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"layer 0, the first {n} of {BH} (b,h) pairs (whole slabs, L={cfg.L}), {reps} repetitions, fp64, "
                  f"OpenMP over (b,h); one thread: the first {n1} pairs, {reps1} repetitions",
        "single_thread_value": reps1 * n1 * cfg.L / dt1,
        "max_abs_diff_gpu_vs_oracle": err,
    }


if __name__ == "__main__":
    main()
