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
# WRITE_SIZE, recorded under profiles/*_hbm_counters.md).  Entry: (FETCH_SIZE per dispatch,
# FETCH_SIZE of lookat::stream_read_kernel in the same run, KiB that kernel reads, WRITE_SIZE
# per dispatch in KiB).  bytes = (fetch * known_KiB / stream_fetch + write) * 1024.
COUNTED_TRAFFIC = {
    ("C1", True): (1249.5, 776.004, 1536.0, 3.375),
    ("C1", False): (826.5, 776.004, 1536.0, 3.0),
    ("C2", True): (26393.0, 24584.0, 49152.0, 108.0),
    ("C2", False): (26144.5, 24584.0, 49152.0, 96.0),
    ("C3", True): (1.0838e6, 1.04858e6, 2097152.0, 136.0),
    ("C3", False): (1.08264e6, 1.04858e6, 2097152.0, 268.0),
    ("C4", "score_prefill"): (37033.6, 1.0, 2.0, 2.10989e6),   # FETCH_SIZE at 2 KiB per count (calibration of the 2 GiB read)
}


def counted_traffic(key):
    if key not in COUNTED_TRAFFIC:
        return None
    fetch, stream_fetch, known_kib, write_kib = COUNTED_TRAFFIC[key]
    return int(round((fetch * known_kib / stream_fetch + write_kib) * 1024.0))


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
            "kernel": "lookat::decode_split_kernel" + (" (fused step instance)" if fused else ""),
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if args.batch else counted_traffic((cfg.name, fused)),
            "bytes_per_launch": bytes_per_launch,
            "us_per_launch": us_per_launch,
            "launches_timed": n_launch,
            "attend_decode_alone_us": us_decode_alone,
            "attend_decode_alone_GBs": bytes_per_launch / us_decode_alone / 1e3,
            "read_stream_GBs": stream_gbs,
            "frac_of_read_stream": achieved / stream_gbs,
        },
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, layers, scale, args.cpu_seconds)
    print(json.dumps(result), flush=True)


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
    as a materialised array (matrix cores), score the causal block from on-chip tables.  One JSON
    line with the step rate and one roofline entry per kernel."""
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
    for name, fn in calls.items():
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
        "roofline": {"bound": "hbm", "kernel": "lookat::score_prefill_kernel (scores written; its LDS and vector floors are lower)",
                     "achieved": score_bytes / us["score_prefill"] / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": score_bytes / us["score_prefill"] / 1e3 / HBM_PEAK_GBS,
                     "traffic": counted_traffic((cfg.name, "score_prefill")),
                     "us_per_launch": us["score_prefill"], "bytes_per_launch": score_bytes,
                     "lds_gather_GBs": lds_bytes / us["score_prefill"] / 1e3, "lds_peak_GBs": LDS_PEAK,
                     "write_stream_GBs": write_stream_gbs},
        "kernels": {
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
    (encode the new key, build the tables, attend) on whole (b,h) slabs of the first layer,
    as many batch entries as fit the time budget.  Also checks the GPU output on that sample."""
    import numpy as np

    import oracle

    ly = layers[0]
    nb = cfg.B
    codes = ly.codes.cpu().numpy()
    values = ly.values.cpu().numpy()
    q = ly.q.cpu().numpy()
    cb = ly.cb.cpu().numpy()
    new_key = ly.new_key.cpu().numpy()
    gpu_out = ly.out.cpu().numpy()
    threads = oracle.num_threads()

    def once(n):
        c = codes[:n].copy()
        c[:, :, cfg.L - 1:cfg.L] = oracle.encode_keys(new_key[:n], cb)
        lut = oracle.build_lut(q[:n], cb)
        return oracle.attend_decode(lut[:, :, 0], c, values[:n], scale)

    # size the sample: time one batch entry, then take as many as fit the budget
    t0 = time.perf_counter()
    once(1)
    t1 = time.perf_counter() - t0
    n = int(max(1, min(nb, budget_s / max(t1, 1e-6) / 2)))
    reps = 0
    t0 = time.perf_counter()
    while True:
        out = once(n)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= min(budget_s, 2.0) or reps >= 50:
            break
    keys = reps * n * cfg.H * cfg.L
    err = float(np.max(np.abs(out - gpu_out[:n])))
    return {
        "value": keys / dt,
        "unit": "keys/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"layer 0, batch entries 0..{n - 1} of {cfg.B} (all {cfg.H} heads, L={cfg.L}), "
                  f"{reps} repetitions, fp64, OpenMP over (b,h)",
        "max_abs_diff_gpu_vs_oracle": err,
    }


if __name__ == "__main__":
    main()
