#!/usr/bin/env python3
"""Benchmark of the cache-hit re-attachment path on one MI355X.

A *step* is one pass of the whole hot path -- irm_cdc_chunk, irm_chunk_hash,
irm_lookup, irm_reattach, back to back on one stream with device-side counts --
over one synthetic request batch whose inputs are already resident in HBM.
Several batch variants against the same pool are cycled so that consecutive
steps do not re-read the same rows from the last-level cache.

Prints ONE JSON line: whole-path re-attached tokens/s (``value``), the achieved
HBM bandwidth of the re-attach row kernel against the 8 TB/s peak
(``roofline``), and the CPU oracle timed on this machine's host cores
(``cpu_baseline``).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

ROW_BYTES = 1152                                     # bf16 rows; main() takes the format's own size
HBM_PEAK_GBS = 8000.0


def build_parser() -> argparse.ArgumentParser:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: per workload, see DEFAULTS)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c4",
                    help="c0..c4; the headline is c4, the largest configuration that fits one GPU (61 layers, "
                         "32 x 65,536 tokens, the whole serve path on one stream)")
    ap.add_argument("--size", default="full", choices=["full", "small"])
    ap.add_argument("--variants", type=int, default=None, help="request batches cycled through (default: per workload)")
    ap.add_argument("--cdc", default="config", choices=["config", "paper"],
                    help="CDC rule: config = the measured configurations' (mask 0xFF, chunks of 64..1024 tokens); "
                         "paper = the paper's own (Sec. 7.2, App. B: mask 0x7F, chunks of 32..512 tokens)")
    ap.add_argument("--secondary", default=None,
                    help="comma-separated workloads measured after the headline in the same process and reported in "
                         "the 'secondary' block of the JSON line, each as name or name:paper (default with the c4 "
                         "headline: c1,c2,c3,c1:paper; '' = none)")
    ap.add_argument("--slots", default="contiguous", choices=["contiguous", "permuted"])
    ap.add_argument("--layers", type=int, default=0,
                    help="layer count of the pools instead of the configuration's own (0 = its own): the same "
                         "batches over fewer or more layers, to separate a launch's fixed cost from its per-layer cost")
    ap.add_argument("--grid", type=int, default=0, help="workgroups of the row kernel (0 = library default)")
    ap.add_argument("--reattach", default="full", choices=["full", "kr", "kr-dense", "ref"],
                    help="full = c_KV copied + k_r rotated (the headline); kr = split-pool variant, "
                         "only the k_r slice is materialised (256 B per token and layer), read from "
                         "the packed 576-wide source rows; kr-dense = the same from a dense k_r_base pool; ref = "
                         "no-materialise variant, only row references and the per-hit rotation table are written "
                         "(8 B per token, once, not per layer)")
    ap.add_argument("--rows", default="bf16", choices=["bf16", "fp8"],
                    help="row format of the pools: bf16 = 1152-byte rows (the headline); fp8 = 656-byte rows, c_KV "
                         "as 512 e4m3 bytes and four fp32 scales moved bit for bit, k_r in bf16 rotated as usual "
                         "(hit stage with --reattach full or kr, admit stage, attend stage: c_KV dequantised on load)")
    ap.add_argument("--row-stride", type=int, default=0, metavar="BYTES",
                    help="hit stage, --reattach full: row stride of both pools in bytes, a multiple of 16 "
                         "(0 = packed rows; 768 puts every fp8 row on its own 128-byte lines)")
    ap.add_argument("--heads", type=int, default=16, help="attend stage: query rows per request, a multiple of 16 "
                                                              "(heads, or new tokens x heads over a cached prefix)")
    ap.add_argument("--linear-rows", action="store_true",
                    help="attend stage: every slot refers to the pool row of the same number (no rotation), i.e. "
                         "purely sequential reads: the yardstick for what the gather pattern costs")
    ap.add_argument("--splits", type=int, default=8, help="attend stage: workgroups per request and 16 heads")
    ap.add_argument("--stage", default="hit", choices=["hit", "admit", "s1", "attend", "yardstick"],
                    help="hit = the cache-hit path (the headline); admit = the miss path on a cold registry: "
                         "every chunk of the batch is copied from the request pool into the shared pool and "
                         "registered (irm_admit alone is timed, with events on its stream); s1 = the hit path "
                         "on UNALIGNED batches followed by the S1 fallback (128-token windows inside the chunks "
                         "that missed, end-anchored): eight calls per step; attend = the no-materialise scheme end to end: "
                         "front end + irm_reattach_ref once, then irm_attend_ref (decode attention over the "
                         "references, k_r rotated on load) on every layer; yardstick = no part of the path: plain read-only, "
                         "write-only and copy streams over 9 GiB in a sweep of launch shapes (irm_yardstick), the "
                         "bandwidth this machine gives a kernel that only moves bytes")
    ap.add_argument("--streams", type=int, default=1,
                    help="batches in flight: step k runs on stream k mod S with its own context and destination "
                         "pool, so the front end of one batch overlaps the row kernel of another (hit and s1 "
                         "stages with --reattach full; --variants must be a multiple of S)")
    ap.add_argument("--graph", action="store_true",
                    help="capture each batch variant's step in a HIP graph once and replay it in the timed loop "
                         "(no per-kernel events then, so no roofline figure); pays off where the step is "
                         "launch-bound (c0)")
    ap.add_argument("--tune", default="", help="comma-separated knob=value pairs for irm_ctx_tune (sweeps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", type=int, default=0, metavar="N",
                    help="also run N plain 1 GiB copies (irm_calibrate_copy) before the timed loop: the "
                         "known-traffic yardstick for hardware counters")
    ap.add_argument("--kernel-timing", type=int, default=None, metavar="E",
                    help="HIP events around every E-th row-kernel launch of each batch variant inside the "
                         "timed region (0 = none, no roofline; default: every 4th on c0 and c1, whose launches "
                         "take a fraction of a millisecond, every launch on the larger workloads)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU budget of the oracle baseline")
    ap.add_argument("--extras", default=None,
                    help="'all' or '': after the headline and the secondary workloads, also run the path's other "
                         "variants (split pool, fp8 rows, miss path, S1 fallback, rotate-on-load attention) and "
                         "report them in the 'other_paths' block (default with the c4 headline: all)")
    return ap


def main() -> int:
    args = build_parser().parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path is built and measured on ONE GPU; --gpus above 1 is not supported "
              "(it would shard by layer or by request, with no exchange step)", file=sys.stderr)
        return 2

    if args.stage == "yardstick":
        print(json.dumps(bench_yardstick(args)), flush=True)
        return 0
    plain = (args.stage == "hit" and args.reattach == "full" and args.rows == "bf16" and args.streams == 1
             and not args.graph and not args.row_stride and args.size == "full")
    if args.secondary is None:
        args.secondary = "c1,c2,c3,c1:paper" if plain and args.workload == "c4" and args.cdc == "config" else ""
    out = run(with_defaults(args, args.workload, args.cdc, args.steps, args.warmup, args.variants))
    if args.secondary:
        assert plain, "--secondary goes with the plain hit path (bf16 rows, one stream)"
        out["secondary"] = []
        for item in filter(None, args.secondary.split(",")):
            name, _, cdc = item.partition(":")
            try:
                sub = run(with_defaults(args, name, cdc or "config", None, None, None, cpu=False))
            except Exception as exc:                             # the headline is printed whatever happens here
                out["secondary"].append({"workload": item, "error": f"{type(exc).__name__}: {exc}"})
                continue
            out["secondary"].append({"workload": sub["config"]["workload"], "steps": sub["steps"],
                                     "ms_per_step": sub["ms_per_step"], "value": sub["value"], "unit": sub["unit"],
                                     "hit_tokens_per_step": sub["config"]["hit_tokens_per_step"],
                                     "hits_per_step": sub["config"]["hits_per_step"],
                                     "roofline": sub["roofline"]})
    if args.extras is None:
        args.extras = "all" if plain and args.workload == "c4" and args.cdc == "config" and args.secondary else ""
    if args.extras:
        out["other_paths"] = []
        for flags in EXTRAS:
            a = with_defaults(args, flags.get("workload", "c2"), "config", flags.get("steps"), flags.get("warmup"),
                              flags.get("variants"), cpu=False)
            for k, v in flags.items():
                setattr(a, k, v)
            try:
                sub = run(a)
            except Exception as exc:
                out["other_paths"].append({"what": flags["what"], "error": f"{type(exc).__name__}: {exc}"})
                continue
            out["other_paths"].append({"what": flags["what"], "metric": sub["metric"], "workload": sub["config"]["workload"],
                                       "steps": sub["steps"], "ms_per_step": sub["ms_per_step"], "value": sub["value"],
                                       "unit": sub["unit"], "roofline": sub["roofline"]})
    print(json.dumps(out), flush=True)
    return 0


# the path's other variants, each a set of flags of this script (one short run each)
EXTRAS = [
    dict(what="split pool, k_r only, packed source rows", workload="c2", reattach="kr", steps=24, warmup=4),
    dict(what="split pool, k_r only, dense k_r_base source", workload="c2", reattach="kr-dense", steps=24, warmup=4),
    dict(what="no-materialise variant: references and rotation table only", workload="c2", reattach="ref", steps=40, warmup=5),
    dict(what="fp8 pool rows (656 B)", workload="c2", rows="fp8"),
    dict(what="fp8 pool rows (656 B), 32 K-token request", workload="c1", rows="fp8"),
    dict(what="two batches in flight on two streams (the front end of one hides behind the other's row kernel; "
              "the kernel columns then span both streams and say nothing)", workload="c1", streams=2),
    dict(what="miss path, irm_admit alone", workload="c2", stage="admit", steps=8, warmup=2),
    dict(what="hit path + S1 window fallback on unaligned batches", workload="c1", stage="s1"),
    dict(what="rotate-on-load decode attention over the references, 16 heads", workload="c2", stage="attend",
         splits=4, steps=6, warmup=2),
]


# per workload: timed steps, warm-up steps, request batches cycled (sized so that every run takes seconds)
DEFAULTS = {"c0": (200, 20, 1), "c1": (200, 20, 8), "c2": (12, 3, 2), "c3": (60, 6, 2), "c4": (20, 5, 1)}


def with_defaults(args, name, cdc, steps, warmup, variants, cpu=True):
    import copy
    a = copy.copy(args)
    d = DEFAULTS[name]
    a.workload, a.cdc = name, cdc
    a.steps = d[0] if steps is None else steps
    a.warmup = d[1] if warmup is None else warmup
    a.variants = d[2] if variants is None else variants
    if a.kernel_timing is None:
        a.kernel_timing = 4 if name in ("c0", "c1") else 1
    if not cpu:
        a.no_cpu_baseline = True
    return a


def run(args) -> dict:
    """One workload through the stage the flags name; returns the result record."""
    import gc
    import torch
    from paper_2605_05696_amd import binding as B
    from paper_2605_05696_amd import workloads as wl
    from paper_2605_05696_amd.pipeline import Session

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    gc.collect()
    torch.cuda.empty_cache()
    name = args.workload
    dims = wl.CONFIGS[name][args.size]
    mask, min_chunk, max_chunk = wl.CDC_RULES[args.cdc]

    # ---- inputs: chunked and fingerprinted by the library itself -------------
    max_stream = max(dims["pool"], dims.get("n_req", 1) * dims.get("req_len", dims["pool"]) * 2 + 16384)
    gear = wl.gear_table()
    front = Session(gear, mask, min_chunk, max_chunk, 32, 1, wl.inv_freq_plain(), max_stream, 1, dev)

    def gpu_chunker(tokens, req_offsets, gear_, mask_, lo, hi):
        assert (mask_, lo, hi) == (mask, min_chunk, max_chunk)
        st, ln, rco, _ = front.chunk_host(tokens, req_offsets)
        return st, ln, rco

    n_var = 1 if name == "c0" else max(1, args.variants)
    s1 = args.stage == "s1"
    works = [wl.make_workload(name, gpu_chunker, size=args.size, variant=v, slots=args.slots,
                              assembly="unaligned" if s1 else "aligned", s1_window=128 if s1 else 0, cdc=args.cdc)
             for v in range(n_var)]
    if args.layers:
        for w in works:
            w.n_layers = args.layers
    w0 = works[0]
    _, _, _, pool_hash = front.chunk_host(w0.pool_tokens, np.array([0, len(w0.pool_tokens)], np.uint32))
    pool_windows = None
    if s1:
        pool_windows = front.windows_host(w0.pool_tokens, w0.pool_chunk_start, w0.pool_chunk_len,
                                          np.array([0, len(w0.pool_chunk_start)], np.uint32), 128, B.S1_ANCHOR_END)
    front.close()

    L = w0.n_layers
    fp8 = args.rows == "fp8"
    row_format = B.IRM_ROW_FP8 if fp8 else B.IRM_ROW_BF16
    ROW_BYTES = B.ROW_WORDS[row_format] * 2
    if fp8:
        assert args.stage in ("hit", "admit", "attend") and args.reattach in ("full", "kr"), \
            "--rows fp8: hit stage with --reattach full or kr, the admit stage or the attend stage"
    if fp8:
        # whoever only moves the 528 bytes gets random ones; the attention dequantises, so it gets N(0,1) quantised
        src = wl.kv_pool_fp8_torch(L, w0.src_rows, wl.kv_seed(name), dev,
                                   codes="quantised" if args.stage == "attend" else "random")
    else:
        src = wl.kv_pool_torch(L, w0.src_rows, wl.kv_seed(name), dev)
    STRIDE = ROW_BYTES
    if args.row_stride:
        assert args.stage == "hit" and args.reattach == "full", "--row-stride: hit stage with --reattach full"
        assert args.row_stride % 16 == 0 and args.row_stride >= ROW_BYTES, "--row-stride: a multiple of 16, >= the row"
        STRIDE = args.row_stride
        padded = torch.zeros((L, w0.src_rows, STRIDE // 2), dtype=src.dtype, device=dev)
        padded[:, :, :ROW_BYTES // 2].copy_(src)
        src = padded[:, :, :ROW_BYTES // 2]
        del padded
    src_ptrs = B.layer_pointers(src)
    n_streams = max(1, args.streams)
    if n_streams > 1:
        assert args.reattach == "full" and args.stage != "admit" and n_var % n_streams == 0, \
            "--streams needs --reattach full, the hit or s1 stage, and --variants divisible by it"
    if args.reattach == "full":
        dsts = [wl.sentinel_pool_torch(L, w0.dst_rows, dev, STRIDE // 2)[:, :, :ROW_BYTES // 2]
                for _ in range(n_streams)]
        dst_ptrs_of = [B.layer_pointers(d) for d in dsts]
        dst, dst_ptrs = dsts[0], dst_ptrs_of[0]
        bytes_per_token_layer = 2 * ROW_BYTES                        # one row read, one written
    elif args.reattach == "ref":
        row_index = torch.full((w0.dst_rows,), -1, dtype=torch.int32, device=dev)
        hit_index = torch.full((w0.dst_rows,), -1, dtype=torch.int32, device=dev)
        bytes_per_token_layer = 12.0 / L                            # 4 B slot read, 8 B written, per token
    else:
        dst = torch.zeros((L, w0.dst_rows, 64), dtype=torch.bfloat16, device=dev)
        dst_ptrs = B.kr_layer_pointers(dst)
        if args.reattach == "kr":
            kr_src_ptrs, kr_src_stride = B.kr_slice_pointers(src), ROW_BYTES
        else:
            kr_base = torch.empty((L, w0.src_rows, 64), dtype=torch.bfloat16, device=dev)
            for l in range(L):
                kr_base[l].copy_(src[l, :, 512:])
            kr_src_ptrs, kr_src_stride = B.kr_layer_pointers(kr_base), 128
        ckv_index = torch.full((w0.dst_rows,), -1, dtype=torch.int32, device=dev)
        bytes_per_token_layer = 2 * 128                              # k_r slice read and written

    sessions, dev_in = [], []
    for w in works:
        s = Session.for_workload(w, dev, row_format=row_format)
        reg = w.registry(pool_hash)
        if s1:
            wreg = w.window_registry(pool_windows[0], pool_windows[1], pool_windows[2], pool_windows[3], len(reg["hash"]))
            reg = {k: np.concatenate([reg[k], wreg[k]]) for k in reg}
        s.build_table(w.table_slots, reg)
        sessions.append(s)
        dev_in.append(dict(tokens=torch.from_numpy(w.tokens).to(dev), req_offsets=s.to_dev_u32(w.req_offsets),
                           pos_base=torch.from_numpy(w.pos_base).to(dev),
                           dst_slots=torch.from_numpy(w.dst_slots).to(dev),
                           buf=s.alloc_front(len(w.tokens), w.n_req),
                           wbuf=s.alloc_windows(len(w.tokens), w.n_req, 128) if s1 else None))
        if args.reattach == "ref":
            dev_in[-1]["trig"] = torch.zeros((dev_in[-1]["buf"]["cap"], 32, 2), dtype=torch.float32, device=dev)
        if args.grid:
            B.irm_ctx_tune(s.ctx, 0, args.grid)
        for kv in filter(None, args.tune.split(",")):
            B.irm_ctx_tune(s.ctx, int(kv.split("=")[0]), int(kv.split("=")[1]))

    streams = [torch.cuda.Stream(device=dev) for _ in range(n_streams)]
    stream = streams[0]
    torch.cuda.synchronize()
    if args.stage == "attend":
        with torch.cuda.stream(stream):
            calibrate(args.calibrate, dev, stream)
        out = bench_attend(args, works, sessions, dev_in, src, stream)
        for s in sessions:
            s.close()
        return out
    if args.stage == "admit":
        with torch.cuda.stream(stream):
            calibrate(args.calibrate, dev, stream)
        out = bench_admit(args, works, sessions, dev_in, src, stream)
        for s in sessions:
            s.close()
        return out

    def step(v):
        s, d = sessions[v], dev_in[v]
        if args.reattach == "full":
            st, dp = streams[v % n_streams], dst_ptrs_of[v % n_streams]   # a context stays on one stream
            s.serve(d["tokens"], d["req_offsets"], d["pos_base"], d["dst_slots"], src_ptrs, STRIDE,
                    w0.src_rows, dp, STRIDE, w0.dst_rows, d["buf"], st)
            if s1:
                s.s1_serve(d["tokens"], d["req_offsets"], d["pos_base"], d["dst_slots"], src_ptrs, STRIDE,
                           w0.src_rows, dp, STRIDE, w0.dst_rows, d["buf"], d["wbuf"], B.S1_ANCHOR_END, st)
        elif args.reattach == "ref":
            s.serve_ref(d["tokens"], d["req_offsets"], d["pos_base"], d["dst_slots"], w0.src_rows, row_index,
                        hit_index, d["trig"], d["buf"], stream)
        else:
            s.serve_kr(d["tokens"], d["req_offsets"], d["pos_base"], d["dst_slots"], kr_src_ptrs,
                       kr_src_stride, w0.src_rows, dst_ptrs, 128, w0.dst_rows, ckv_index, d["buf"], stream)

    with torch.cuda.stream(stream):
        # one pass per variant: learn the hit counts, check the error words
        hit_tokens, window_tokens, n_hits = [], [], []
        for v in range(n_var):
            step(v)
            torch.cuda.synchronize()
            n_hits.append(int(dev_in[v]["buf"]["n_hits"].item()))
            hit_tokens.append(int(dev_in[v]["buf"]["hit_tokens"].item())
                              + (int(dev_in[v]["wbuf"]["hit_tokens"].item()) if s1 else 0))
            if s1:
                window_tokens.append(int(dev_in[v]["wbuf"]["hit_tokens"].item()))
            flags = sessions[v].error_flags()
            assert flags == 0, f"device error flags {flags:#x}"
        for k in range(args.warmup):
            step(k % n_var)
        torch.cuda.synchronize()
        calibrate(args.calibrate, dev, stream)
        graphs = None
        if args.graph:
            assert n_streams == 1, "--graph replays on one stream"
            graphs = []
            for v in range(n_var):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    step(v)
                graphs.append(g)
            torch.cuda.synchronize()
        for s in sessions:
            if args.kernel_timing and not args.graph:
                # with S1 every step calls irm_reattach twice: sample the chunk-level launches only
                B.irm_ctx_profile_begin(s.ctx, args.steps // n_var + 1, args.kernel_timing * (2 if s1 else 1))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if graphs:
            for k in range(args.steps):
                graphs[k % n_var].replay()
        else:
            for k in range(args.steps):
                step(k % n_var)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        kernel_ms, kernel_n, kernel_tokens = 0.0, 0, 0
        for v, s in enumerate(sessions):
            ms, n = B.irm_ctx_profile_end(s.ctx, streams[v % n_streams])
            kernel_ms += ms
            kernel_n += n
            kernel_tokens += n * (hit_tokens[v] - (window_tokens[v] if s1 else 0))

    total_tokens = sum(hit_tokens[k % n_var] for k in range(args.steps))
    value = total_tokens / elapsed
    alg_bytes = kernel_tokens * L * bytes_per_token_layer
    achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
    # HBM bytes per launch as counted by rocprofv3 (FETCH_SIZE, WRITE_SIZE, scaled by a plain copy): a STORED
    # profile of this workload and kernel, not a measurement of this run
    traffic, traffic_source = None, None
    tfile = os.path.join(ROOT, "profiles", f"reattach_rows_{'fp8_' if fp8 else ''}{name}"
                                           f"{'_paper' if args.cdc == 'paper' else ''}_traffic.json")
    if (args.size == "full" and args.reattach == "full" and args.stage == "hit" and args.slots == "contiguous"
            and not args.row_stride and not args.layers and os.path.exists(tfile)):
        stored = json.load(open(tfile))
        traffic = stored.get("hbm_bytes_per_launch")
        traffic_source = f"stored: profiles/{os.path.basename(tfile)} ({stored.get('kernel', 'reattach_rows')})"

    out = {
        "metric": "re-attached KV tokens/s (all layers), whole hot path, 1 MI355X",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{name}-{args.size}: {w0.n_req} request(s) x {dims.get('req_len', dims['pool'])} tokens, "
                               f"{L} layers, pool {w0.src_rows} tokens, slots {args.slots}"
                               + (", paper-native CDC rule" if args.cdc == "paper" else "")
                               + (", fp8 rows (656 B: e4m3 c_KV + scales copied, bf16 k_r rotated)" if fp8 else "")
                               + (f", row stride {STRIDE} B" if STRIDE != ROW_BYTES else ""),
                   "cdc_rule": f"mask {mask:#x}, chunks of {min_chunk}..{max_chunk} tokens",
                   "variants": n_var, "streams": n_streams, "hip_graph": bool(args.graph),
                   "hit_tokens_per_step": float(np.mean(hit_tokens)), "hits_per_step": float(np.mean(n_hits)),
                   "stages": "irm_cdc_chunk+irm_chunk_hash+irm_lookup+irm_reattach%s %s"
                             % ({"full": "", "ref": "_ref"}.get(args.reattach, "_kr"),
                                "on one stream" if n_streams == 1 else
                                f"per batch on one stream, {n_streams} batches in flight on {n_streams} streams")
                             + ("; then S1: irm_s1_windows+irm_chunk_hash+irm_lookup+irm_reattach on the windows of "
                                "the missed chunks" if s1 else "")},
        "roofline": {"bound": "hbm", "kernel": {"full": "reattach_rows", "ref": "reattach_ref_rows"}.get(args.reattach, "reattach_kr_rows"), "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": alg_bytes / max(kernel_n, 1),
                     "bytes_per_token_layer": bytes_per_token_layer, "launches": kernel_n,
                     "avg_launch_us": kernel_ms / max(kernel_n, 1) * 1e3,
                     "kernel_tokens_per_s": kernel_tokens / (kernel_ms * 1e-3) if kernel_ms > 0 else 0.0},
    }

    if s1:
        out["metric"] = "re-attached KV tokens/s (all layers), hit path + S1 window fallback on unaligned batches, 1 MI355X"
        out["config"]["window_hit_tokens_per_step"] = float(np.mean(window_tokens))
        out["config"]["assembly"] = "unaligned"
    if not args.no_cpu_baseline and not s1:
        out["cpu_baseline"] = cpu_baseline(works, src, args.cpu_seconds)

    for s in sessions:
        s.close()
    return out


def bench_attend(args, works, sessions, dev_in, pool, stream):
    """The no-materialise scheme end to end for one decode step of a batch: chunk, fingerprint,
    look up, write the references (irm_reattach_ref), then attend over them on every layer
    (irm_attend_ref, one query token per request, k_r rotated as the rows are staged)."""
    import torch
    from paper_2605_05696_amd import binding as B

    w0 = works[0]
    ROW_BYTES = pool.shape[2] * 2                                # 1152 (bf16 rows) or 656 (fp8 rows)
    L, dev, H = w0.n_layers, pool.device, args.heads
    n_req = w0.n_req
    scale = 1.0 / np.sqrt(192.0)
    q = torch.randn((n_req, H, 576), device=dev, generator=torch.Generator(dev).manual_seed(1)).to(torch.bfloat16)
    out = torch.zeros((n_req, H, 512), dtype=torch.float32, device=dev)
    lse = torch.zeros((n_req, H), dtype=torch.float32, device=dev)
    ws = torch.empty(B.irm_attend_ref_workspace_bytes(n_req, H, args.splits), dtype=torch.uint8, device=dev)
    for v, (s, d, w) in enumerate(zip(sessions, dev_in, works)):
        d["row"] = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=dev)
        d["hit"] = torch.full((w.dst_rows,), -1, dtype=torch.int32, device=dev)
        d["trig"] = torch.zeros((d["buf"]["cap"], 32, 2), dtype=torch.float32, device=dev)

    def step(v):
        s, d = sessions[v], dev_in[v]
        s.serve_ref(d["tokens"], d["req_offsets"], d["pos_base"], d["dst_slots"], w0.src_rows, d["row"], d["hit"],
                    d["trig"], d["buf"], stream)
        for l in range(L):
            B.irm_attend_ref(s.ctx, q, pool[l], ROW_BYTES, d["dst_slots"], d["req_offsets"], d["row"], d["hit"],
                             d["trig"], scale, args.splits, ws, out, lse, stream)

    with torch.cuda.stream(stream):
        for v in range(len(works)):                              # first pass: the tokens no hit covers get
            step(v)                                              # plain pool rows ("prefilled and admitted")
            stream.synchronize()
            sessions[v].error_flags()                            # the first pass met unfilled slots: clear the word
            d = dev_in[v]
            miss = d["row"] < 0
            d["row"][miss] = torch.randint(0, w0.src_rows, (int(miss.sum().item()),), device=dev, dtype=torch.int32)
            step(v)
            stream.synchronize()
            assert sessions[v].error_flags() == 0
        if args.linear_rows:
            def step(v):                                         # attention only, rows in slot order
                s, d = sessions[v], dev_in[v]
                for l in range(L):
                    B.irm_attend_ref(s.ctx, q, pool[l], ROW_BYTES, d["dst_slots"], d["req_offsets"], d["row"],
                                     d["hit"], d["trig"], scale, args.splits, ws, out, lse, stream)
            for d in dev_in:
                d["row"].copy_(torch.arange(d["row"].numel(), dtype=torch.int32, device=dev))
                d["hit"].fill_(-1)
        for k in range(args.warmup):
            step(k % len(works))
        for s in sessions:
            if args.kernel_timing:
                B.irm_ctx_profile_begin(s.ctx, (args.steps // len(works) + 1) * L, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(k % len(works))
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        kernel_ms, kernel_n = 0.0, 0
        for s in sessions:
            ms, n = B.irm_ctx_profile_end(s.ctx, stream)
            kernel_ms += ms
            kernel_n += n
            assert s.error_flags() == 0, "the timed steps raised an error flag"
    ctx_tokens = len(w0.tokens)                                  # every request attends over all of its tokens
    # a row is streamed once per workgroup pass: 64 heads when the heads are a multiple of 64 (four head groups
    # share every staged tile), 32 when a multiple of 32, else 16
    groups = H // 64 if H % 64 == 0 else H // 32 if H % 32 == 0 else H // 16
    alg = ctx_tokens * ROW_BYTES * groups                        # per layer launch
    achieved = alg * kernel_n / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
    return {"metric": "attended context tokens/s (all layers), no-materialise scheme: front end + references + "
                      "rotate-on-load decode attention, 1 MI355X",
            "value": ctx_tokens * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": ("fp8 rows (656 B, c_KV dequantised on load), " if ROW_BYTES == 656 else "") +
                                   f"{w0.name}: {n_req} request(s), one decode query each over its whole context "
                                   f"({ctx_tokens} tokens in all), {H} heads, {L} layers, splits {args.splits}",
                       "variants": len(works),
                       "stages": "irm_cdc_chunk+irm_chunk_hash+irm_lookup+irm_reattach_ref once, irm_attend_ref per layer"},
            "roofline": {"bound": "hbm", "kernel": "attend_ref_split+attend_ref_merge", "achieved": achieved,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                         "bytes_per_token_layer": ROW_BYTES * groups, "launches": kernel_n,
                         "avg_launch_us": kernel_ms / max(kernel_n, 1) * 1e3,
                         # the two products: 576 + 512 multiply-adds per token and query row
                         "mfma_tflops": (2.0 * (576 + 512) * H * ctx_tokens * kernel_n / (kernel_ms * 1e-3) / 1e12
                                         if kernel_ms > 0 else 0.0),
                         "mfma_peak_tflops": 2500.0}}


def bench_yardstick(args):
    """Read-only, write-only and copy streams in a sweep of launch shapes: what the memory system gives
    a kernel that does nothing but move bytes (the ceiling of the row kernels)."""
    import torch
    from paper_2605_05696_amd import binding as B
    dev = "cuda:0"
    torch.cuda.set_device(0)
    n = 9 << 30                                                  # divisible by every grid x lanes x vectors x 16 below
    src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 256)
    dst = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 256)
    stream = torch.cuda.Stream(device=dev)
    rows = []
    reps = max(1, args.steps or 5)
    with torch.cuda.stream(stream):
        for mode, mname in ((B.YARDSTICK_READ, "read"), (B.YARDSTICK_WRITE, "write"), (B.YARDSTICK_COPY, "copy")):
            # the large grids give every workgroup one or two steps only: no loop, workgroups dispatched in
            # address order like the row kernel's, instead of a few thousand private ranges walked side by side
            for grid in (2048, 4096, 8192, 16384, 65536, 131072, 147456, 262144, 294912, 589824):
                for lanes, vec in ((256, 2), (256, 4), (256, 9), (256, 18), (256, 36), (512, 2), (512, 4), (512, 9),
                                   (1024, 2), (1024, 4)):
                    if n % (grid * lanes * vec * 16):
                        continue                                 # ranges must be whole steps
                    # the address-ordered shapes also with the row kernels' mapping: one contiguous eighth per XCD
                    for xcd in ((0, B.YARDSTICK_XCD_RANGES) if grid >= 131072 else (0,)):
                        B.irm_yardstick(dst, src, mode | xcd, grid, lanes, vec, stream)      # warm-up
                        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        a.record(stream)
                        for _ in range(reps):
                            B.irm_yardstick(dst, src, mode | xcd, grid, lanes, vec, stream)
                        b.record(stream)
                        b.synchronize()
                        ms = a.elapsed_time(b) / reps
                        moved = n * (2 if mode == B.YARDSTICK_COPY else 1)
                        rows.append({"mode": mname, "grid": grid, "lanes": lanes, "vectors_per_lane": vec,
                                     "xcd_ranges": bool(xcd), "steps_per_workgroup": n // (grid * lanes * vec * 16),
                                     "ms": ms, "gbs": moved / (ms * 1e-3) / 1e9})
    best = {m: max((r for r in rows if r["mode"] == m), key=lambda r: r["gbs"]) for m in ("read", "write", "copy")}
    median = {m: float(np.median([r["gbs"] for r in rows if r["mode"] == m])) for m in ("read", "write", "copy")}
    # a copy whose reads and writes take turns on the memory bus at their own best rates
    serial = 2.0 / (1.0 / best["read"]["gbs"] + 1.0 / best["write"]["gbs"])
    return {"metric": "plain streams over 9 GiB, HBM GB/s by launch shape, 1 MI355X", "unit": "GB/s",
            "value": best["copy"]["gbs"], "best": best, "median": median,
            "copy_if_reads_and_writes_took_turns": serial, "peak": HBM_PEAK_GBS, "reps": reps, "shapes": rows}


def calibrate(n, dev, stream):
    """n plain 1 GiB copies: known traffic to scale the hardware counters by."""
    if not n:
        return
    import torch
    from paper_2605_05696_amd import binding as B
    a = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    b = torch.empty_like(a)
    for _ in range(n):
        B.irm_calibrate_copy(b, a, 0, stream)
    stream.synchronize()
    del a, b


def bench_admit(args, works, sessions, dev_in, pool, stream):
    """Miss path on a cold registry: chunk, fingerprint and look the batch up against an EMPTY
    table (untimed), then time irm_admit, which copies every chunk past the carve-out from the
    request pool into the shared pool, all layers, and registers it."""
    import torch
    from paper_2605_05696_amd import binding as B
    from paper_2605_05696_amd import workloads as wl

    w0 = works[0]
    L, dev = w0.n_layers, pool.device
    fp8 = pool.shape[2] == 328
    ROW_BYTES = pool.shape[2] * 2
    req = (wl.kv_pool_fp8_torch if fp8 else wl.kv_pool_torch)(L, w0.dst_rows, 4242, dev)
    req_ptrs, pool_ptrs = B.layer_pointers(req), B.layer_pointers(pool)
    cursor = torch.zeros(1, dtype=torch.int32, device=dev)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    admitted_tokens = []
    t_wall = time.perf_counter()
    with torch.cuda.stream(stream):
        for k in range(args.warmup + args.steps):
            v = k % len(works)
            s, d, w = sessions[v], dev_in[v], works[v]
            buf = d["buf"]
            if s.table is not None:
                B.irm_table_destroy(s.table)
            s.table = B.irm_table_create(s.ctx, int(w.table_slots))
            adm = torch.empty(buf["cap"], dtype=torch.int32, device=dev)
            cursor.zero_()
            B.irm_cdc_chunk(s.ctx, d["tokens"], d["req_offsets"], buf["chunk_start"], buf["chunk_len"],
                            buf["req_chunk_offsets"], buf["n_chunks"], stream)
            B.irm_chunk_hash(s.ctx, d["tokens"], buf["chunk_start"], buf["chunk_len"], buf["n_chunks"],
                             buf["chunk_hash"], stream)
            B.irm_lookup(s.ctx, s.table, buf["chunk_hash"], buf["chunk_start"], buf["chunk_len"],
                         buf["req_chunk_offsets"], d["req_offsets"], d["pos_base"], buf["n_chunks"],
                         buf["chunk_entry"], buf["hits"], buf["n_hits"], buf["hit_tokens"], stream)
            timed = k >= args.warmup
            if timed:
                ev[k - args.warmup][0].record(stream)
            s.admit(d["req_offsets"], d["pos_base"], d["dst_slots"], req_ptrs, ROW_BYTES, w0.dst_rows, pool_ptrs,
                    ROW_BYTES, w0.src_rows, cursor, adm, buf, stream)
            if timed:
                ev[k - args.warmup][1].record(stream)
            stream.synchronize()
            flags = s.error_flags()
            assert flags == 0, f"device error flags {flags:#x}"
            if timed:
                admitted_tokens.append(int(cursor.item()))
    ms = sum(a.elapsed_time(b) for a, b in ev)
    tokens = sum(admitted_tokens)
    achieved = tokens * L * 2 * ROW_BYTES / (ms * 1e-3) / 1e9
    return {"metric": "admitted KV tokens/s (all layers), miss path irm_admit alone, cold registry, 1 MI355X",
            "value": tokens / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms / args.steps, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "u8", "data": "synthetic",
            "config": {"workload": f"{w0.name}: every chunk past the carve-out admitted, {L} layers, slots {args.slots}"
                                   + (", fp8 rows (656 B)" if fp8 else ""),
                       "variants": len(works), "admitted_tokens_per_step": float(np.mean(admitted_tokens)),
                       "stages": "irm_admit (admit_claim + admit_rows), events on its stream; chunking, hashing, "
                                 "the lookup against the empty table and the table reset are outside the timed span",
                       "wall_s": time.perf_counter() - t_wall},
            "roofline": {"bound": "hbm", "kernel": "admit_claim+admit_rows", "achieved": achieved,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                         "bytes_per_token_layer": 2 * ROW_BYTES, "launches": args.steps,
                         "avg_launch_us": ms / args.steps * 1e3}}


def cpu_baseline(works, src, budget_s):
    """The CPU oracle, as it stands, on the same request batches: chunk, fingerprint,
    lookup and re-attach, single thread, until about ``budget_s`` of CPU time is spent."""
    import torch
    from oracle import irm_oracle as orc
    from paper_2605_05696_amd import workloads as wl

    w0 = works[0]
    pool_hash = orc.chunk_hash(w0.pool_tokens, w0.pool_chunk_start, w0.pool_chunk_len)
    spent, tokens, batches = 0.0, 0, 0
    L = src.shape[0]
    k = 0
    while spent < min(budget_s, 10.0) and k < 64:            # cycle the batches until ~10 s of CPU work
        w = works[k % len(works)]
        k += 1
        reg = w.registry(pool_hash)
        t0 = time.perf_counter()
        st, ln, rco = orc.cdc_chunk(w.tokens, w.req_offsets, w.gear, w.mask, w.min_chunk, w.max_chunk)
        ch = orc.chunk_hash(w.tokens, st, ln)
        _, hits, hit_tokens = orc.lookup(reg["hash"], reg["src_row"], reg["p_src"], reg["len"],
                                         reg["entry_id"], ch, st, ln, rco, w.req_offsets, w.pos_base,
                                         w.carve_out)
        front_s = time.perf_counter() - t0
        # bound the sample: hits are taken in order until the remaining budget is used up
        rows_per_s = 4.0e5
        room = max(budget_s - spent - front_s, 0.5) * rows_per_s / L
        keep = int(np.searchsorted(np.cumsum(hits.len.astype(np.int64)), room, side="right"))
        keep = max(1, min(keep, len(hits)))
        lens = hits.len[:keep].astype(np.int64)
        off = np.concatenate([[0], np.cumsum(lens)])
        within = np.arange(off[-1]) - np.repeat(off[:-1], lens)
        src_idx = torch.from_numpy(np.repeat(hits.src_row[:keep].astype(np.int64), lens) + within).to(src.device)
        src_c = np.stack([src[l].index_select(0, src_idx).view(torch.int16).cpu().numpy().view(np.uint16)
                          for l in range(L)])
        dst_c = np.zeros_like(src_c)
        compact = orc.Hits(off[:-1].astype(np.uint32), off[:-1].astype(np.uint32), lens.astype(np.uint32),
                           hits.delta[:keep].copy())
        t1 = time.perf_counter()
        orc.reattach(src_c, dst_c, np.arange(off[-1], dtype=np.int32), compact, w.inv_freq)
        re_s = time.perf_counter() - t1
        # the integer stages ran on the whole batch: charge them in proportion to the sample
        share = off[-1] / max(hit_tokens, 1)
        spent += front_s * share + re_s
        tokens += int(off[-1])
        batches += 1
    # the same oracle calls fanned out over (layer, group of hits) on the host's cores, last sample
    # (ctypes releases the interpreter lock during a call; the integer stages stay on one thread)
    from concurrent.futures import ThreadPoolExecutor
    cores = max(1, min(16, os.cpu_count() or 1))     # a one-GPU machine's share of the host is 16 threads
    slots = np.arange(off[-1], dtype=np.int32)
    groups = np.array_split(np.arange(keep), max(1, min(keep, -(-4 * cores // L))))
    def one(task):
        l, g = task
        sub = orc.Hits(compact.src_row[g], compact.dst_tok[g], compact.len[g], compact.delta[g])
        orc.reattach(src_c[l:l + 1], dst_c[l:l + 1], slots, sub, w.inv_freq)
    tasks = [(l, g) for l in range(L) for g in groups if len(g)]
    t2 = time.perf_counter()
    with ThreadPoolExecutor(cores) as pool:
        list(pool.map(one, tasks))
    mt_s = time.perf_counter() - t2 + front_s * share
    return {"value": tokens / spent, "unit": "tokens/s", "cores": 1, "host_cores": os.cpu_count(), "kind": "oracle",
            "sample": f"{tokens} re-attached tokens x {L} layers from {batches} batch pass(es) over the same workload "
                      f"(chunk+hash+lookup+re-attach, single thread), {spent:.1f} s of CPU time",
            "all_cores": {"value": int(off[-1]) / mt_s, "unit": "tokens/s", "cores": cores,
                          "host_cores": os.cpu_count(),
                          "sample": f"the last pass's {int(off[-1])} tokens x {L} layers, re-attach fanned out over "
                                    f"{len(tasks)} (layer, hit group) tasks on {cores} threads"}}


if __name__ == "__main__":
    sys.exit(main())
