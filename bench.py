#!/usr/bin/env python3
"""Benchmark of the fused Flash Decode hot path on one MI355X.

One "step" = one fd_decode call: the whole hot path (work decomposition, K/V
streaming, online softmax, partial write, arrival count, last-arriver combine)
over one batch of synthetic input already resident in HBM.  The default
workload is the long-context configuration (c5), the one the benchmark's target
(>= 70 % of the HBM roofline) is quoted on.  K/V are rotated over several
identical copies so that no call finds its data in the 256 MB Infinity Cache.

Prints ONE JSON line.  `value` is achieved algorithmic HBM bandwidth of the
fused call (GB/s); the fused and bulk-synchronous latencies are beside it.
Timing follows the paper's protocol (Section 5.1: warm-up, then timed
iterations, mean) with HIP events on the launch stream.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", default="c5", help="c1..c5 (default c5, the long-context workload)")
    ap.add_argument("--copies", type=int, default=0, help="rotating K/V copies (0 = enough to exceed 1 GiB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bsp", action="store_true")
    ap.add_argument("--no-waits", action="store_true", help="skip the fine-grained-waits variant (fd_decode_waits)")
    ap.add_argument("--no-hot", action="store_true", help="skip the hot-cache figure (one K/V copy) of the workloads that fit the Infinity Cache")
    ap.add_argument("--print-sources-digest", action="store_true", help="print the digest of the kernel sources that a profile summary records, and exit")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the same calls")
    ap.add_argument("--no-probe", action="store_true", help="skip the read-only streaming kernel (achievable bandwidth)")
    ap.add_argument("--xcd-groups", type=int, default=0)
    ap.add_argument("--wgs-per-cu", type=int, default=0)
    ap.add_argument("--path", type=int, default=0)
    ap.add_argument("--ring-stages", type=int, default=0)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "fp16", "fp8kv"],
                    help="element type of q/K/V (fp16 = the paper's; fp8kv = bf16 q over an E4M3 cache, scales 1/32)")
    ap.add_argument("--autotune", action="store_true",
                    help="let fd_autotune pick the options for this shape first (untimed); the choice is reported")
    ap.add_argument("--page-size", type=int, default=0,
                    help="time fd_decode_paged over a page pool of this page size (pages placed in seeded random order)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy 3 times (known HBM traffic: 1 GiB read + 1 GiB "
                         "written per launch) so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    return ap.parse_args()


def settle(fn, torch, seconds=0.12):
    """Untimed calls until the device has been busy for a while: the first tens of milliseconds of work after an
    idle period run measurably slower (1-3 %), whatever kernel is launched; no timed loop starts inside them."""
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(50):
            fn(i)
            i += 1
        torch.cuda.synchronize()


def time_calls(fn, n_warm, n_steps, torch):
    """Mean duration of one call in ms: HIP events on the launch stream around n_steps calls."""
    settle(fn, torch)
    for i in range(n_warm):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(n_steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / n_steps
    return e0.elapsed_time(e1) / n_steps, wall_ms


def time_graph(fn, n_steps, torch):
    """The same n_steps calls recorded once into a HIP graph and replayed: mean ms per call (None if the capture
    fails).  The calls only launch kernels on the stream they are given, so they can be captured."""
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            st = torch.cuda.current_stream().cuda_stream
            for i in range(n_steps):
                fn(i, st)
        torch.cuda.synchronize()
        settle(fn, torch)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n_steps
    except Exception as exc:                          # a figure beside the headline: never fatal
        print(f"bench: graph replay skipped ({exc})", file=sys.stderr)
        return None


def per_call_percentiles(fn, n_calls, torch):
    """p10 / median / p90 of single calls, each bracketed by its own pair of HIP events (us)."""
    import numpy as np
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_calls)]
    for i, (a, b) in enumerate(ev):
        a.record()
        fn(i)
        b.record()
    torch.cuda.synchronize()
    d = np.array([a.elapsed_time(b) * 1e3 for a, b in ev])
    return [round(float(np.percentile(d, q)), 2) for q in (10, 50, 90)]


def streaming_probe(fd, torch, stream):
    """Bandwidth of a read-only kernel (the library's 128-bit non-temporal loads) over 1 GiB: GB/s."""
    src = torch.empty(1 << 28, device="cuda", dtype=torch.float32).fill_(1.0)
    sink = torch.zeros(1, device="cuda", dtype=torch.int32)
    nbytes = src.numel() * 4
    for _ in range(3):
        fd.fd_debug_stream_read(src, nbytes, sink, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        fd.fd_debug_stream_read(src, nbytes, sink, stream)
    e1.record()
    torch.cuda.synchronize()
    gbs = nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src
    return gbs


def read_traffic(workload_name, dtype, page_size):
    """HBM bytes per launch of the fused kernel from the committed rocprofv3 --pmc summary of THIS workload, element
    type and cache layout, or None if there is none.  Warns when the summary was measured on other kernel sources."""
    tag = ("" if dtype == "bf16" else f"_{dtype}") + (f"_page{page_size}" if page_size else "")
    path = os.path.join(ROOT, "profiles", f"fd_fused{tag}_{workload_name}_pmc.txt")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    # the summary names the kernel sources it was measured on (a digest of their contents); file
    # times say nothing after a checkout
    rec = re.search(r"^kernel_sources_sha256\s*=\s*([0-9a-f]+)", text, re.M)
    if rec is None or rec.group(1) != kernel_sources_digest():
        print(f"bench.py: warning: {os.path.relpath(path, ROOT)} was not measured on the current kernel sources; "
              "roofline.traffic may be stale", file=sys.stderr)
    m = re.search(r"^traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", text, re.M)
    return float(m.group(1)) if m else None


def kernel_sources_digest():
    """sha256 over the kernel sources (names and contents, in name order), first 16 hex digits."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2511_02168_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def cpu_baseline(inp, wl, fi, fmt="bf16", n_threads=0, seconds=10.0):
    """The fp64 oracle as it stands, timed on the host cores (n_threads = 0: all of them) on a bounded sample."""
    import numpy as np
    import oracle
    # sample: whole sequences of the first sequences / heads, sized to what the oracle gets through in ~10-30 s
    budget_keys_heads = 6.0e7 * 4 if n_threads == 0 else 2.0e7
    sl = inp.seq_lens.cpu().numpy()
    B = 0
    acc = 0
    while B < wl.B and (B == 0 or acc + int(sl[B]) * wl.Hq <= budget_keys_heads):
        acc += int(sl[B]) * wl.Hq
        B += 1
    q, k, v = fi.bits(inp.q[:B]), fi.bits(inp.k[:B]), fi.bits(inp.v[:B])
    oracle.decode(q[:1, :, :], k[:1, :, :64].copy(), v[:1, :, :64].copy(), np.minimum(sl[:1], 64), fmt=fmt)   # load + warm
    t0 = time.perf_counter()
    reps = 0
    while True:
        oracle.decode(q, k, v, sl[:B], fmt=fmt, n_threads=n_threads)
        reps += 1
        if time.perf_counter() - t0 > seconds or reps >= 20:
            break
    dt = (time.perf_counter() - t0) / reps
    nbytes = fi.algorithmic_bytes(wl, sl[:B])
    return {"value": round(nbytes / dt / 1e9, 3), "unit": "GB/s", "cores": int(n_threads or oracle.max_threads()),
            "kind": "oracle", "us_per_call": round(dt * 1e6, 1),
            "sample": f"first {B} of {wl.B} sequences, all {wl.Hq} query heads, full length "
                      f"({int(sl[:B].sum())} keys), {reps} runs, mean"}


def main():
    args = parse_args()
    if args.print_sources_digest:
        print(kernel_sources_digest())
        return
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X's share of the work); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2511_02168_amd import binding as fd
    from paper_2511_02168_amd import inputs as fi

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    wl = fi.workload(args.config)
    inp = fi.make_inputs(wl, "cuda", dtype=torch.float16 if args.dtype == "fp16" else torch.bfloat16)
    sl_host = inp.seq_lens.cpu().numpy()
    fp8 = args.dtype == "fp8kv"
    if fp8:
        inp.k, inp.v = fi.to_fp8_cache(inp)
    alg_bytes = fi.algorithmic_bytes(wl, sl_host, 1 if fp8 else 2)
    kv_bytes = inp.k.numel() * inp.k.element_size() * 2
    copies = args.copies or max(2, -(-(1 << 30) // kv_bytes) + 1)
    copies = min(copies, 64)
    ks = [inp.k] + [inp.k.clone() for _ in range(copies - 1)]
    vs = [inp.v] + [inp.v.clone() for _ in range(copies - 1)]
    max_splits = wl.n_splits if wl.n_splits > 0 else -(-wl.S_max // 512)
    dec = fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=max_splits, dtype=args.dtype,
                         k_scale=1.0 / 32 if fp8 else 0.0, v_scale=1.0 / 32 if fp8 else 0.0)
    for key, val in ((fd.FD_OPT_XCD_GROUPS, args.xcd_groups), (fd.FD_OPT_WGS_PER_CU, args.wgs_per_cu),
                     (fd.FD_OPT_PATH, args.path), (fd.FD_OPT_RING_STAGES, args.ring_stages)):
        if val:
            fd.fd_set_option(dec.h, key, val)
    out = torch.empty(wl.B, wl.Hq, wl.D, device="cuda", dtype=torch.float32)
    lse = torch.empty(wl.B, wl.Hq, device="cuda", dtype=torch.float32)
    stream = torch.cuda.current_stream().cuda_stream

    if args.page_size:
        pg = fi.make_paged(inp, args.page_size, seed=wl.seed)
        ks = [pg.k_pages] + [pg.k_pages.clone() for _ in range(copies - 1)]
        vs = [pg.v_pages] + [pg.v_pages.clone() for _ in range(copies - 1)]

        def fused(i, st=stream):
            j = i % copies
            fd.fd_decode_paged(dec.h, inp.q, ks[j], vs[j], pg.block_table, args.page_size, inp.seq_lens, out, lse,
                               wl.n_splits, st)

        def bsp(i, st=stream):
            j = i % copies
            fd.fd_decode_paged(dec.h, inp.q, ks[j], vs[j], pg.block_table, args.page_size, inp.seq_lens, out, lse,
                               wl.n_splits, st, bsp=True)
    else:
        def fused(i, st=stream):
            j = i % copies
            fd.fd_decode(dec.h, inp.q, ks[j], vs[j], inp.seq_lens, out, lse, wl.n_splits, st)

        def bsp(i, st=stream):
            j = i % copies
            fd.fd_decode_bsp(dec.h, inp.q, ks[j], vs[j], inp.seq_lens, out, lse, wl.n_splits, st)

    if args.pmc_calibration:
        src = torch.empty(1 << 28, device="cuda", dtype=torch.float32).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    tuned = None
    if args.autotune and not args.page_size:
        fd.fd_autotune(dec.h, inp.q, ks[0], vs[0], inp.seq_lens, out, lse, wl.n_splits, stream, reps=30)
        tuned = {"path": fd.fd_get_option(dec.h, fd.FD_OPT_PATH), "xcd_groups": fd.fd_get_option(dec.h, fd.FD_OPT_XCD_GROUPS),
                 "wgs_per_cu": fd.fd_get_option(dec.h, fd.FD_OPT_WGS_PER_CU),
                 "ring_stages": fd.fd_get_option(dec.h, fd.FD_OPT_RING_STAGES),
                 "adaptive_split_keys": fd.fd_get_option(dec.h, fd.FD_OPT_SPLIT_KEYS) if wl.n_splits == 0 else None}
    fused_ms, fused_wall_ms = time_calls(fused, args.warmup, args.steps, torch)
    grid = fd.fd_get_option(dec.h, fd.FD_INFO_LAST_GRID)
    path = fd.fd_get_option(dec.h, fd.FD_INFO_LAST_PATH)
    bsp_ms = None
    if not args.no_bsp:
        bsp_ms, _ = time_calls(bsp, args.warmup, args.steps, torch)

    waits_ms = None
    if not args.no_waits and not args.page_size and path == 2 and args.dtype == "bf16":
        def waits(i):
            j = i % copies
            fd.fd_decode_waits(dec.h, inp.q, ks[j], vs[j], inp.seq_lens, out, lse, wl.n_splits, stream)
        waits_ms, _ = time_calls(waits, args.warmup, args.steps, torch)
        if fd.fd_get_option(dec.h, fd.FD_INFO_WAIT_GAVE_UP):
            waits_ms = None
    # hot cache: one K/V copy, for the workloads whose K/V fit the 256 MB Infinity Cache
    hot_ms = None
    if not args.no_hot and copies > 1 and kv_bytes <= (256 << 20):
        hot_ms, _ = time_calls(lambda i: fused(0), args.warmup, args.steps, torch)
    # the same calls launched as one HIP graph
    graph_fused_ms = graph_bsp_ms = None
    if not args.no_graph:
        graph_fused_ms = time_graph(fused, args.steps, torch)
        if not args.no_bsp and graph_fused_ms is not None:
            graph_bsp_ms = time_graph(bsp, args.steps, torch)
    pct_fused = per_call_percentiles(fused, min(args.steps, 200), torch)
    pct_bsp = None if args.no_bsp else per_call_percentiles(bsp, min(args.steps, 200), torch)
    probe_gbs = None if args.no_probe else streaming_probe(fd, torch, stream)

    gbs = alg_bytes / (fused_ms * 1e-3) / 1e9
    rec = {
        "metric": "decode-attention us/call + achieved HBM GB/s (% of roofline), fused vs BSP",
        "value": round(gbs, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(fused_ms, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "dtype_detail": f"{args.dtype} q/K/V, products and sums in f32 (MFMA f32 accumulate), f32 out and lse",
        "data": "synthetic (seeded N(0,1) q/K/V rounded to " + {"bf16": "bf16", "fp16": "IEEE half", "fp8kv": "bf16, K/V then to E4M3 bytes with scale 1/32"}[args.dtype]
                + "; ragged lengths, scaled K and aligned keys per workload)",
        "config": {"workload": wl.name, "B": wl.B, "Hq": wl.Hq, "Hkv": wl.Hkv, "D": wl.D, "S_max": wl.S_max,
                   "n_splits": wl.n_splits, "total_keys": int(sl_host.sum()), "kv_copies_rotated": copies,
                   "kv_layout": f"paged, page_size {args.page_size}, random placement" if args.page_size else "contiguous",
                   "autotuned_options": tuned, "grid_workgroups": grid, "kernel_path": {1: "valu", 2: "mfma"}.get(path, str(path))},
        "us_per_call_fused": round(fused_ms * 1e3, 3),
        "us_per_call_fused_host_wall": round(fused_wall_ms * 1e3, 3),
        "us_per_call_bsp": None if bsp_ms is None else round(bsp_ms * 1e3, 3),
        "us_per_call_fine_grained_waits": None if waits_ms is None else round(waits_ms * 1e3, 3),
        "us_per_call_fused_hot_cache": None if hot_ms is None else round(hot_ms * 1e3, 3),
        "us_per_call_fused_graph_replay": None if graph_fused_ms is None else round(graph_fused_ms * 1e3, 3),
        "us_per_call_bsp_graph_replay": None if graph_bsp_ms is None else round(graph_bsp_ms * 1e3, 3),
        "fused_over_bsp": None if bsp_ms is None else round(fused_ms / bsp_ms, 4),
        "us_single_call_fused_p10_p50_p90": pct_fused,
        "us_single_call_bsp_p10_p50_p90": pct_bsp,
        "streaming_read_probe_gbs": None if probe_gbs is None else round(probe_gbs, 1),
        "pct_of_streaming_read_probe": None if probe_gbs is None else round(100.0 * gbs / probe_gbs, 2),
        "pct_of_hbm_roofline": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "algorithmic_bytes_per_call": alg_bytes,
        "roofline": {"bound": "hbm", "achieved": round(gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": read_traffic(wl.name, args.dtype, args.page_size),
                     "kernel": "fd fused persistent kernel (one launch per call)"},
    }
    if not args.no_cpu_baseline and not fp8:
        rec["cpu_baseline"] = cpu_baseline(inp, wl, fi, args.dtype)
        if wl.index <= 2:                     # the small workloads also on one core
            rec["cpu_baseline_1core"] = cpu_baseline(inp, wl, fi, args.dtype, n_threads=1, seconds=5.0)
    dec.close()
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
