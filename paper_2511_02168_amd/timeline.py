"""In-kernel timeline of one fused (or split) Flash Decode call: where the microseconds of a call go.

    python -m paper_2511_02168_amd.timeline --config c2 [--dtype fp8kv] [--bsp] [--xcd-groups 8]
    python -m paper_2511_02168_amd.timeline --shape 1 96 8 16384 32      (B Hq Hkv S n_splits, full-length sequences)

Attaches a trace buffer (fd_debug_set_trace), runs a few calls of the workload and prints, for the
last of them, the spread over the workgroups of every milestone a workgroup stamps with the 100 MHz
wall clock: start, first K/V stage landed, streaming loop left, partial stored, stores
acknowledged, arrival counted, tile combined, end, and inside a combine: fence passed, weights
ready, rows accumulated.  Times are microseconds after the earliest workgroup's start.
"""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as fd
from . import inputs as fi

EVENTS = ["start", "first_stage", "loop_end", "partial_out", "stores_acked", "counted", "combined", "end",
          "comb_entered", "comb_fenced", "comb_weights", "comb_rows"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c5")
    ap.add_argument("--shape", type=int, nargs=5, metavar=("B", "HQ", "HKV", "S", "N_SPLITS"),
                    help="an ad-hoc workload instead of --config (seeded N(0,1) inputs, every sequence S keys long)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "fp16", "fp8kv"])
    ap.add_argument("--bsp", action="store_true", help="trace fd_decode_bsp (kernel 1's workgroups, then kernel 2's)")
    ap.add_argument("--xcd-groups", type=int, default=0)
    ap.add_argument("--calls", type=int, default=3, help="traced calls (the last one is reported)")
    args = ap.parse_args()

    if args.shape:
        B, Hq, Hkv, S, n = args.shape
        wl = fi.Workload(f"shape_b{B}_hq{Hq}_hkv{Hkv}_s{S}_n{n}", 4242, B=B, Hq=Hq, Hkv=Hkv, S_max=S, n_splits=n)
    else:
        wl = fi.workload(args.config)
    inp = fi.make_inputs(wl, "cuda", dtype=torch.float16 if args.dtype == "fp16" else torch.bfloat16)
    fp8 = args.dtype == "fp8kv"
    if fp8:
        inp.k, inp.v = fi.to_fp8_cache(inp)
    kv_bytes = inp.k.numel() * inp.k.element_size() * 2
    copies = min(max(2, -(-(1 << 30) // kv_bytes) + 1), 16)
    ks = [inp.k] + [inp.k.clone() for _ in range(copies - 1)]
    vs = [inp.v] + [inp.v.clone() for _ in range(copies - 1)]
    max_splits = wl.n_splits if wl.n_splits > 0 else -(-wl.S_max // 512)
    dec = fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=max_splits, dtype=args.dtype,
                         k_scale=1.0 / 32 if fp8 else 0.0, v_scale=1.0 / 32 if fp8 else 0.0)
    if args.xcd_groups:
        fd.fd_set_option(dec.h, fd.FD_OPT_XCD_GROUPS, args.xcd_groups)
    out = torch.empty(wl.B, wl.Hq, wl.D, device="cuda", dtype=torch.float32)
    lse = torch.empty(wl.B, wl.Hq, device="cuda", dtype=torch.float32)
    stream = torch.cuda.current_stream().cuda_stream
    call = fd.fd_decode_bsp if args.bsp else fd.fd_decode
    for i in range(10):                                                  # untraced warm-up
        call(dec.h, inp.q, ks[i % copies], vs[i % copies], inp.seq_lens, out, lse, wl.n_splits, stream)
    torch.cuda.synchronize()
    cap = 4096
    tr = torch.zeros(cap, fd.FD_TRACE_EVENTS, device="cuda", dtype=torch.int64)
    fd.fd_debug_set_trace(dec.h, tr, cap)
    for i in range(args.calls):
        tr.zero_()
        call(dec.h, inp.q, ks[i % copies], vs[i % copies], inp.seq_lens, out, lse, wl.n_splits, stream)
        torch.cuda.synchronize()
    fd.fd_debug_set_trace(dec.h, None, 0)
    grid = fd.fd_get_option(dec.h, fd.FD_INFO_LAST_GRID)
    t = tr[:max(grid, wl.B * wl.Hkv)].cpu().numpy().astype(np.float64)
    dec.close()

    t0 = t[:, 0][t[:, 0] > 0].min()
    print(f"workload {wl.name}, dtype {args.dtype}, {'fd_decode_bsp' if args.bsp else 'fd_decode'}, grid {grid} workgroups, "
          f"call {args.calls} of {args.calls} traced; microseconds after the earliest workgroup start")
    print(f"  {'milestone':13s} {'n':>5s} {'min':>8s} {'p10':>8s} {'median':>8s} {'p90':>8s} {'max':>8s}")
    for e, name in enumerate(EVENTS):
        col = t[:, e]
        ok = col > 0
        if not ok.any():
            continue
        rel = (col[ok] - t0) / 100.0
        print(f"  {name:13s} {int(ok.sum()):5d} {rel.min():8.2f} {np.percentile(rel, 10):8.2f} {np.median(rel):8.2f} "
              f"{np.percentile(rel, 90):8.2f} {rel.max():8.2f}")
    busy = (t[:grid, 1] > 0) & (t[:grid, 2] > 0)
    if busy.any():
        dur = (t[:grid, 2] - t[:grid, 1])[busy] / 100.0
        print(f"  streaming loop (first stage landed -> loop left): min {dur.min():.2f}  median {np.median(dur):.2f}  max {dur.max():.2f}")
        for x in range(8):
            sel = busy & (np.arange(grid) % 8 == x)
            if sel.any():
                le = (t[:grid, 2][sel] - t0) / 100.0
                print(f"    workgroups with id % 8 == {x} (one XCD): loop left at min {le.min():.1f}  median {np.median(le):.1f}  max {le.max():.1f}")
    comb = t[:, 6] > 0
    if comb.any():
        d = lambda a, b: (t[comb, a] - t[comb, b]) / 100.0
        print(f"  combining workgroups ({int(comb.sum())}): counted -> fence passed {np.median(d(9, 5)):.2f}, -> weights ready "
              f"{np.median(d(10, 5)):.2f}, -> rows accumulated {np.median(d(11, 5)):.2f}, -> combined {np.median(d(6, 5)):.2f} (medians)")
    last_loop = (t[:grid, 2][busy].max() - t0) / 100.0 if busy.any() else float("nan")
    end = (t[:, 7][t[:, 7] > 0].max() - t0) / 100.0
    print(f"  last workgroup left its loop at {last_loop:.2f}, the kernel's last workgroup ended at {end:.2f}: tail {end - last_loop:.2f} us")


if __name__ == "__main__":
    main()
