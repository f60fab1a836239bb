"""GPU parity of the two-level combine (tiles with more partials than FD_OPT_TREE_ROWS).

Shapes that reach it by themselves (one or two tiles cut into hundreds of splits) and ordinary
shapes with the threshold forced down to a handful of partials.  The bars are the same as
everywhere: out within atol = rtol = 2e-3 of the fp64 oracle, LSE within 1e-4 relative, fused and
bulk-synchronous results bitwise equal, counters back at zero, nothing left over for the next call.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2511_02168_amd import binding as fd
from paper_2511_02168_amd import inputs as fi

pytestmark = pytest.mark.gpu

ATOL = RTOL = 2e-3
LSE_RTOL = 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check(out, lse, ref_o, ref_l, what):
    out = out.cpu().numpy().astype(np.float64)
    lse = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all(), f"{what}: non-finite output"
    assert (np.abs(out - ref_o) <= ATOL + RTOL * np.abs(ref_o)).all(), f"{what}: out outside tolerance ({np.abs(out - ref_o).max():.2e})"
    inf = np.isneginf(ref_l)
    assert np.array_equal(np.isneginf(lse), inf), f"{what}: -inf pattern of lse differs"
    assert (np.abs(lse[~inf] - ref_l[~inf]) <= LSE_RTOL * np.maximum(1.0, np.abs(ref_l[~inf]))).all(), f"{what}: lse outside tolerance"


def both(dec, inp, n, what):
    """fused and BSP, twice each (the second pair finds counters the first left armed wrongly)"""
    res = []
    for rep in range(2):
        fd.fd_debug_poison_workspace(dec.h)
        of, lf = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n)
        ob, lb = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n, bsp=True)
        torch.cuda.synchronize()
        assert torch.equal(of.view(torch.int32), ob.view(torch.int32)), f"{what}: fused and BSP out differ bitwise (pass {rep})"
        assert torch.equal(lf.view(torch.int32), lb.view(torch.int32)), f"{what}: fused and BSP lse differ bitwise (pass {rep})"
        assert all(c == 0 for c in fd.fd_debug_read_counters(dec.h, dec.cfg.B * dec.cfg.Hkv)), f"{what}: tile counters not re-armed"
        res.append((of, lf))
    assert torch.equal(res[0][0].view(torch.int32), res[1][0].view(torch.int32)), f"{what}: second call differs from the first"
    return res[1]


# B, Hq, Hkv, S_max, ragged, n_splits, max_splits, tree_rows (0 = auto, 64), xcd_groups, wgs_per_cu,
# several first-level groups for sure (the result must then differ from the one-level result in rounding)
SHAPES = [
    (1, 8, 1, 16384, False, 256, 256, 0, 0, 0, True),     # one tile, 256 partials: 16 groups of 16
    (1, 8, 1, 9000, False, 200, 200, 0, 0, 0, True),      # 64-key splits, the last ones past the end: 141 partials, last group of 13
    (1, 4, 1, 20000, False, 300, 300, 0, 0, 2, True),     # 2 workgroups per CU: 300 partials of one tile
    (2, 8, 1, 12000, True, 128, 128, 0, 0, 0, False),     # two sequences of different lengths, 128 splits each
    (1, 16, 2, 8192, False, 128, 128, 0, 1, 0, True),     # G = 8, two tiles in one list, 128 partials each
    (1, 12, 1, 6000, False, 90, 96, 20, 0, 0, True),      # G = 12 (two passes over the (head, dims) pairs), 47 partials
    (1, 16, 1, 5000, False, 70, 80, 20, 0, 0, True),      # G = 16, 40 partials, groups of 16, 16 and 8
    (1, 2, 2, 70000, False, 0, 256, 0, 0, 0, True),       # adaptive: 137 splits per tile, G = 1
    (3, 6, 3, 5000, True, 40, 40, 5, 0, 0, False),        # forced: threshold 5 on an ordinary ragged shape
    (8, 32, 8, 4096, False, 16, 16, 2, 8, 0, False),      # forced on a c2-like shape: 4 partials per tile, lists per XCD
    (8, 32, 8, 4096, False, 16, 16, 2, 1, 0, False),      # the same with one list
    (4, 16, 8, 3000, True, 0, 8, 2, 0, 0, False),         # forced, adaptive splits
    (5, 6, 3, 900, True, 4, 8, 2, 8, 2, False),           # forced, tile count not a multiple of 8 asked for 8 lists, 2 per CU
]


@pytest.mark.parametrize("B,Hq,Hkv,S,ragged,n,max_splits,tree_rows,xcd,per_cu,several_groups", SHAPES)
def test_two_level_combine_matches_oracle_and_bsp(B, Hq, Hkv, S, ragged, n, max_splits, tree_rows, xcd, per_cu, several_groups):
    wl = fi.Workload(f"tree_b{B}_hq{Hq}_hkv{Hkv}_s{S}", 9100 + B + Hq + S % 97, B=B, Hq=Hq, Hkv=Hkv, S_max=S, n_splits=n, ragged=ragged)
    say(f"case two-level combine B={B} Hq={Hq} Hkv={Hkv} S<={S} n_splits={n} tree_rows={tree_rows or 'auto'} lists={xcd or 'auto'} per_cu={per_cu or 'auto'}")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(B, Hq, Hkv, S, max_splits=max_splits) as dec:
        for key, val in ((fd.FD_OPT_TREE_ROWS, tree_rows), (fd.FD_OPT_XCD_GROUPS, xcd), (fd.FD_OPT_WGS_PER_CU, per_cu)):
            if val:
                fd.fd_set_option(dec.h, key, val)
        out, lse = both(dec, inp, n, "two levels")
        check(out, lse, ref_o, ref_l, "two levels")
        # one level (threshold out of reach): same inputs, same bars; differs from two levels in rounding only
        fd.fd_set_option(dec.h, fd.FD_OPT_TREE_ROWS, 4096)
        out1, lse1 = both(dec, inp, n, "one level")
        check(out1, lse1, ref_o, ref_l, "one level")
        assert float((out - out1).abs().max()) <= 1e-5, "one and two levels differ by more than rounding"
        if several_groups:                            # another summation order
            assert not torch.equal(out.view(torch.int32), out1.view(torch.int32)), "the two-level path did not run"


@pytest.mark.parametrize("dtype", ["fp16", "fp8kv"])
def test_two_level_combine_other_element_types(dtype):
    wl = fi.Workload(f"tree_{dtype}", 9201, B=1, Hq=8, Hkv=2, S_max=12000, n_splits=128)
    say(f"case two-level combine, {dtype}, 128 partials per tile")
    ks = vs = 1.0 / 32
    if dtype == "fp16":
        inp = fi.make_inputs(wl, "cuda", dtype=torch.float16)
        q, k, v = inp.q, inp.k, inp.v
        ref_o, ref_l = oracle.decode(fi.bits(q), fi.bits(k), fi.bits(v), inp.seq_lens.cpu().numpy(), fmt="fp16")
    else:
        inp = fi.make_inputs(wl, "cuda")
        q = inp.q
        k, v = fi.to_fp8_cache(inp, ks, vs)
        ref_o, ref_l = oracle.decode_fp8kv(fi.bits(q), fi.bytes_of(k), fi.bytes_of(v), inp.seq_lens.cpu().numpy(),
                                           k_scale=ks, v_scale=vs)
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=128, dtype=dtype, k_scale=ks, v_scale=vs) as dec:
        of, lf = dec.decode(q, k, v, inp.seq_lens, 128)
        ob, lb = dec.decode(q, k, v, inp.seq_lens, 128, bsp=True)
        torch.cuda.synchronize()
        assert torch.equal(of.view(torch.int32), ob.view(torch.int32)) and torch.equal(lf.view(torch.int32), lb.view(torch.int32))
        check(of, lf, ref_o, ref_l, dtype)


def test_two_level_combine_is_deterministic_and_sees_no_leftovers():
    """300 calls alternating two different caches on one handle: a first-level result or a group count left
    over from the other cache would show; every result of a cache must equal its first, bit for bit."""
    wl = fi.Workload("tree_alt", 9301, B=1, Hq=8, Hkv=1, S_max=16384, n_splits=256)
    say("case two-level combine, alternating inputs, 300 calls")
    a = fi.make_inputs(wl, "cuda")
    b = fi.make_inputs(fi.Workload("tree_alt_b", 9302, B=1, Hq=8, Hkv=1, S_max=16384, n_splits=256), "cuda")
    b.seq_lens.fill_(9000)                                # fewer live partials than the other: 141 of 256
    with fd.FlashDecode(1, 8, 1, 16384, max_splits=256) as dec:
        first = {}
        for i in range(300):
            inp = (a, b)[i % 2]
            out, lse = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 256)
            if i < 2:
                first[i] = (out.clone(), lse.clone())
            elif i % 50 < 2:
                torch.cuda.synchronize()
                assert torch.equal(out.view(torch.int32), first[i % 2][0].view(torch.int32)), f"call {i} differs"
                assert torch.equal(lse.view(torch.int32), first[i % 2][1].view(torch.int32)), f"call {i} lse differs"
        torch.cuda.synchronize()
        for i, inp in enumerate((a, b)):
            ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
            check(first[i][0], first[i][1], ref_o, ref_l, f"cache {i}")


def test_two_level_combine_through_the_static_workspace_and_a_paged_cache():
    wl = fi.Workload("tree_static", 9401, B=1, Hq=8, Hkv=2, S_max=10000, n_splits=100)
    say("case two-level combine: fd_decode_static, fd_decode_paged")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    cfg = fd.fd_config(wl.B, wl.Hq, wl.Hkv, 128, wl.S_max, 100, 0, 0.0, fd.FD_DTYPE_BF16, 0.0, 0.0)
    out = torch.full((wl.B, wl.Hq, 128), float("nan"), device="cuda")
    lse = torch.full((wl.B, wl.Hq), float("nan"), device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    for rep in range(2):
        fd.fd_decode_static(cfg, inp.q, inp.k, inp.v, inp.seq_lens, out, lse, 100, st)
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=100) as dec:
        oh, lh = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 100)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), oh.view(torch.int32)) and torch.equal(lse.view(torch.int32), lh.view(torch.int32))
        check(out, lse, ref_o, ref_l, "static workspace")
        pg = fi.make_paged(inp, 64, seed=9402)
        op, lp = dec.decode_paged(inp.q, pg.k_pages, pg.v_pages, pg.block_table, 64, inp.seq_lens, 100)
        opb, lpb = dec.decode_paged(inp.q, pg.k_pages, pg.v_pages, pg.block_table, 64, inp.seq_lens, 100, bsp=True)
        torch.cuda.synchronize()
        assert torch.equal(op.view(torch.int32), opb.view(torch.int32)) and torch.equal(lp.view(torch.int32), lpb.view(torch.int32))
        check(op, lp, ref_o, ref_l, "paged cache")
        # the waiting variant always merges in one level: same bars, not the same bits
        ow, lw = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 100, waits=True)
        torch.cuda.synchronize()
        check(ow, lw, ref_o, ref_l, "fine-grained waits")


def test_tree_rows_option_validation():
    with fd.FlashDecode(1, 8, 1, 1024, max_splits=4) as dec:
        assert fd.fd_get_option(dec.h, fd.FD_OPT_TREE_ROWS) == 0
        for bad in (-1, 1):
            with pytest.raises(fd.FdError) as e:
                fd.fd_set_option(dec.h, fd.FD_OPT_TREE_ROWS, bad)
            assert e.value.code == fd.FD_ERR_INVALID_ARG
        fd.fd_set_option(dec.h, fd.FD_OPT_TREE_ROWS, 2)
        assert fd.fd_get_option(dec.h, fd.FD_OPT_TREE_ROWS) == 2
