"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle.

Tolerances are the benchmark definition's: out within atol = rtol = 2e-3,
LSE within 1e-4 relative (|d| <= 1e-4 * max(1, |ref|)).  Fused and
bulk-synchronous results must be bitwise equal (same partials, fixed-order
merge).  Inputs are seeded synthetic tensors (paper_2511_02168_amd.inputs).
"""
import dataclasses
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


def check_out(got, ref, what):
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref)
    bound = ATOL + RTOL * np.abs(ref)
    worst = float((err / bound).max()) if err.size else 0.0
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    assert worst <= 1.0, f"{what}: out error {err.max():.3e} exceeds tolerance (ratio {worst:.2f})"
    return float(err.max())


def check_lse(got, ref, what):
    got = np.asarray(got, dtype=np.float64)
    inf = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf), f"{what}: -inf pattern of lse differs"
    err = np.abs(got[~inf] - ref[~inf])
    bound = LSE_RTOL * np.maximum(1.0, np.abs(ref[~inf]))
    assert (err <= bound).all(), f"{what}: lse error {err.max():.3e} exceeds 1e-4 relative"
    return float(err.max()) if err.size else 0.0


def run_both(dec, inp, n_splits, want_lse=True):
    """Fused and BSP through the C ABI; asserts bitwise equality; returns numpy results."""
    out_f, lse_f = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n_splits, want_lse=want_lse)
    out_b, lse_b = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n_splits, bsp=True, want_lse=want_lse)
    torch.cuda.synchronize()
    assert torch.equal(out_f.view(torch.int32), out_b.view(torch.int32)), "fused and BSP outputs differ bitwise"
    if want_lse:
        assert torch.equal(lse_f.view(torch.int32), lse_b.view(torch.int32)), "fused and BSP lse differ bitwise"
    n_tiles = dec.cfg.B * dec.cfg.Hkv
    assert all(c == 0 for c in fd.fd_debug_read_counters(dec.h, n_tiles)), "arrival counters not re-armed"
    return out_f.cpu().numpy(), (lse_f.cpu().numpy() if want_lse else None)


def full_parity(wl, inp, n_splits, max_splits=None, what=""):
    ms = max_splits or max(n_splits, 1)
    with fd.FlashDecode(inp.q.shape[0], wl.Hq, wl.Hkv, inp.k.shape[2], max_splits=ms) as dec:
        fd.fd_debug_poison_workspace(dec.h)
        out, lse = run_both(dec, inp, n_splits)
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    eo = check_out(out, ref_o, what)
    el = check_lse(lse, ref_l, what)
    say(f"  {what}: max |out err| {eo:.2e}, max |lse err| {el:.2e}")


# ---------------------------------------------------------------- the five workloads

def test_c1_tiny_mha_full():
    wl = fi.workload("c1")
    say(f"case {wl.name} B{wl.B} Hq{wl.Hq} Hkv{wl.Hkv} S{wl.S_max} n{wl.n_splits}")
    inp = fi.make_inputs(wl, "cuda")
    full_parity(wl, inp, wl.n_splits, what=wl.name)


def test_c2_gqa_full():
    wl = fi.workload("c2")
    say(f"case {wl.name} B{wl.B} Hq{wl.Hq} Hkv{wl.Hkv} S{wl.S_max} n{wl.n_splits}")
    inp = fi.make_inputs(wl, "cuda")
    full_parity(wl, inp, wl.n_splits, what=wl.name)


def test_c3_group8_full():
    wl = fi.workload("c3")
    say(f"case {wl.name} B{wl.B} Hq{wl.Hq} Hkv{wl.Hkv} S{wl.S_max} n{wl.n_splits}")
    inp = fi.make_inputs(wl, "cuda")
    full_parity(wl, inp, wl.n_splits, what=wl.name)


def test_c4_ragged_full_size_full_oracle():
    """Every (b, h) row of the full-size ragged workload against the oracle: the one configuration
    that drives the adaptive work list over all 512 tiles (about 16.6 thousand items)."""
    wl = fi.workload("c4")
    say(f"case {wl.name} B{wl.B} Hq{wl.Hq} Hkv{wl.Hkv} S<= {wl.S_max} adaptive splits, full size, every row")
    inp = fi.make_inputs(wl, "cuda")
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=64) as dec:
        fd.fd_debug_poison_workspace(dec.h)
        out, lse = run_both(dec, inp, 0)
    assert np.isfinite(out).all() and np.isfinite(lse).all()      # NaN padding past seq_lens was never read
    sl = inp.seq_lens.cpu().numpy()
    q_bits = fi.bits(inp.q)
    worst_o = worst_l = 0.0
    for b0 in range(0, wl.B, 16):                                 # 16 sequences at a time bound the host copies
        b1 = min(b0 + 16, wl.B)
        ref_o, ref_l = oracle.decode(q_bits[b0:b1], fi.bits(inp.k[b0:b1]), fi.bits(inp.v[b0:b1]), sl[b0:b1])
        worst_o = max(worst_o, check_out(out[b0:b1], ref_o, f"{wl.name} sequences {b0}..{b1 - 1}"))
        worst_l = max(worst_l, check_lse(lse[b0:b1], ref_l, f"{wl.name} sequences {b0}..{b1 - 1}"))
        say(f"  sequences {b0}..{b1 - 1} done")
    say(f"  {wl.name}: all {wl.B * wl.Hq} rows, max |out err| {worst_o:.2e}, max |lse err| {worst_l:.2e}")


def test_c4_ragged_reduced_full_oracle():
    wl = fi.workload("c4")
    say(f"case {wl.name} reduced to B=16, S_max=3000 (ragged, NaN padded), adaptive and fixed splits, full oracle")
    inp = fi.make_inputs(wl, "cuda", S_max=3000, B=16)
    full_parity(wl, inp, 0, max_splits=16, what=wl.name + "/reduced/adaptive")
    full_parity(wl, inp, 5, max_splits=16, what=wl.name + "/reduced/n5")


def test_c5_long_context_full_size_full_oracle():
    """Every query head of the full-size long-context workload against the oracle."""
    wl = fi.workload("c5")
    say(f"case {wl.name} B{wl.B} Hq{wl.Hq} Hkv{wl.Hkv} S{wl.S_max} n{wl.n_splits}, full size, every row")
    inp = fi.make_inputs(wl, "cuda")
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=wl.n_splits) as dec:
        fd.fd_debug_poison_workspace(dec.h)
        out, lse = run_both(dec, inp, wl.n_splits)
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    eo = check_out(out, ref_o, wl.name)
    el = check_lse(lse, ref_l, wl.name)
    say(f"  {wl.name}: all {wl.B * wl.Hq} rows, max |out err| {eo:.2e}, max |lse err| {el:.2e}")
    # peaked attention: the aligned keys must dominate (lse well above the ln(S) of flat attention)
    assert float(lse.min()) > np.log(wl.S_max) + 1.0


def test_c5_reduced_full_oracle():
    wl = fi.workload("c5")
    say(f"case {wl.name} reduced to S=8200, n_splits 16 and 7, full oracle")
    inp = fi.make_inputs(wl, "cuda", S_max=8200)
    full_parity(wl, inp, 16, what=wl.name + "/reduced/n16")
    full_parity(wl, inp, 7, what=wl.name + "/reduced/n7")


# ---------------------------------------------------------------- edge shapes

def _generic(B, Hq, Hkv, S_max, seed, ragged=False, k_scale=1.0):
    return fi.Workload(f"edge_b{B}_hq{Hq}_hkv{Hkv}_s{S_max}", seed, B=B, Hq=Hq, Hkv=Hkv, S_max=S_max, n_splits=0,
                       ragged=ragged, k_scale=k_scale)


@pytest.mark.parametrize("S", [1, 2, 31, 32, 33, 63, 64, 65, 127, 129, 511, 512, 513, 1000])
def test_edge_sequence_lengths(S):
    wl = _generic(2, 8, 2, S, 100 + S)
    say(f"case edge S={S} G=4, n_splits 1, 3, adaptive")
    inp = fi.make_inputs(wl, "cuda")
    for n in (1, 3, 0):
        full_parity(wl, inp, n, max_splits=8, what=f"S={S} n={n}")


@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 15, 16])
def test_every_group_size(G):
    wl = _generic(3, 2 * G, 2, 777, 200 + G, ragged=True)
    say(f"case group size G={G}, ragged S<=777, n_splits 4 and adaptive")
    inp = fi.make_inputs(wl, "cuda")
    full_parity(wl, inp, 4, max_splits=8, what=f"G={G} n=4")
    full_parity(wl, inp, 0, max_splits=8, what=f"G={G} adaptive")


@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 6, 7, 8])
def test_valu_kernel_every_group_size(G):
    """The VALU kernel (FD_OPT_PATH = 1; no longer the default anywhere) on ragged lengths and edge sizes."""
    wl = _generic(3, 2 * G, 2, 777, 220 + G, ragged=True)
    say(f"case VALU kernel, G={G}, ragged S<=777 and S in 1, 33, 512")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=8) as dec:
        fd.fd_set_option(dec.h, fd.FD_OPT_PATH, 1)
        for n in (4, 0):
            fd.fd_debug_poison_workspace(dec.h)
            out, lse = run_both(dec, inp, n)
            assert fd.fd_get_option(dec.h, fd.FD_INFO_LAST_PATH) == 1
            check_out(out, ref_o, f"VALU G={G} n={n}")
            check_lse(lse, ref_l, f"VALU G={G} n={n}")
    for S in (1, 33, 512):
        wl2 = _generic(2, 2 * G, 2, S, 230 + G + S)
        inp2 = fi.make_inputs(wl2, "cuda")
        ref_o, ref_l = oracle.decode(fi.bits(inp2.q), fi.bits(inp2.k), fi.bits(inp2.v), inp2.seq_lens.cpu().numpy())
        with fd.FlashDecode(wl2.B, wl2.Hq, wl2.Hkv, wl2.S_max, max_splits=4) as dec:
            fd.fd_set_option(dec.h, fd.FD_OPT_PATH, 1)
            for n in (1, 3):
                out, lse = run_both(dec, inp2, n)
                check_out(out, ref_o, f"VALU G={G} S={S} n={n}")
                check_lse(lse, ref_l, f"VALU G={G} S={S} n={n}")


@pytest.mark.parametrize("G,path,per_cu", [(1, 2, 1), (4, 2, 1), (4, 2, 2), (8, 1, 2), (8, 2, 1), (8, 2, 2), (16, 2, 2)])
def test_both_kernels_on_the_same_shapes(G, path, per_cu):
    """FD_OPT_PATH forces the VALU (1) or MFMA (2) kernel; per_cu picks the MFMA ring depth."""
    wl = _generic(4, 2 * G, 2, 1500, 250 + G, ragged=True)
    say(f"case forced kernel path={path} wgs_per_cu={per_cu} G={G}, ragged S<=1500")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=8) as dec:
        fd.fd_set_option(dec.h, fd.FD_OPT_PATH, path)
        fd.fd_set_option(dec.h, fd.FD_OPT_WGS_PER_CU, per_cu)
        for n in (1, 3, 8, 0):
            fd.fd_debug_poison_workspace(dec.h)
            out, lse = run_both(dec, inp, n)
            assert fd.fd_get_option(dec.h, fd.FD_INFO_LAST_PATH) == path
            check_out(out, ref_o, f"path={path} G={G} n={n}")
            check_lse(lse, ref_l, f"path={path} G={G} n={n}")


@pytest.mark.parametrize("stages", [2, 3, 4])
def test_every_ring_depth_of_the_mfma_kernel(stages):
    """FD_OPT_RING_STAGES: the depth of each wave's LDS ring changes how far the K/V stream
    runs ahead, never the arithmetic: all depths give bitwise the same result."""
    wl = _generic(3, 16, 2, 2100, 260 + stages, ragged=True)
    say(f"case ring stages={stages}, G=8, ragged S<=2100")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    outs = []
    for st in (stages, 0):
        with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=8) as dec:
            fd.fd_set_option(dec.h, fd.FD_OPT_RING_STAGES, st)
            assert fd.fd_get_option(dec.h, fd.FD_OPT_RING_STAGES) == st
            for n in (1, 5, 0):
                fd.fd_debug_poison_workspace(dec.h)
                out, lse = run_both(dec, inp, n)
                check_out(out, ref_o, f"stages={st} n={n}")
                check_lse(lse, ref_l, f"stages={st} n={n}")
                outs.append(out)
    for a, b in zip(outs[:3], outs[3:]):
        assert np.array_equal(a, b), "ring depth changed the result"


@pytest.mark.parametrize("S", [1, 15, 16, 17, 63, 64, 65, 100, 1023, 1025])
def test_edge_sequence_lengths_group8(S):
    wl = _generic(2, 16, 2, S, 150 + S)
    say(f"case edge S={S} G=8 (MFMA kernel), n_splits 1, 3, adaptive")
    inp = fi.make_inputs(wl, "cuda")
    for n in (1, 3, 0):
        full_parity(wl, inp, n, max_splits=8, what=f"G=8 S={S} n={n}")


@pytest.mark.parametrize("G,n_splits,per_cu", [(1, 512, 2), (2, 300, 2), (4, 256, 1), (8, 256, 1), (8, 1000, 2),
                                               (16, 248, 1), (16, 512, 2), (16, 1024, 2)])
def test_one_tile_with_many_live_partials(G, n_splits, per_cu):
    """A single (batch, KV head) tile cut into more splits than there are workgroups: every
    workgroup leaves one partial, so the combine sees hundreds of live rows (several row
    batches per thread, a liveness scan of more than 256 slots, and for G = 16 with more
    than 248 rows the variant that does not stage its weights in LDS)."""
    S = 64 * n_splits + 37
    wl = _generic(1, G, 1, S, 900 + G + n_splits)
    say(f"case one tile, G={G}, n_splits={n_splits}, wgs_per_cu={per_cu}, S={S}")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(1, G, 1, S, max_splits=1024) as dec:
        fd.fd_set_option(dec.h, fd.FD_OPT_WGS_PER_CU, per_cu)
        fd.fd_debug_poison_workspace(dec.h)
        out, lse = run_both(dec, inp, n_splits)
        say(f"  grid {fd.fd_get_option(dec.h, fd.FD_INFO_LAST_GRID)} workgroups")
    check_out(out, ref_o, f"many partials G={G} n={n_splits}")
    check_lse(lse, ref_l, f"many partials G={G} n={n_splits}")


def test_more_splits_than_key_blocks():
    wl = _generic(2, 4, 1, 100, 300)
    say("case n_splits=16 over 100 keys (most splits empty)")
    inp = fi.make_inputs(wl, "cuda")
    full_parity(wl, inp, 16, what="n16/S100")


def test_zero_and_one_length_sequences_in_a_batch():
    wl = _generic(5, 8, 2, 600, 400)
    say("case seq_lens = [0, 1, 600, 64, 0]")
    inp = fi.make_inputs(wl, "cuda")
    inp.seq_lens = torch.tensor([0, 1, 600, 64, 0], dtype=torch.int32, device="cuda")
    for b, s in enumerate([0, 1, 600, 64, 0]):            # poison everything past the end
        inp.k[b, :, s:] = float("nan")
        inp.v[b, :, s:] = float("nan")
    for n in (0, 1, 4):
        full_parity(wl, inp, n, max_splits=4, what=f"zero/one lengths n={n}")


@pytest.mark.parametrize("B,Hq,Hkv,S,n,xcd", [(80, 8, 2, 700, 0, 0), (43, 14, 7, 300, 0, 0), (70, 4, 2, 500, 3, 0),
                                              (5, 6, 3, 900, 0, 8), (5, 6, 3, 900, 4, 8), (67, 8, 1, 400, 0, 8)])
def test_batches_beyond_64_and_uneven_xcd_groups(B, Hq, Hkv, S, n, xcd):
    """Shapes the five workloads do not reach: more than 64 sequences (the sequence length of an item is then a
    load, not a lane of the prefetched vector), more than 256 tiles in one work list (several tiles per thread in
    the adaptive scan), and 8 work lists over a tile count that 8 does not divide."""
    wl = _generic(B, Hq, Hkv, S, 330 + B + Hkv, ragged=True)
    say(f"case B={B} Hq={Hq} Hkv={Hkv} ragged S<={S} n_splits={n} xcd_groups={xcd or 'auto'}")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=8) as dec:
        if xcd:
            fd.fd_set_option(dec.h, fd.FD_OPT_XCD_GROUPS, xcd)
        for per_cu in (0, 2):
            fd.fd_set_option(dec.h, fd.FD_OPT_WGS_PER_CU, per_cu)
            fd.fd_debug_poison_workspace(dec.h)
            out, lse = run_both(dec, inp, n)
            check_out(out, ref_o, f"B={B} tiles={B * Hkv} n={n} per_cu={per_cu}")
            check_lse(lse, ref_l, f"B={B} tiles={B * Hkv} n={n} per_cu={per_cu}")


def test_lse_pointer_may_be_null():
    wl = _generic(2, 8, 2, 700, 500)
    say("case lse = NULL")
    inp = fi.make_inputs(wl, "cuda")
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=4) as dec:
        out, _ = run_both(dec, inp, 4, want_lse=False)
    ref_o, _ = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    check_out(out, ref_o, "lse=NULL")


def test_peaked_two_key_attention():
    """Two dominant keys with opposite values: the hardest case for weight rounding."""
    wl = _generic(1, 8, 1, 256, 600)
    say("case two dominant keys, opposite values (G=8)")
    inp = fi.make_inputs(wl, "cuda")
    q32 = inp.q.float()
    for h in range(8):                      # keys 2h and 2h+1 aligned with head h, others left random
        qh = q32[0, h]
        inp.k[0, 0, 2 * h] = (qh * 1.5).to(torch.bfloat16)
        inp.k[0, 0, 2 * h + 1] = (qh * 1.5).to(torch.bfloat16)
        inp.v[0, 0, 2 * h] = 1.0
        inp.v[0, 0, 2 * h + 1] = -1.0
    full_parity(wl, inp, 2, what="two-key peaked")


def test_custom_scale():
    wl = _generic(2, 4, 2, 300, 700)
    say("case scale = 0.25 (not 1/sqrt(D))")
    inp = fi.make_inputs(wl, "cuda")
    cfg = dict(B=wl.B, Hq=wl.Hq, Hkv=wl.Hkv, S_max=wl.S_max, max_splits=4, scale=0.25)
    with fd.FlashDecode(**cfg) as dec:
        out, lse = run_both(dec, inp, 3)
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy(), scale=0.25)
    check_out(out, ref_o, "scale 0.25")
    check_lse(lse, ref_l, "scale 0.25")


# ---------------------------------------------------------------- protocol checks

def test_repeat_determinism_with_poisoned_workspace():
    wl = fi.workload("c2")
    say("case 1000 repeated fused calls on c2 (S reduced to 2048), NaN-poisoned workspace before each")
    inp = fi.make_inputs(wl, "cuda", S_max=2048)
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, 2048, max_splits=16) as dec:
        first_o, first_l = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 16)
        first_o, first_l = first_o.clone(), first_l.clone()
        for it in range(1000):
            fd.fd_debug_poison_workspace(dec.h, torch.cuda.current_stream().cuda_stream)
            o, l = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 16)
            assert torch.equal(o.view(torch.int32), first_o.view(torch.int32)), f"iteration {it}: output changed"
            assert torch.equal(l.view(torch.int32), first_l.view(torch.int32)), f"iteration {it}: lse changed"
        assert all(c == 0 for c in fd.fd_debug_read_counters(dec.h, wl.B * wl.Hkv))


@pytest.mark.parametrize("xcd", [1, 8])
def test_alternating_inputs_never_see_the_previous_calls_partials(xcd):
    """Two different K/V caches attended in turn on one handle, 600 calls, the partial buffer poisoned with NaN
    before each: every result must equal, bit for bit, the first result for the same cache.  A combine that read
    a partial the previous call (other cache) left in some cache level, instead of what this call wrote, would
    show.  With one work list a tile's partials come from all 8 XCDs; with eight from the combiner's own."""
    wl = fi.workload("c2")
    say(f"case alternating inputs, c2 with S reduced to 4096, xcd_groups={xcd}")
    inp_a = fi.make_inputs(wl, "cuda", S_max=4096)
    inp_b = fi.make_inputs(dataclasses.replace(wl, index=77), "cuda", S_max=4096)
    ref_o, ref_l = oracle.decode(fi.bits(inp_b.q), fi.bits(inp_b.k), fi.bits(inp_b.v), inp_b.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, 4096, max_splits=16) as dec:
        fd.fd_set_option(dec.h, fd.FD_OPT_XCD_GROUPS, xcd)
        first = {}
        for name, inp in (("a", inp_a), ("b", inp_b)):
            o, l = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 16)
            first[name] = (o.clone(), l.clone())
        assert not torch.equal(first["a"][0], first["b"][0])
        check_out(first["b"][0].cpu().numpy(), ref_o, "alternating b")
        check_lse(first["b"][1].cpu().numpy(), ref_l, "alternating b")
        stream = torch.cuda.current_stream().cuda_stream
        for it in range(600):
            name, inp = (("a", inp_a), ("b", inp_b))[it & 1]
            fd.fd_debug_poison_workspace(dec.h, stream)
            fn = dec.decode
            o, l = fn(inp.q, inp.k, inp.v, inp.seq_lens, 16, bsp=(it % 5 == 4))
            assert torch.equal(o.view(torch.int32), first[name][0].view(torch.int32)), f"iteration {it}: output differs"
            assert torch.equal(l.view(torch.int32), first[name][1].view(torch.int32)), f"iteration {it}: lse differs"
        assert all(c == 0 for c in fd.fd_debug_read_counters(dec.h, wl.B * wl.Hkv))


def test_xcd_grouping_and_grid_size_change_only_rounding():
    """The launch shape decides which consecutive splits one workgroup attends in one go,
    i.e. the summation order: results may differ by rounding only, and fused == BSP
    bitwise for every shape."""
    wl = fi.workload("c2")
    say("case c2 (S reduced to 4096): XCD groups 1 vs 8, 1 or 2 workgroups per CU")
    inp = fi.make_inputs(wl, "cuda", S_max=4096)
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, 4096, max_splits=16) as dec:
        for xg in (1, 8):
            for per_cu in (1, 2):
                fd.fd_set_option(dec.h, fd.FD_OPT_XCD_GROUPS, xg)
                fd.fd_set_option(dec.h, fd.FD_OPT_WGS_PER_CU, per_cu)
                fd.fd_debug_poison_workspace(dec.h)
                out, lse = run_both(dec, inp, 16)
                check_out(out, ref_o, f"xcd_groups={xg} wgs_per_cu={per_cu}")
                check_lse(lse, ref_l, f"xcd_groups={xg} wgs_per_cu={per_cu}")
        fd.fd_set_option(dec.h, fd.FD_OPT_WGS_PER_CU, 4)             # more than the MFMA kernel runs per CU: refused, not clamped
        with pytest.raises(fd.FdError) as e:
            dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 16)
        assert e.value.code == fd.FD_ERR_INVALID_ARG


def test_argument_errors_on_device():
    say("case argument validation with a live handle")
    with fd.FlashDecode(1, 8, 8, 1024, max_splits=4) as dec:
        t = torch.zeros(1, 8, 128, device="cuda", dtype=torch.bfloat16)
        kv = torch.zeros(1, 8, 1024, 128, device="cuda", dtype=torch.bfloat16)
        sl = torch.full((1,), 1024, device="cuda", dtype=torch.int32)
        out = torch.empty(1, 8, 128, device="cuda")
        with pytest.raises(fd.FdError) as e:
            fd.fd_decode(dec.h, t, kv, kv, sl, out, None, 5)        # n_splits > max_splits
        assert e.value.code == fd.FD_ERR_INVALID_ARG
        with pytest.raises(fd.FdError) as e:
            fd.fd_decode(dec.h, None, kv, kv, sl, out, None, 4)
        assert e.value.code == fd.FD_ERR_INVALID_ARG
        with pytest.raises(fd.FdError) as e:
            fd.fd_decode(dec.h, t, kv, kv, sl, out, None, -1)
        assert e.value.code == fd.FD_ERR_INVALID_ARG
        for key, bad in ((fd.FD_OPT_PATH, 3), (fd.FD_OPT_XCD_GROUPS, 4), (fd.FD_OPT_WGS_PER_CU, 17),
                         (fd.FD_OPT_RING_STAGES, 5), (fd.FD_OPT_RING_STAGES, 1), (999, 0), (fd.FD_INFO_NUM_CUS, 1)):
            with pytest.raises(fd.FdError) as e:
                fd.fd_set_option(dec.h, key, bad)
            assert e.value.code == fd.FD_ERR_INVALID_ARG
        assert fd.fd_get_option(dec.h, fd.FD_INFO_NUM_CUS) == 256


def test_reset_trace_and_stream_probe_entry_points():
    """The maintenance / measurement entry points: fd_reset re-zeroes the counters, the
    timeline trace records ordered milestones for every workgroup and leaves results
    unchanged, the read-only streaming kernel runs and validates its arguments."""
    wl = _generic(2, 16, 2, 3000, 777)
    say("case fd_reset, fd_debug_set_trace, fd_debug_stream_read")
    inp = fi.make_inputs(wl, "cuda")
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=16) as dec:
        out0, lse0 = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 16)
        fd.fd_reset(dec.h)
        torch.cuda.synchronize()
        assert all(c == 0 for c in fd.fd_debug_read_counters(dec.h, wl.B * wl.Hkv))
        grid_cap = 1024
        tr = torch.zeros(grid_cap, fd.FD_TRACE_EVENTS, device="cuda", dtype=torch.int64)
        fd.fd_debug_set_trace(dec.h, tr, grid_cap)
        out1, lse1 = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 16)
        torch.cuda.synchronize()
        fd.fd_debug_set_trace(dec.h, None, 0)
        grid = fd.fd_get_option(dec.h, fd.FD_INFO_LAST_GRID)
        t = tr[:grid].cpu().numpy()
        assert (t[:, 0] > 0).all() and (t[:, 7] >= t[:, 0]).all(), "every workgroup records start <= end"
        busy = t[:, 2] > 0
        assert busy.any() and (t[busy, 2] >= t[busy, 1]).all() and (t[busy, 1] >= t[busy, 0]).all()
        assert (tr[grid:] == 0).all()
        assert torch.equal(out0.view(torch.int32), out1.view(torch.int32)) and torch.equal(lse0, lse1)
        out2, _ = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 16)
        torch.cuda.synchronize()
        assert torch.equal(out0.view(torch.int32), out2.view(torch.int32))
    src = torch.ones((1 << 20) + 5, device="cuda", dtype=torch.float32)       # ragged tail: not a whole chunk
    sink = torch.zeros(1, device="cuda", dtype=torch.int32)
    fd.fd_debug_stream_read(src, src.numel() * 4, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0
    with pytest.raises(fd.FdError) as e:
        fd.fd_debug_stream_read(None, 1024, sink)
    assert e.value.code == fd.FD_ERR_INVALID_ARG
    with pytest.raises(fd.FdError) as e:
        fd.fd_debug_stream_read(src[1:], 1024, sink)                           # 4-byte aligned only
    assert e.value.code == fd.FD_ERR_INVALID_ARG


# ---------------------------------------------------------------- paged KV cache

def _paged_parity(wl, page_size, n_values, what, max_splits=8, seed=0):
    inp = fi.make_inputs(wl, "cuda")
    pg = fi.make_paged(inp, page_size, seed=seed)
    ref_o, ref_l = oracle.decode_paged(fi.bits(pg.q), fi.bits(pg.k_pages), fi.bits(pg.v_pages),
                                       pg.block_table.cpu().numpy(), pg.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=max_splits) as dec:
        for n in n_values:
            fd.fd_debug_poison_workspace(dec.h)
            out_f, lse_f = dec.decode_paged(pg.q, pg.k_pages, pg.v_pages, pg.block_table, page_size, pg.seq_lens, n)
            out_b, lse_b = dec.decode_paged(pg.q, pg.k_pages, pg.v_pages, pg.block_table, page_size, pg.seq_lens, n,
                                            bsp=True)
            out_c, lse_c = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n)
            torch.cuda.synchronize()
            assert fd.fd_get_option(dec.h, fd.FD_INFO_LAST_PATH) == 2
            assert torch.equal(out_f.view(torch.int32), out_b.view(torch.int32)), "paged fused != paged BSP"
            assert torch.equal(lse_f.view(torch.int32), lse_b.view(torch.int32))
            if out_c is not None:      # same partition, same key order, separately compiled loop: equal to rounding
                assert torch.allclose(out_f, out_c, rtol=1e-5, atol=1e-6), "paged != contiguous"
                assert torch.allclose(lse_f, lse_c, rtol=1e-6, atol=1e-6)
            eo = check_out(out_f.cpu().numpy(), ref_o, f"{what} n={n}")
            el = check_lse(lse_f.cpu().numpy(), ref_l, f"{what} n={n}")
            say(f"  {what} n={n}: max |out err| {eo:.2e}, max |lse err| {el:.2e}")


@pytest.mark.parametrize("page_size", [16, 32, 64, 128, 256, 1024])
def test_paged_cache_every_page_size(page_size):
    wl = _generic(3, 16, 2, 2500, 600 + page_size, ragged=True)
    say(f"case paged cache, page_size={page_size}, G=8, ragged S<=2500, n_splits 1, 5, adaptive")
    _paged_parity(wl, page_size, (1, 5, 0), f"paged ps={page_size}")


@pytest.mark.parametrize("G", [1, 2, 3, 4, 7, 8, 12, 16])
def test_paged_cache_every_group_size(G):
    wl = _generic(2, 2 * G, 2, 1111, 650 + G, ragged=True)
    say(f"case paged cache, page_size=16, G={G}, ragged S<=1111")
    _paged_parity(wl, 16, (3, 0), f"paged G={G}")


def test_paged_cache_long_range_refills_its_page_slots():
    """One workgroup-range longer than the 256 page-number slots per wave (16K keys): the
    stream is refilled mid-range and the softmax state carries across."""
    wl = _generic(1, 8, 1, 70000, 700)
    say("case paged cache, one sequence of 70000 keys, n_splits=1 and 2, page_size 16 and 128")
    for ps in (16, 128):
        _paged_parity(wl, ps, (1, 2), f"paged long ps={ps}", max_splits=2, seed=ps)


def test_paged_cache_short_and_empty_sequences():
    wl = _generic(5, 8, 2, 300, 710)
    say("case paged cache, seq_lens = [0, 1, 300, 16, 17]")
    inp = fi.make_inputs(wl, "cuda")
    inp.seq_lens = torch.tensor([0, 1, 300, 16, 17], dtype=torch.int32, device="cuda")
    pg = fi.make_paged(inp, 16, seed=3)
    ref_o, ref_l = oracle.decode_paged(fi.bits(pg.q), fi.bits(pg.k_pages), fi.bits(pg.v_pages),
                                       pg.block_table.cpu().numpy(), pg.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=4) as dec:
        for n in (0, 1, 4):
            out, lse = dec.decode_paged(pg.q, pg.k_pages, pg.v_pages, pg.block_table, 16, pg.seq_lens, n)
            torch.cuda.synchronize()
            check_out(out.cpu().numpy(), ref_o, f"paged short n={n}")
            check_lse(lse.cpu().numpy(), ref_l, f"paged short n={n}")


def test_paged_argument_errors():
    say("case paged argument validation")
    with fd.FlashDecode(1, 8, 2, 1024, max_splits=4) as dec:
        q = torch.zeros(1, 8, 128, device="cuda", dtype=torch.bfloat16)
        pool = torch.zeros(64, 2, 16, 128, device="cuda", dtype=torch.bfloat16)
        table = torch.zeros(1, 64, device="cuda", dtype=torch.int32)
        sl = torch.full((1,), 1024, device="cuda", dtype=torch.int32)
        out = torch.empty(1, 8, 128, device="cuda")
        for bad_ps in (8, 24, 0):
            with pytest.raises(fd.FdError) as e:
                fd.fd_decode_paged(dec.h, q, pool, pool, table, bad_ps, sl, out, None, 1)
            assert e.value.code == fd.FD_ERR_INVALID_ARG
        with pytest.raises(fd.FdError) as e:                      # table rows too short for S_max
            fd.fd_decode_paged(dec.h, q, pool, pool, table[:, :32].contiguous(), 16, sl, out, None, 1)
        assert e.value.code == fd.FD_ERR_INVALID_ARG
        with pytest.raises(fd.FdError) as e:
            fd.fd_decode_paged(dec.h, q, pool, pool, None, 16, sl, out, None, 1)
        assert e.value.code == fd.FD_ERR_INVALID_ARG
        fd.fd_set_option(dec.h, fd.FD_OPT_PATH, 1)
        with pytest.raises(fd.FdError) as e:
            fd.fd_decode_paged(dec.h, q, pool, pool, table, 16, sl, out, None, 1)
        assert e.value.code == fd.FD_ERR_UNSUPPORTED
        fd.fd_set_option(dec.h, fd.FD_OPT_PATH, 0)
        # out-of-range table entries are clamped into the pool: the call must complete
        table.fill_(10 ** 6)
        fd.fd_decode_paged(dec.h, q, pool, pool, table, 16, sl, out, None, 1)
        torch.cuda.synchronize()
        assert torch.isfinite(out).all()


def test_autotune_leaves_valid_options_and_results():
    say("case fd_autotune on two shapes")
    for wl in (_generic(4, 16, 2, 3000, 800, ragged=True), _generic(2, 12, 3, 900, 801)):
        inp = fi.make_inputs(wl, "cuda")
        ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
        with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=8) as dec:
            out = torch.empty(wl.B, wl.Hq, 128, device="cuda")
            lse = torch.empty(wl.B, wl.Hq, device="cuda")
            us = fd.fd_autotune(dec.h, inp.q, inp.k, inp.v, inp.seq_lens, out, lse, 0, reps=5)
            assert us > 0
            # 0 = the options the handle came with (the defaults' rules) were not beaten
            assert fd.fd_get_option(dec.h, fd.FD_OPT_PATH) in (0, 1, 2)
            assert fd.fd_get_option(dec.h, fd.FD_OPT_XCD_GROUPS) in (0, 1, 8)
            say(f"  chose path {fd.fd_get_option(dec.h, fd.FD_OPT_PATH)} lists {fd.fd_get_option(dec.h, fd.FD_OPT_XCD_GROUPS)} "
                f"per CU {fd.fd_get_option(dec.h, fd.FD_OPT_WGS_PER_CU)} ring {fd.fd_get_option(dec.h, fd.FD_OPT_RING_STAGES)} "
                f"split keys {fd.fd_get_option(dec.h, fd.FD_OPT_SPLIT_KEYS)}: {us:.1f} us")
            check_out(out.cpu().numpy(), ref_o, "autotune result")        # the last timed call's result is valid
            check_lse(lse.cpu().numpy(), ref_l, "autotune result")
            out2, lse2 = run_both(dec, inp, 0)
            check_out(out2, ref_o, "after autotune")
            check_lse(lse2, ref_l, "after autotune")
            with pytest.raises(fd.FdError) as e:
                fd.fd_autotune(dec.h, inp.q, inp.k, inp.v, inp.seq_lens, out, lse, 0, reps=0)
            assert e.value.code == fd.FD_ERR_INVALID_ARG


@pytest.mark.parametrize("dtype", ["fp16", "fp8kv"])
def test_autotune_on_half_and_fp8_handles(dtype):
    """fd_autotune builds its candidates from what the handle's element type is built for (no VALU kernel, no
    deeper rings for half; the MFMA kernel only for FP8) and skips combinations a shape does not allow."""
    wl = _generic(4, 16, 4, 3000, 810, ragged=True)            # G = 4
    say(f"case fd_autotune on a {dtype} handle, G=4")
    ks = vs = 1.0 / 32
    if dtype == "fp16":
        inp = fi.make_inputs(wl, "cuda", dtype=torch.float16)
        k, v = inp.k, inp.v
        ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(k), fi.bits(v), inp.seq_lens.cpu().numpy(), fmt="fp16")
    else:
        inp = fi.make_inputs(wl, "cuda")
        k, v = fi.to_fp8_cache(inp, ks, vs)
        ref_o, ref_l = oracle.decode_fp8kv(fi.bits(inp.q), fi.bytes_of(k), fi.bytes_of(v), inp.seq_lens.cpu().numpy(),
                                           k_scale=ks, v_scale=vs)
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=16, dtype=dtype, k_scale=ks, v_scale=vs) as dec:
        out = torch.empty(wl.B, wl.Hq, 128, device="cuda")
        lse = torch.empty(wl.B, wl.Hq, device="cuda")
        for n in (0, 6):
            us = fd.fd_autotune(dec.h, inp.q, k, v, inp.seq_lens, out, lse, n, reps=5)
            assert us > 0 and fd.fd_get_option(dec.h, fd.FD_OPT_PATH) == 2
            say(f"  n={n}: lists {fd.fd_get_option(dec.h, fd.FD_OPT_XCD_GROUPS)} per CU {fd.fd_get_option(dec.h, fd.FD_OPT_WGS_PER_CU)} "
                f"ring {fd.fd_get_option(dec.h, fd.FD_OPT_RING_STAGES)} split keys {fd.fd_get_option(dec.h, fd.FD_OPT_SPLIT_KEYS)}: {us:.1f} us")
            check_out(out.cpu().numpy(), ref_o, f"autotune {dtype} n={n}")
            check_lse(lse.cpu().numpy(), ref_l, f"autotune {dtype} n={n}")
            out2, lse2 = dec.decode(inp.q, k, v, inp.seq_lens, n)
            torch.cuda.synchronize()
            check_out(out2.cpu().numpy(), ref_o, f"after autotune {dtype} n={n}")
            check_lse(lse2.cpu().numpy(), ref_l, f"after autotune {dtype} n={n}")


def test_autotune_skips_what_a_shape_does_not_allow():
    """More than 2048 tiles with adaptive splits: one work list is not built for that (FD_ERR_UNSUPPORTED), eight
    lists are; the search must skip the former, not fail."""
    wl = _generic(2056, 1, 1, 64, 820)
    say("case fd_autotune with 2056 tiles, adaptive splits")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=2) as dec:
        out = torch.empty(wl.B, wl.Hq, 128, device="cuda")
        lse = torch.empty(wl.B, wl.Hq, device="cuda")
        us = fd.fd_autotune(dec.h, inp.q, inp.k, inp.v, inp.seq_lens, out, lse, 0, reps=3)
        assert us > 0 and fd.fd_get_option(dec.h, fd.FD_OPT_XCD_GROUPS) in (0, 8)     # 0: the default, which is 8 lists here
        check_out(out.cpu().numpy(), ref_o, "autotune 2056 tiles")
        check_lse(lse.cpu().numpy(), ref_l, "autotune 2056 tiles")


@pytest.mark.parametrize("keys", [64, 256, 1024, 4096])
def test_adaptive_split_granularity_option(keys):
    """FD_OPT_SPLIT_KEYS: how finely a tile is cut when the library picks the split count (the granularity
    axis of the autotune).  Any value changes only the partition, i.e. rounding."""
    wl = _generic(6, 16, 2, 9000, 830 + keys, ragged=True)
    say(f"case adaptive splits of {keys} keys, G=8, ragged S<=9000")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=64) as dec:
        fd.fd_set_option(dec.h, fd.FD_OPT_SPLIT_KEYS, keys)
        assert fd.fd_get_option(dec.h, fd.FD_OPT_SPLIT_KEYS) == keys
        for xg in (1, 8) if (wl.B * wl.Hkv) % 8 == 0 else (1,):
            fd.fd_set_option(dec.h, fd.FD_OPT_XCD_GROUPS, xg)
            fd.fd_debug_poison_workspace(dec.h)
            out, lse = run_both(dec, inp, 0)
            check_out(out, ref_o, f"split keys {keys} lists {xg}")
            check_lse(lse, ref_l, f"split keys {keys} lists {xg}")
        for bad in (32, 100, 65600, -64):
            with pytest.raises(fd.FdError) as e:
                fd.fd_set_option(dec.h, fd.FD_OPT_SPLIT_KEYS, bad)
            assert e.value.code == fd.FD_ERR_INVALID_ARG


# ---------------------------------------------------------------- fine-grained waits

@pytest.mark.parametrize("shape", [(2, 16, 2, 3000, 8), (8, 8, 8, 1024, 4), (1, 8, 1, 40000, 64), (3, 12, 3, 700, 0),
                                   (40, 16, 8, 600, 0)])
def test_fine_grained_waits_equal_the_fused_result(shape):
    """fd_decode_waits: kernel 1 and a waiting combine kernel side by side on two streams.
    Same partition and same combine order as the fused kernel: bitwise equal.  Calls are
    repeated back to back and interleaved with fused calls (shared counters must re-arm)."""
    B, Hq, Hkv, S, n = shape
    wl = _generic(B, Hq, Hkv, S, 900 + B + S, ragged=(n == 0))
    say(f"case fine-grained waits B{B} Hq{Hq} Hkv{Hkv} S{S} n{n}")
    inp = fi.make_inputs(wl, "cuda")
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=max(n, 1) if n else 8) as dec:
        fd.fd_debug_poison_workspace(dec.h)
        out_f, lse_f = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n)
        for rep in range(4):
            out_w, lse_w = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n, waits=True)
            if rep == 2:
                dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n)
            torch.cuda.synchronize()
            assert torch.equal(out_w.view(torch.int32), out_f.view(torch.int32)), f"waits != fused (rep {rep})"
            assert torch.equal(lse_w.view(torch.int32), lse_f.view(torch.int32))
        assert fd.fd_get_option(dec.h, fd.FD_INFO_WAIT_GAVE_UP) == 0
        assert all(c == 0 for c in fd.fd_debug_read_counters(dec.h, wl.B * wl.Hkv)), "counters not re-armed"
    check_out(out_w.cpu().numpy(), ref_o, "waits")
    check_lse(lse_w.cpu().numpy(), ref_l, "waits")


def test_fine_grained_waits_give_up_cleanly_when_told_to():
    """The bounded wait, forced from the host: with a spin limit of one poll the combine
    kernel gives up on tiles whose counts are not complete yet; every kernel still ends, the
    condition is reported, and after fd_reset the handle works again."""
    wl = _generic(1, 8, 1, 60000, 950)
    say("case fine-grained waits with FD_OPT_SPIN_LIMIT = 1")
    inp = fi.make_inputs(wl, "cuda")
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=64) as dec:
        out_f, lse_f = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 64)
        fd.fd_set_option(dec.h, fd.FD_OPT_SPIN_LIMIT, 1)
        dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 64, waits=True)
        torch.cuda.synchronize()
        gave_up = fd.fd_get_option(dec.h, fd.FD_INFO_WAIT_GAVE_UP)
        say(f"  gave up: {gave_up}")
        fd.fd_set_option(dec.h, fd.FD_OPT_SPIN_LIMIT, 0)
        fd.fd_reset(dec.h)
        torch.cuda.synchronize()
        assert fd.fd_get_option(dec.h, fd.FD_INFO_WAIT_GAVE_UP) == 0
        out_w, lse_w = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 64, waits=True)
        torch.cuda.synchronize()
        assert torch.equal(out_w.view(torch.int32), out_f.view(torch.int32))
        assert fd.fd_get_option(dec.h, fd.FD_INFO_WAIT_GAVE_UP) == 0
        pool = torch.zeros(64, 1, 16, 128, device="cuda", dtype=torch.bfloat16)
        fd.fd_set_option(dec.h, fd.FD_OPT_PATH, 1)
        with pytest.raises(fd.FdError) as e:
            dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, 64, waits=True)
        assert e.value.code == fd.FD_ERR_UNSUPPORTED


# ---------------------------------------------------------------- IEEE half inputs

@pytest.mark.parametrize("shape", [(2, 8, 8, 1000, 4), (3, 16, 2, 2500, 0), (2, 12, 4, 777, 3), (1, 16, 1, 30000, 37),
                                   (2, 32, 2, 513, 0)])
def test_half_inputs(shape):
    """dtype = FD_DTYPE_FP16 (the paper's precision): same tolerances against the oracle reading
    the same half bit patterns; fused and BSP bitwise equal; paged as well."""
    B, Hq, Hkv, S, n = shape
    wl = _generic(B, Hq, Hkv, S, 1200 + S + Hq, ragged=(n == 0))
    say(f"case half inputs B{B} Hq{Hq} Hkv{Hkv} S{S} n{n}")
    inp = fi.make_inputs(wl, "cuda", dtype=torch.float16)
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy(), fmt="fp16")
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=max(n, 8), dtype="fp16") as dec:
        fd.fd_debug_poison_workspace(dec.h)
        out, lse = run_both(dec, inp, n)
        eo = check_out(out, ref_o, "half")
        el = check_lse(lse, ref_l, "half")
        say(f"  max |out err| {eo:.2e}, max |lse err| {el:.2e}")
        pg = fi.make_paged(inp, 32, seed=1)
        out_p, lse_p = dec.decode_paged(pg.q, pg.k_pages, pg.v_pages, pg.block_table, 32, pg.seq_lens, n)
        out_pb, _ = dec.decode_paged(pg.q, pg.k_pages, pg.v_pages, pg.block_table, 32, pg.seq_lens, n, bsp=True)
        torch.cuda.synchronize()
        assert torch.equal(out_p.view(torch.int32), out_pb.view(torch.int32))
        check_out(out_p.cpu().numpy(), ref_o, "half paged")
        check_lse(lse_p.cpu().numpy(), ref_l, "half paged")
        fd.fd_set_option(dec.h, fd.FD_OPT_PATH, 1)
        with pytest.raises(fd.FdError) as e:
            dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n)
        assert e.value.code == fd.FD_ERR_UNSUPPORTED
        fd.fd_set_option(dec.h, fd.FD_OPT_PATH, 0)
        with pytest.raises(fd.FdError) as e:
            dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n, waits=True)
        assert e.value.code == fd.FD_ERR_UNSUPPORTED


def test_half_inputs_peaked_attention():
    """Two dominant keys with opposite values in half precision (weights near 0.5 each, everything else tiny)."""
    wl = _generic(1, 8, 1, 4096, 1300)
    inp = fi.make_inputs(wl, "cuda", dtype=torch.float16)
    inp.k[0, 0, 100] = inp.q[0, 0] * 3.0
    inp.k[0, 0, 3000] = inp.q[0, 0] * 3.0
    inp.v[0, 0, 100] = 50.0
    inp.v[0, 0, 3000] = -50.0
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy(), fmt="fp16")
    with fd.FlashDecode(1, 8, 1, 4096, max_splits=16, dtype="fp16") as dec:
        out, lse = run_both(dec, inp, 16)
    check_out(out, ref_o, "half peaked")
    check_lse(lse, ref_l, "half peaked")


# ---------------------------------------------------------------- FP8 (E4M3) KV cache

@pytest.mark.parametrize("shape", [(2, 8, 8, 1000, 4), (3, 16, 2, 2500, 0), (2, 12, 4, 777, 3), (1, 16, 1, 30000, 37),
                                   (2, 32, 2, 513, 0), (1, 8, 1, 31, 1), (1, 8, 1, 33, 2), (4, 4, 4, 64, 0)])
def test_fp8_kv_cache(shape):
    """dtype = FD_DTYPE_FP8_KV: bf16 q, E4M3 K/V bytes with per-tensor scales.  The oracle reads the same bytes;
    the kernel converts them exactly, so the tolerances are the bf16 ones."""
    B, Hq, Hkv, S, n = shape
    wl = _generic(B, Hq, Hkv, S, 1400 + S + Hq, ragged=(n == 0))
    say(f"case FP8 KV cache B{B} Hq{Hq} Hkv{Hkv} S{S} n{n}")
    inp = fi.make_inputs(wl, "cuda")
    ks, vs = 1.0 / 32, 1.0 / 16
    k8, v8 = fi.to_fp8_cache(inp, ks, vs)
    ref_o, ref_l = oracle.decode_fp8kv(fi.bits(inp.q), fi.bytes_of(k8), fi.bytes_of(v8), inp.seq_lens.cpu().numpy(),
                                       k_scale=ks, v_scale=vs)
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=max(n, 8), dtype="fp8kv", k_scale=ks, v_scale=vs) as dec:
        fd.fd_debug_poison_workspace(dec.h)
        out_f, lse_f = dec.decode(inp.q, k8, v8, inp.seq_lens, n)
        out_b, lse_b = dec.decode(inp.q, k8, v8, inp.seq_lens, n, bsp=True)
        torch.cuda.synchronize()
        assert torch.equal(out_f.view(torch.int32), out_b.view(torch.int32)) and torch.equal(lse_f, lse_b)
        eo = check_out(out_f.cpu().numpy(), ref_o, "fp8 kv")
        el = check_lse(lse_f.cpu().numpy(), ref_l, "fp8 kv")
        say(f"  max |out err| {eo:.2e}, max |lse err| {el:.2e}")
        fd.fd_set_option(dec.h, fd.FD_OPT_WGS_PER_CU, 2)
        out_2, lse_2 = dec.decode(inp.q, k8, v8, inp.seq_lens, n)
        torch.cuda.synchronize()
        check_out(out_2.cpu().numpy(), ref_o, "fp8 kv, 2 per CU")
        fd.fd_set_option(dec.h, fd.FD_OPT_WGS_PER_CU, 0)
        with pytest.raises(fd.FdError) as e:
            dec.decode(inp.q, k8, v8, inp.seq_lens, n, waits=True)
        assert e.value.code == fd.FD_ERR_UNSUPPORTED


def test_fp8_kv_cache_every_byte_value():
    """A cache holding every finite E4M3 byte (both signs, subnormals, the 448 maximum) with tiny scales."""
    wl = _generic(1, 8, 1, 512, 1500)
    inp = fi.make_inputs(wl, "cuda")
    allb = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    allb[allb == 0x7F] = 0x7E
    allb[allb == 0xFF] = 0xFE
    gen = torch.Generator().manual_seed(3)
    kb = allb[torch.randint(0, 256, (1, 1, 512, 128), generator=gen)].cuda()
    vb = allb[torch.randint(0, 256, (1, 1, 512, 128), generator=gen)].cuda()
    k8, v8 = kb.view(torch.float8_e4m3fn), vb.view(torch.float8_e4m3fn)
    ks, vs = 1.0 / 4096, 1.0 / 8
    ref_o, ref_l = oracle.decode_fp8kv(fi.bits(inp.q), fi.bytes_of(k8), fi.bytes_of(v8), inp.seq_lens.cpu().numpy(),
                                       k_scale=ks, v_scale=vs)
    with fd.FlashDecode(1, 8, 1, 512, max_splits=8, dtype="fp8kv", k_scale=ks, v_scale=vs) as dec:
        out, lse = dec.decode(inp.q, k8, v8, inp.seq_lens, 4)
        torch.cuda.synchronize()
    ref_scale = np.abs(ref_o).max()
    say(f"case FP8 every byte value: |out| up to {ref_scale:.2f}")
    check_out(out.cpu().numpy(), ref_o, "fp8 all bytes")
    check_lse(lse.cpu().numpy(), ref_l, "fp8 all bytes")


@pytest.mark.parametrize("page_size", [32, 64, 256])
def test_fp8_kv_cache_paged(page_size):
    wl = _generic(3, 16, 2, 2500, 1600 + page_size, ragged=True)
    say(f"case FP8 KV cache, paged, page_size={page_size}, G=8, ragged S<=2500")
    inp = fi.make_inputs(wl, "cuda")
    ks, vs = 1.0 / 32, 1.0 / 16
    inp.k, inp.v = fi.to_fp8_cache(inp, ks, vs)
    pg = fi.make_paged(inp, page_size, seed=2)
    ref_o, ref_l = oracle.decode_fp8kv_paged(fi.bits(pg.q), fi.bytes_of(pg.k_pages), fi.bytes_of(pg.v_pages),
                                             pg.block_table.cpu().numpy(), pg.seq_lens.cpu().numpy(), k_scale=ks, v_scale=vs)
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=8, dtype="fp8kv", k_scale=ks, v_scale=vs) as dec:
        for n in (1, 5, 0):
            fd.fd_debug_poison_workspace(dec.h)
            out_f, lse_f = dec.decode_paged(pg.q, pg.k_pages, pg.v_pages, pg.block_table, page_size, pg.seq_lens, n)
            out_b, lse_b = dec.decode_paged(pg.q, pg.k_pages, pg.v_pages, pg.block_table, page_size, pg.seq_lens, n, bsp=True)
            out_c, lse_c = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n)
            torch.cuda.synchronize()
            assert torch.equal(out_f.view(torch.int32), out_b.view(torch.int32)) and torch.equal(lse_f, lse_b)
            assert torch.allclose(out_f, out_c, rtol=1e-5, atol=1e-6)
            check_out(out_f.cpu().numpy(), ref_o, f"fp8 paged n={n}")
            check_lse(lse_f.cpu().numpy(), ref_l, f"fp8 paged n={n}")
        pool16 = fi.make_paged(inp, 16, seed=2)
        with pytest.raises(fd.FdError) as e:
            dec.decode_paged(pool16.q, pool16.k_pages, pool16.v_pages, pool16.block_table, 16, pool16.seq_lens, 1)
        assert e.value.code == fd.FD_ERR_UNSUPPORTED


def test_calls_recorded_into_a_hip_graph_replay_like_eager_calls():
    """fd_reset, fd_decode, fd_decode_bsp and fd_decode_static only launch kernels on the caller's
    stream (no memset node, no allocation, no host wait), so a stream holding them can be recorded
    into a HIP graph.  Every replay sees the CURRENT contents of q and seq_lens (both are read on the
    device) and must equal an eager call on the same contents bit for bit; eager work and
    synchronisations lie between the replays."""
    wl = fi.Workload("graph", 8101, B=4, Hq=32, Hkv=8, S_max=5000, n_splits=12, ragged=True)
    say(f"case {wl.name} B{wl.B} Hq{wl.Hq} Hkv{wl.Hkv} S{wl.S_max} n{wl.n_splits}")
    inp = fi.make_inputs(wl, "cuda")
    cfg = fd.fd_config(wl.B, wl.Hq, wl.Hkv, 128, wl.S_max, 16, 0, 0.0, fd.FD_DTYPE_BF16, 0.0, 0.0)
    q = inp.q.clone()
    sl = inp.seq_lens.clone()
    outs = {name: torch.empty(wl.B, wl.Hq, 128, device="cuda") for name in ("fused", "bsp", "static")}
    lses = {name: torch.empty(wl.B, wl.Hq, device="cuda") for name in outs}
    side = torch.cuda.Stream()
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=16) as dec, \
            fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=16) as eager:

        def record(st):
            fd.fd_reset(dec.h, st)
            fd.fd_decode(dec.h, q, inp.k, inp.v, sl, outs["fused"], lses["fused"], wl.n_splits, st)
            fd.fd_decode_bsp(dec.h, q, inp.k, inp.v, sl, outs["bsp"], lses["bsp"], wl.n_splits, st)
            fd.fd_decode_static(cfg, q, inp.k, inp.v, sl, outs["static"], lses["static"], wl.n_splits, st)

        # once outside the capture: per-kernel and per-device set-up happens on a first call
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            record(side.cuda_stream)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            record(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()

        gen = torch.Generator(device="cuda").manual_seed(8102)
        for rep in range(4):
            say(f"  replay {rep}")
            q.copy_(torch.randn(q.shape, device="cuda", generator=gen).to(torch.bfloat16))
            # new lengths within the rows that hold data (past the workload's own lengths lies NaN)
            frac = torch.rand(sl.shape, device="cuda", generator=gen)
            sl.copy_(torch.minimum((frac * (inp.seq_lens + 1)).to(torch.int32), inp.seq_lens).clamp_(min=1))
            if rep == 2:
                sl[0] = 0
            ref_o, ref_l = eager.decode(q, inp.k, inp.v, sl, wl.n_splits)
            for name in outs:
                outs[name].fill_(float("nan"))
                lses[name].fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name in outs:
                assert torch.equal(outs[name].view(torch.int32), ref_o.view(torch.int32)), f"replay {rep}: {name} out differs from eager"
                assert torch.equal(lses[name].view(torch.int32), ref_l.view(torch.int32)), f"replay {rep}: {name} lse differs from eager"
        o64, l64 = oracle.decode(fi.bits(q), fi.bits(inp.k), fi.bits(inp.v), sl.cpu().numpy())
        check_out(outs["fused"].cpu().numpy(), o64, "graph replay")
        check_lse(lses["fused"].cpu().numpy(), l64, "graph replay")


def test_two_handles_on_two_streams_at_once():
    """Two persistent launches share the GPU: neither fits beside the other completely, so workgroups of one
    start only as workgroups of the other leave.  No workgroup ever waits for another (the last arriver
    combines), so both finish, and each call's result is that of the call run alone, bit for bit."""
    wa = fi.Workload("conc_a", 8201, B=8, Hq=32, Hkv=8, S_max=4096, n_splits=16)
    wb = fi.Workload("conc_b", 8202, B=1, Hq=8, Hkv=1, S_max=16384, n_splits=256)      # two-level combine
    say("case two handles, two streams, 200 overlapping calls each")
    ia, ib = fi.make_inputs(wa, "cuda"), fi.make_inputs(wb, "cuda")
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    with fd.FlashDecode(wa.B, wa.Hq, wa.Hkv, wa.S_max, max_splits=16) as da, \
            fd.FlashDecode(wb.B, wb.Hq, wb.Hkv, wb.S_max, max_splits=256) as db:
        alone_a = da.decode(ia.q, ia.k, ia.v, ia.seq_lens, 16)
        alone_b = db.decode(ib.q, ib.k, ib.v, ib.seq_lens, 256)
        torch.cuda.synchronize()
        outs_a = [torch.empty_like(alone_a[0]) for _ in range(4)]
        outs_b = [torch.empty_like(alone_b[0]) for _ in range(4)]
        lse_a, lse_b = torch.empty_like(alone_a[1]), torch.empty_like(alone_b[1])
        for i in range(200):
            bsp = i % 3 == 2
            da.decode(ia.q, ia.k, ia.v, ia.seq_lens, 16, out=outs_a[i % 4], lse=lse_a, bsp=bsp, stream=sa.cuda_stream)
            db.decode(ib.q, ib.k, ib.v, ib.seq_lens, 256, out=outs_b[i % 4], lse=lse_b, bsp=bsp, stream=sb.cuda_stream)
        torch.cuda.synchronize()
        for o in outs_a:
            assert torch.equal(o.view(torch.int32), alone_a[0].view(torch.int32)), "stream A: result differs from the call run alone"
        for o in outs_b:
            assert torch.equal(o.view(torch.int32), alone_b[0].view(torch.int32)), "stream B: result differs from the call run alone"
        assert all(c == 0 for c in fd.fd_debug_read_counters(da.h, wa.B * wa.Hkv))
        assert all(c == 0 for c in fd.fd_debug_read_counters(db.h, wb.B * wb.Hkv))
