"""The entry point that allocates nothing (fd_decode_static) against fd_decode on a handle.

Same kernels, same launch shape: results must be bitwise equal, and each is also held to the
oracle's tolerances.  Two calls in a row share the one static workspace, the second on a smaller
input; further calls switch dtype and shape again.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2511_02168_amd import binding as fd
from paper_2511_02168_amd import inputs as fi

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _cfg(wl, S, max_splits, dtype=fd.FD_DTYPE_BF16, ks=0.0, vs=0.0):
    return fd.fd_config(wl.B, wl.Hq, wl.Hkv, 128, S, max_splits, 0, 0.0, dtype, ks, vs)


def _one(wl, n_splits, max_splits, what):
    say(f"case static workspace: {what} B{wl.B} Hq{wl.Hq} Hkv{wl.Hkv} S{wl.S_max} n{n_splits}")
    inp = fi.make_inputs(wl, "cuda")
    cfg = _cfg(wl, wl.S_max, max_splits)
    out_s = torch.full((wl.B, wl.Hq, 128), float("nan"), device="cuda")
    lse_s = torch.full((wl.B, wl.Hq), float("nan"), device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    fd.fd_decode_static(cfg, inp.q, inp.k, inp.v, inp.seq_lens, out_s, lse_s, n_splits, stream)
    with fd.FlashDecode(wl.B, wl.Hq, wl.Hkv, wl.S_max, max_splits=max_splits) as dec:
        out_h, lse_h = dec.decode(inp.q, inp.k, inp.v, inp.seq_lens, n_splits)
        torch.cuda.synchronize()
    assert torch.equal(out_s.view(torch.int32), out_h.view(torch.int32)), f"{what}: static != handle (out)"
    assert torch.equal(lse_s.view(torch.int32), lse_h.view(torch.int32)), f"{what}: static != handle (lse)"
    ref_o, ref_l = oracle.decode(fi.bits(inp.q), fi.bits(inp.k), fi.bits(inp.v), inp.seq_lens.cpu().numpy())
    o = out_s.cpu().numpy().astype(np.float64)
    l = lse_s.cpu().numpy().astype(np.float64)
    assert (np.abs(o - ref_o) <= 2e-3 + 2e-3 * np.abs(ref_o)).all(), f"{what}: out outside tolerance"
    assert (np.abs(l - ref_l) <= 1e-4 * np.maximum(1.0, np.abs(ref_l))).all(), f"{what}: lse outside tolerance"


def test_static_workspace_entry_point_matches_the_handle():
    big = fi.Workload("static_big", 7001, B=4, Hq=32, Hkv=8, S_max=6000, n_splits=16, ragged=True)
    small = fi.Workload("static_small", 7002, B=2, Hq=8, Hkv=2, S_max=700, n_splits=3)
    _one(big, 16, 16, "first call")
    _one(small, 3, 4, "second call, smaller input")                 # leftovers of the first call lie in the workspace
    _one(big, 0, 16, "third call, adaptive splits")
    _one(fi.Workload("static_g8", 7003, B=1, Hq=16, Hkv=2, S_max=20000, n_splits=64), 64, 64, "fourth call, G=8")


def test_static_workspace_refuses_shapes_beyond_its_size():
    wl = fi.Workload("static_too_big", 7004, B=64, Hq=32, Hkv=8, S_max=1024, n_splits=0)
    cfg = _cfg(wl, 1024, 64)                                        # 512 tiles x 64 slots x 4 heads x 512 B = 64 MiB
    assert fd.fd_workspace_bytes(cfg) > fd.FD_STATIC_SCRATCH_BYTES
    q = torch.zeros(wl.B, wl.Hq, 128, device="cuda", dtype=torch.bfloat16)
    kv = torch.zeros(wl.B, wl.Hkv, 1024, 128, device="cuda", dtype=torch.bfloat16)
    sl = torch.full((wl.B,), 1024, device="cuda", dtype=torch.int32)
    out = torch.empty(wl.B, wl.Hq, 128, device="cuda")
    with pytest.raises(fd.FdError) as e:
        fd.fd_decode_static(cfg, q, kv, kv, sl, out, None, 0)
    assert e.value.code == fd.FD_ERR_WORKSPACE
    assert "static workspace" in str(e.value)
