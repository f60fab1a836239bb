"""Seeded synthetic inputs for the Flash Decode workloads.

This module only draws random numbers and lays them out; it contains none of
the attention arithmetic and is the one module both the HIP path's tests and
the CPU oracle's tests may share.

The paper's Flash Decode experiment (Section 5.3) is batch 1, 96 query heads,
head dimension 128, a KV cache sharded over 8 GPUs and a sweep of global KV
lengths; it uses no public dataset and does not state the value distribution
of its tensors.  The five workloads below are seeded stand-ins with the same
structure (single-query decode, D = 128, grouped KV heads, long KV ranges).

Tensors are produced with torch on the requested device (CPU or GPU), in fp32,
then rounded to bf16 (round-to-nearest-even); ``bits()`` hands the exact bf16
bit patterns to numpy as uint16.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

BASE_SEED = 20251102
D_HEAD = 128


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    Hq: int
    Hkv: int
    S_max: int
    n_splits: int            # 0 = adaptive (library decides per sequence)
    ragged: bool = False     # seq_lens ~ U[1, S_max]
    k_scale: float = 1.0     # K multiplied by this before rounding
    aligned_frac: float = 0.0  # fraction of keys rotated toward q (peaked attention)
    D: int = D_HEAD

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


# The five configurations of the benchmark definition, in its order.
WORKLOADS: List[Workload] = [
    Workload("c1_tiny_mha", 0, B=1, Hq=8, Hkv=8, S_max=1024, n_splits=4),
    Workload("c2_gqa_llama8b", 1, B=8, Hq=32, Hkv=8, S_max=8192, n_splits=16),
    Workload("c3_head_shard_g8", 2, B=32, Hq=8, Hkv=1, S_max=16384, n_splits=32),
    Workload("c4_ragged", 3, B=64, Hq=32, Hkv=8, S_max=32768, n_splits=0, ragged=True,
             k_scale=0.5),
    Workload("c5_long_context", 4, B=1, Hq=64, Hkv=8, S_max=131072, n_splits=256,
             aligned_frac=0.01),
]


def workload(name_or_index) -> Workload:
    for w in WORKLOADS:
        if w.name == name_or_index or w.index == name_or_index or \
                w.name.split("_")[0] == str(name_or_index).lower():
            return w
    raise KeyError(name_or_index)


@dataclass
class Inputs:
    q: torch.Tensor          # [B, Hq, D] bf16
    k: torch.Tensor          # [B, Hkv, S_max, D] bf16
    v: torch.Tensor          # [B, Hkv, S_max, D] bf16
    seq_lens: torch.Tensor   # [B] int32
    wl: Workload = field(repr=False, default=None)


def to_fp8_cache(inp: "Inputs", k_scale: float = 1.0 / 32, v_scale: float = 1.0 / 32):
    """K and V of a bf16 workload quantised to OCP E4M3 bytes standing for value * scale: returns (k8, v8) as
    torch.float8_e4m3fn tensors of the same shape (NaN padding stays NaN).  N(0,1) / (1/32) stays far below 448."""
    k8 = (inp.k.to(torch.float32) / k_scale).to(torch.float8_e4m3fn)
    v8 = (inp.v.to(torch.float32) / v_scale).to(torch.float8_e4m3fn)
    return k8, v8


def bytes_of(t: torch.Tensor) -> np.ndarray:
    """Raw bytes of an 8-bit tensor as a host uint8 array."""
    return t.contiguous().view(torch.uint8).cpu().numpy()


def bits(t: torch.Tensor) -> np.ndarray:
    """Exact bit patterns of a bf16 (or fp16) tensor as a host uint16 array."""
    assert t.dtype in (torch.bfloat16, torch.float16)
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even), returning uint16 bit patterns (numpy only)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _align_keys(k32: torch.Tensor, q32: torch.Tensor, frac: float, gen: torch.Generator) -> None:
    """Rotate a seeded subset of keys toward the queries that share them (in place).

    k32 [Hkv, S, D], q32 [Hq, D] (one batch entry).  Per KV head, floor(frac*S)
    distinct key indices are drawn; key j is aimed at query head g = j mod G of
    its group:  k_j <- |k_j| * (0.9 * qhat_g + sqrt(0.19) * nhat), where nhat is
    the unit part of the old k_j orthogonal to qhat_g.  cos(k_j, q_g) = 0.9, the
    norm of k_j is kept, so its score is about 0.9 * |q||k| / sqrt(D) ~ 10.
    """
    Hkv, S, D = k32.shape
    G = q32.shape[0] // Hkv
    n_al = int(math.floor(frac * S))
    if n_al <= 0:
        return
    for kvh in range(Hkv):
        idx = torch.randperm(S, generator=gen, device=k32.device)[:n_al]
        g = idx % G
        qh = q32[kvh * G + g]                                  # [n_al, D]
        qhat = qh / qh.norm(dim=-1, keepdim=True)
        kj = k32[kvh, idx]                                     # [n_al, D]
        norm = kj.norm(dim=-1, keepdim=True)
        ortho = kj - (kj * qhat).sum(-1, keepdim=True) * qhat
        nhat = ortho / ortho.norm(dim=-1, keepdim=True)
        k32[kvh, idx] = norm * (0.9 * qhat + math.sqrt(0.19) * nhat)


def make_inputs(wl: Workload, device="cpu", S_max: Optional[int] = None,
                B: Optional[int] = None, nan_pad: bool = True, dtype: torch.dtype = torch.bfloat16) -> Inputs:
    """Draw q, K, V ~ N(0,1) (K scaled by wl.k_scale), round to bf16.

    S_max / B override the workload's sizes (for reduced copies the oracle can
    finish quickly); the structure (head layout, raggedness, aligned keys) stays.
    For ragged workloads, positions >= seq_lens[b] are filled with NaN so any
    read past the sequence end poisons the result.
    """
    S = int(S_max if S_max is not None else wl.S_max)
    Bn = int(B if B is not None else wl.B)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed)
    q32 = torch.randn(Bn, wl.Hq, wl.D, generator=gen, device=dev, dtype=torch.float32)
    q = q32.to(dtype)
    if wl.ragged:
        sl = torch.randint(1, S + 1, (Bn,), generator=gen, device=dev, dtype=torch.int32)
    else:
        sl = torch.full((Bn,), S, device=dev, dtype=torch.int32)
    k = torch.empty(Bn, wl.Hkv, S, wl.D, device=dev, dtype=dtype)
    v = torch.empty(Bn, wl.Hkv, S, wl.D, device=dev, dtype=dtype)
    sl_host = sl.cpu().tolist()
    for b in range(Bn):                      # one batch entry at a time bounds the fp32 temporaries
        k32 = torch.randn(wl.Hkv, S, wl.D, generator=gen, device=dev, dtype=torch.float32)
        v32 = torch.randn(wl.Hkv, S, wl.D, generator=gen, device=dev, dtype=torch.float32)
        if wl.k_scale != 1.0:
            k32 *= wl.k_scale
        if wl.aligned_frac > 0.0:
            # aim at the bf16-rounded q the kernels will actually see
            _align_keys(k32, q[b].to(torch.float32), wl.aligned_frac, gen)
        if wl.ragged and nan_pad and sl_host[b] < S:
            k32[:, sl_host[b]:, :] = float("nan")
            v32[:, sl_host[b]:, :] = float("nan")
        k[b] = k32.to(dtype)
        v[b] = v32.to(dtype)
    return Inputs(q=q, k=k, v=v, seq_lens=sl, wl=wl)


@dataclass
class PagedInputs:
    q: torch.Tensor            # [B, Hq, D] bf16
    k_pages: torch.Tensor      # [num_pages, Hkv, page_size, D] bf16
    v_pages: torch.Tensor      # [num_pages, Hkv, page_size, D] bf16
    block_table: torch.Tensor  # [B, max_pages_per_seq] int32
    seq_lens: torch.Tensor     # [B] int32
    page_size: int = 16


def make_paged(inp: Inputs, page_size: int, seed: int = 0) -> PagedInputs:
    """Scatters a contiguous cache into a page pool: the pages a sequence reaches get distinct
    pool slots in a seeded random order; the pool holds one extra page of NaN, and every table
    entry past a sequence's last page points at it (a read through such an entry poisons the
    result).  Rows of the last page past seq_lens[b] keep what the contiguous cache held there.
    """
    kv_dtype = inp.k.dtype
    k_src, v_src = inp.k, inp.v
    if kv_dtype == torch.float8_e4m3fn:                 # moved as raw bytes; 0x7f is the E4M3 NaN
        k_src, v_src = inp.k.view(torch.uint8), inp.v.view(torch.uint8)
    B, Hkv, S, D = inp.k.shape
    dev = inp.k.device
    max_pages = -(-S // page_size)
    sl = inp.seq_lens.cpu().tolist()
    used = [-(-s // page_size) for s in sl]
    n_used = sum(used)
    gen = torch.Generator(device="cpu")
    gen.manual_seed(1000003 * page_size + seed)
    slots = torch.randperm(n_used, generator=gen).tolist()
    nan_page = n_used
    fill = 0x7F if kv_dtype == torch.float8_e4m3fn else float("nan")
    k_pages = torch.full((n_used + 1, Hkv, page_size, D), fill, device=dev, dtype=k_src.dtype)
    v_pages = torch.full((n_used + 1, Hkv, page_size, D), fill, device=dev, dtype=k_src.dtype)
    table = torch.full((B, max_pages), nan_page, dtype=torch.int32)
    it = iter(slots)
    for b in range(B):
        for pg in range(used[b]):
            slot = next(it)
            table[b, pg] = slot
            lo, hi = pg * page_size, min((pg + 1) * page_size, S)
            k_pages[slot, :, : hi - lo] = k_src[b, :, lo:hi]
            v_pages[slot, :, : hi - lo] = v_src[b, :, lo:hi]
    if kv_dtype == torch.float8_e4m3fn:
        k_pages, v_pages = k_pages.view(kv_dtype), v_pages.view(kv_dtype)
    return PagedInputs(q=inp.q, k_pages=k_pages, v_pages=v_pages, block_table=table.to(dev),
                       seq_lens=inp.seq_lens, page_size=page_size)


def algorithmic_bytes(wl: Workload, seq_lens, kv_elem_bytes: int = 2) -> int:
    """Bytes the method must move: K and V rows of every live key once, q in, out + lse out."""
    lens = [int(s) for s in seq_lens]
    B = len(lens)
    kv = sum(lens) * wl.Hkv * wl.D * kv_elem_bytes * 2
    return kv + B * wl.Hq * wl.D * 2 + B * wl.Hq * wl.D * 4 + B * wl.Hq * 4


def algorithmic_flops(wl: Workload, seq_lens) -> int:
    return 4 * wl.Hq * wl.D * int(sum(int(s) for s in seq_lens))
