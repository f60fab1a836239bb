"""fp64 CPU oracle for Flash Decode -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Thin ctypes access to ``fd_oracle.c`` (plain C, fp64, two-pass softmax
attention + LSE, and the online-softmax Combine of Algorithm 4, Part 2).
Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline
leg may import this package; the HIP library and its Python binding never do,
and this package imports nothing from them.

Inputs are raw bf16 bit patterns held in ``numpy.uint16`` arrays (numpy has no
bf16 type); the C code widens them exactly to fp64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fd_oracle.c")
_LIB = os.path.join(_HERE, "libfd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile fd_oracle.c with gcc into oracle/libfd_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        i32p = ctypes.POINTER(ctypes.c_int32)
        f64p = ctypes.POINTER(ctypes.c_double)
        lib.fd_oracle_decode.restype = ctypes.c_int
        lib.fd_oracle_decode.argtypes = [u16p, u16p, u16p, i32p, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                         ctypes.c_double, ctypes.c_int, f64p, f64p]
        lib.fd_oracle_decode_fmt.restype = ctypes.c_int
        lib.fd_oracle_decode_fmt.argtypes = lib.fd_oracle_decode.argtypes + [ctypes.c_int]
        lib.fd_oracle_element.restype = ctypes.c_double
        lib.fd_oracle_element.argtypes = [ctypes.c_uint16, ctypes.c_int]
        lib.fd_oracle_element_fp8.restype = ctypes.c_double
        lib.fd_oracle_element_fp8.argtypes = [ctypes.c_uint8]
        lib.fd_oracle_decode_fp8kv.restype = ctypes.c_int
        lib.fd_oracle_decode_fp8kv.argtypes = [u16p, ctypes.POINTER(ctypes.c_uint8), ctypes.POINTER(ctypes.c_uint8), i32p,
                                               ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                               ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_int, f64p, f64p]
        lib.fd_oracle_partial.restype = ctypes.c_int
        lib.fd_oracle_partial.argtypes = [u16p, u16p, u16p, ctypes.c_int, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_int64, ctypes.c_double,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int64,
                                          ctypes.c_int64, f64p, f64p]
        lib.fd_oracle_merge.restype = ctypes.c_int
        lib.fd_oracle_merge.argtypes = [f64p, f64p, ctypes.c_int, ctypes.c_int, f64p, f64p]
        lib.fd_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _u16(a: np.ndarray, ndim: int, name: str) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16 or a.ndim != ndim:
        raise TypeError(f"{name}: expected uint16 (bf16 bits) array with {ndim} dims, "
                        f"got {a.dtype} with {a.ndim}")
    return a


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def max_threads() -> int:
    return int(_load().fd_oracle_max_threads())


FORMATS = {"bf16": 0, "fp16": 1}


def element(bits: int, fmt: str = "bf16") -> float:
    """Exact value of one stored 16-bit element."""
    return float(_load().fd_oracle_element(int(bits), FORMATS[fmt]))


def decode(q: np.ndarray, k: np.ndarray, v: np.ndarray, seq_lens: np.ndarray,
           scale: float = 0.0, n_threads: int = 0, fmt: str = "bf16"):
    """softmax(scale * q K^T) V and LSE for every (b, h).

    q [B,Hq,D], k/v [B,Hkv,S_max,D] as bf16 (or, fmt="fp16", IEEE half) bits; seq_lens [B] int32.
    Returns (out [B,Hq,D] float64, lse [B,Hq] float64, natural log).
    """
    q = _u16(q, 3, "q")
    k = _u16(k, 4, "k")
    v = _u16(v, 4, "v")
    B, Hq, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[3] != D:
        raise ValueError(f"shape mismatch: q {q.shape}, k {k.shape}, v {v.shape}")
    Hkv, S_max = k.shape[1], k.shape[2]
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if sl.shape != (B,):
        raise ValueError("seq_lens must have shape [B]")
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    rc = _load().fd_oracle_decode_fmt(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16),
                                      _ptr(v, ctypes.c_uint16), _ptr(sl, ctypes.c_int32),
                                      B, Hq, Hkv, D, S_max, float(scale), int(n_threads),
                                      _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double), FORMATS[fmt])
    if rc != 0:
        raise ValueError("fd_oracle_decode rejected its arguments")
    return out, lse


def partial(q: np.ndarray, k: np.ndarray, v: np.ndarray, b: int, h: int, j0: int, j1: int,
            scale: float = 0.0):
    """Attention of query row (b, h) over keys [j0, j1) only: (o [D], lse)."""
    q = _u16(q, 3, "q")
    k = _u16(k, 4, "k")
    v = _u16(v, 4, "v")
    _, Hq, D = q.shape
    Hkv, S_max = k.shape[1], k.shape[2]
    if not (0 <= b < q.shape[0]) or k.shape != v.shape or k.shape[0] != q.shape[0]:
        raise ValueError("bad batch index or shapes")
    o = np.empty(D, dtype=np.float64)
    lse = np.empty(1, dtype=np.float64)
    rc = _load().fd_oracle_partial(_ptr(q, ctypes.c_uint16), _ptr(k, ctypes.c_uint16),
                                   _ptr(v, ctypes.c_uint16), Hq, Hkv, D, S_max, float(scale),
                                   int(b), int(h), int(j0), int(j1),
                                   _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError("fd_oracle_partial rejected its arguments")
    return o, float(lse[0])


def merge(part_o: np.ndarray, part_lse: np.ndarray):
    """Combine n normalised partials: part_o [n, D], part_lse [n] -> (o [D], lse)."""
    po = np.ascontiguousarray(part_o, dtype=np.float64)
    pl = np.ascontiguousarray(part_lse, dtype=np.float64)
    if po.ndim != 2 or pl.shape != (po.shape[0],):
        raise ValueError("part_o must be [n, D] and part_lse [n]")
    n, D = po.shape
    o = np.empty(D, dtype=np.float64)
    lse = np.empty(1, dtype=np.float64)
    rc = _load().fd_oracle_merge(_ptr(po, ctypes.c_double), _ptr(pl, ctypes.c_double), n, D,
                                 _ptr(o, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError("fd_oracle_merge rejected its arguments")
    return o, float(lse[0])


def decode_paged(q: np.ndarray, k_pages: np.ndarray, v_pages: np.ndarray, block_table: np.ndarray,
                 seq_lens: np.ndarray, scale: float = 0.0, n_threads: int = 0, fmt: str = "bf16"):
    """The same attention over a paged KV cache, by its definition: key j of sequence b is
    row j % page_size of page block_table[b, j // page_size].

    q [B,Hq,D]; k_pages/v_pages [num_pages,Hkv,page_size,D] as bf16 bits; block_table
    [B,max_pages] int; seq_lens [B].  Every sequence's keys are copied out of their pages
    into a contiguous cache, one row at a time, and handed to decode(); table entries of
    pages a sequence does not reach are never looked at.
    """
    q = _u16(q, 3, "q")
    kp = _u16(k_pages, 4, "k_pages")
    vp = _u16(v_pages, 4, "v_pages")
    if kp.shape != vp.shape:
        raise ValueError("k_pages and v_pages differ in shape")
    num_pages, Hkv, page_size, D = kp.shape
    B = q.shape[0]
    bt = np.asarray(block_table)
    sl = np.asarray(seq_lens, dtype=np.int64)
    if bt.ndim != 2 or bt.shape[0] != B or sl.shape != (B,):
        raise ValueError("block_table must be [B, max_pages], seq_lens [B]")
    if (sl < 0).any() or (sl > bt.shape[1] * page_size).any():
        raise ValueError("a sequence is longer than its block table")
    S_max = max(1, int(sl.max()) if B else 1)
    k = np.zeros((B, Hkv, S_max, D), dtype=np.uint16)
    v = np.zeros((B, Hkv, S_max, D), dtype=np.uint16)
    for b in range(B):
        for j in range(int(sl[b])):
            page = int(bt[b, j // page_size])
            if not 0 <= page < num_pages:
                raise ValueError(f"block_table[{b}, {j // page_size}] = {page} is not a page")
            k[b, :, j, :] = kp[page, :, j % page_size, :]
            v[b, :, j, :] = vp[page, :, j % page_size, :]
    return decode(q, k, v, sl.astype(np.int32), scale=scale, n_threads=n_threads, fmt=fmt)


def element_fp8(bits: int) -> float:
    """Exact value of one OCP E4M3 byte."""
    return float(_load().fd_oracle_element_fp8(int(bits)))


def decode_fp8kv(q: np.ndarray, k: np.ndarray, v: np.ndarray, seq_lens: np.ndarray, k_scale: float = 1.0,
                 v_scale: float = 1.0, scale: float = 0.0, n_threads: int = 0):
    """Attention over an FP8 (E4M3) KV cache: q [B,Hq,D] bf16 bits (uint16); k, v [B,Hkv,S_max,D]
    uint8 bytes standing for value * k_scale / v_scale.  Returns (out float64, lse float64)."""
    q = _u16(q, 3, "q")
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    if k.dtype != np.uint8 or v.dtype != np.uint8 or k.ndim != 4 or k.shape != v.shape:
        raise TypeError("k, v: expected equal-shaped uint8 arrays with 4 dims")
    B, Hq, D = q.shape
    if k.shape[0] != B or k.shape[3] != D:
        raise ValueError("shape mismatch")
    Hkv, S_max = k.shape[1], k.shape[2]
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    rc = _load().fd_oracle_decode_fp8kv(_ptr(q, ctypes.c_uint16), k.ctypes.data_as(u8p), v.ctypes.data_as(u8p),
                                        _ptr(sl, ctypes.c_int32), B, Hq, Hkv, D, S_max, float(scale), float(k_scale),
                                        float(v_scale), int(n_threads), _ptr(out, ctypes.c_double), _ptr(lse, ctypes.c_double))
    if rc != 0:
        raise ValueError("fd_oracle_decode_fp8kv rejected its arguments")
    return out, lse


def decode_fp8kv_paged(q: np.ndarray, k_pages: np.ndarray, v_pages: np.ndarray, block_table: np.ndarray,
                       seq_lens: np.ndarray, k_scale: float = 1.0, v_scale: float = 1.0, scale: float = 0.0):
    """decode_fp8kv over a paged cache (uint8 pools [num_pages,Hkv,page_size,D]), by the same
    row-by-row gather as decode_paged."""
    q = _u16(q, 3, "q")
    kp, vp = np.ascontiguousarray(k_pages), np.ascontiguousarray(v_pages)
    if kp.dtype != np.uint8 or vp.dtype != np.uint8 or kp.ndim != 4 or kp.shape != vp.shape:
        raise TypeError("k_pages, v_pages: expected equal-shaped uint8 arrays with 4 dims")
    num_pages, Hkv, page_size, D = kp.shape
    B = q.shape[0]
    bt = np.asarray(block_table)
    sl = np.asarray(seq_lens, dtype=np.int64)
    S_max = max(1, int(sl.max()) if B else 1)
    k = np.zeros((B, Hkv, S_max, D), dtype=np.uint8)
    v = np.zeros((B, Hkv, S_max, D), dtype=np.uint8)
    for b in range(B):
        for j in range(int(sl[b])):
            page = int(bt[b, j // page_size])
            if not 0 <= page < num_pages:
                raise ValueError(f"block_table[{b}, {j // page_size}] = {page} is not a page")
            k[b, :, j, :] = kp[page, :, j % page_size, :]
            v[b, :, j, :] = vp[page, :, j % page_size, :]
    return decode_fp8kv(q, k, v, sl.astype(np.int32), k_scale=k_scale, v_scale=v_scale, scale=scale)
