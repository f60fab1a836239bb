"""ctypes binding over libfd.so -- argument marshalling only.

Function names and argument order follow include/fd.h.  Tensors are torch
tensors on the GPU (torch supplies device memory and streams, nothing else);
every step of the computation runs in the library's HIP kernels.  If libfd.so
has not been built the import of the library fails loudly: there is no CPU or
PyTorch fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfd.so")

FD_OK, FD_ERR_INVALID_ARG, FD_ERR_UNSUPPORTED, FD_ERR_WORKSPACE, FD_ERR_HIP = 0, -1, -2, -3, -4
FD_OPT_PATH, FD_OPT_XCD_GROUPS, FD_OPT_WGS_PER_CU, FD_OPT_RING_STAGES, FD_OPT_SPIN_LIMIT, FD_OPT_SPLIT_KEYS, FD_OPT_TREE_ROWS = 1, 2, 3, 4, 5, 6, 7
FD_DTYPE_BF16, FD_DTYPE_FP16, FD_DTYPE_FP8_KV = 0, 1, 2
FD_INFO_NUM_CUS, FD_INFO_LAST_GRID, FD_INFO_LAST_PATH, FD_INFO_WAIT_GAVE_UP = 100, 101, 102, 103

EXPORTS = ["fd_workspace_bytes", "fd_create", "fd_destroy", "fd_reset", "fd_decode", "fd_decode_bsp",
           "fd_decode_paged", "fd_decode_paged_bsp", "fd_decode_waits", "fd_decode_static", "fd_autotune", "fd_set_option", "fd_get_option", "fd_debug_poison_workspace", "fd_debug_read_counters",
           "fd_debug_set_trace", "fd_debug_stream_read",
           "fd_last_error", "fd_version"]


class fd_config(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("S_max", ctypes.c_int32), ("max_splits", ctypes.c_int32),
                ("kv_layout", ctypes.c_int32), ("scale", ctypes.c_float), ("dtype", ctypes.c_int32),
                ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float)]


class FdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libfd error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """The loaded library; raises if it was never built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2511_02168_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.fd_workspace_bytes.restype = ctypes.c_size_t
        L.fd_workspace_bytes.argtypes = [ctypes.POINTER(fd_config)]
        L.fd_create.restype = ctypes.c_int
        L.fd_create.argtypes = [ctypes.POINTER(fd_config), ctypes.POINTER(vp)]
        L.fd_destroy.restype = ctypes.c_int
        L.fd_destroy.argtypes = [vp]
        L.fd_reset.restype = ctypes.c_int
        L.fd_reset.argtypes = [vp, vp]
        for fn in (L.fd_decode, L.fd_decode_bsp, L.fd_decode_waits):
            fn.restype = ctypes.c_int
            fn.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.fd_decode_static.restype = ctypes.c_int
        L.fd_decode_static.argtypes = [ctypes.POINTER(fd_config), vp, vp, vp, vp, vp, vp, i32, vp]
        L.fd_set_option.restype = ctypes.c_int
        L.fd_set_option.argtypes = [vp, i32, i32]
        L.fd_get_option.restype = ctypes.c_int
        L.fd_get_option.argtypes = [vp, i32, ctypes.POINTER(i32)]
        L.fd_debug_poison_workspace.restype = ctypes.c_int
        L.fd_debug_poison_workspace.argtypes = [vp, vp]
        L.fd_debug_read_counters.restype = ctypes.c_int
        L.fd_debug_read_counters.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32), i32]
        L.fd_debug_set_trace.restype = ctypes.c_int
        L.fd_debug_set_trace.argtypes = [vp, vp, i32]
        for name in ("fd_decode_paged", "fd_decode_paged_bsp"):
            fn = getattr(L, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, i32, vp]
        L.fd_autotune.restype = ctypes.c_int
        L.fd_autotune.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, i32, ctypes.POINTER(ctypes.c_float)]
        L.fd_debug_stream_read.restype = ctypes.c_int
        L.fd_debug_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        L.fd_last_error.restype = ctypes.c_char_p
        L.fd_last_error.argtypes = []
        L.fd_version.restype = ctypes.c_int
        L.fd_version.argtypes = []
        _lib = L
    return _lib


def fd_last_error() -> str:
    return lib().fd_last_error().decode()


def _check(rc: int) -> None:
    if rc != FD_OK:
        raise FdError(rc, fd_last_error())


def fd_version() -> int:
    return int(lib().fd_version())


def fd_workspace_bytes(cfg: fd_config) -> int:
    return int(lib().fd_workspace_bytes(ctypes.byref(cfg)))


def fd_create(cfg: fd_config) -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    _check(lib().fd_create(ctypes.byref(cfg), ctypes.byref(h)))
    return h


def fd_destroy(h) -> None:
    _check(lib().fd_destroy(h))


def fd_decode_paged(h, q, k_pages, v_pages, block_table, page_size: int, seq_lens, out, lse, n_splits: int,
                    stream: int = 0, bsp: bool = False) -> None:
    """k_pages / v_pages [num_pages, Hkv, page_size, D]; block_table [B, pages_per_seq] int32."""
    fn = lib().fd_decode_paged_bsp if bsp else lib().fd_decode_paged
    _check(fn(h, _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), int(page_size),
              0 if block_table is None else int(block_table.shape[1]), int(k_pages.shape[0]), _ptr(seq_lens),
              _ptr(out), _ptr(lse),
              int(n_splits), ctypes.c_void_p(stream)))


def fd_autotune(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits: int, stream: int = 0, reps: int = 20) -> float:
    """Synchronous: measures the option combinations and keeps the fastest; returns its us per call."""
    best = ctypes.c_float(0.0)
    _check(lib().fd_autotune(h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(out), _ptr(lse),
                             int(n_splits), ctypes.c_void_p(stream), int(reps), ctypes.byref(best)))
    return float(best.value)


def fd_reset(h, stream: int = 0) -> None:
    _check(lib().fd_reset(h, ctypes.c_void_p(stream)))


def _ptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def fd_decode(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits: int, stream: int = 0) -> None:
    _check(lib().fd_decode(h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(out), _ptr(lse),
                           int(n_splits), ctypes.c_void_p(stream)))


def fd_decode_waits(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits: int, stream: int = 0) -> None:
    _check(lib().fd_decode_waits(h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(out), _ptr(lse),
                                 int(n_splits), ctypes.c_void_p(stream)))


FD_STATIC_SCRATCH_BYTES = 32 << 20


def fd_decode_static(cfg: fd_config, q, k_cache, v_cache, seq_lens, out, lse, n_splits: int, stream: int = 0) -> None:
    """fd_decode without a handle, out of the library's static device workspace (allocates nothing)."""
    _check(lib().fd_decode_static(ctypes.byref(cfg), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(out),
                                  _ptr(lse), int(n_splits), ctypes.c_void_p(stream)))


def fd_decode_bsp(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits: int, stream: int = 0) -> None:
    _check(lib().fd_decode_bsp(h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(out), _ptr(lse),
                               int(n_splits), ctypes.c_void_p(stream)))


def fd_set_option(h, key: int, value: int) -> None:
    _check(lib().fd_set_option(h, key, value))


def fd_get_option(h, key: int) -> int:
    v = ctypes.c_int32()
    _check(lib().fd_get_option(h, key, ctypes.byref(v)))
    return int(v.value)


def fd_debug_poison_workspace(h, stream: int = 0) -> None:
    _check(lib().fd_debug_poison_workspace(h, ctypes.c_void_p(stream)))


def fd_debug_read_counters(h, n: int):
    buf = (ctypes.c_uint32 * n)()
    _check(lib().fd_debug_read_counters(h, buf, n))
    return list(buf)


FD_TRACE_EVENTS = 12


def fd_debug_set_trace(h, buf, capacity_workgroups: int) -> None:
    _check(lib().fd_debug_set_trace(h, _ptr(buf), int(capacity_workgroups)))


def fd_debug_stream_read(src, nbytes: int, sink, stream: int = 0) -> None:
    _check(lib().fd_debug_stream_read(_ptr(src), int(nbytes), _ptr(sink), ctypes.c_void_p(stream)))


class FlashDecode:
    """Convenience owner of one handle: shapes fixed at construction."""

    def __init__(self, B: int, Hq: int, Hkv: int, S_max: int, max_splits: int = 256, D: int = 128,
                 scale: float = 0.0, dtype: str = "bf16", k_scale: float = 0.0, v_scale: float = 0.0):
        code = {"bf16": FD_DTYPE_BF16, "fp16": FD_DTYPE_FP16, "fp8kv": FD_DTYPE_FP8_KV}[dtype]
        self.cfg = fd_config(B, Hq, Hkv, D, S_max, max_splits, 0, scale, code, k_scale, v_scale)
        self.h = fd_create(self.cfg)

    def close(self) -> None:
        if self.h is not None:
            fd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def _check_tensors(self, q, k, v, seq_lens, out, lse):
        import torch
        c = self.cfg
        assert q.is_cuda and k.is_cuda and v.is_cuda and seq_lens.is_cuda and out.is_cuda
        want = torch.float16 if c.dtype == FD_DTYPE_FP16 else torch.bfloat16
        want_kv = torch.float8_e4m3fn if c.dtype == FD_DTYPE_FP8_KV else want
        assert q.dtype == want and k.dtype == want_kv and v.dtype == want_kv
        assert seq_lens.dtype == torch.int32 and out.dtype == torch.float32
        assert tuple(q.shape) == (c.B, c.Hq, c.D) and q.is_contiguous()
        assert tuple(k.shape) == (c.B, c.Hkv, c.S_max, c.D) and k.is_contiguous()
        assert tuple(v.shape) == (c.B, c.Hkv, c.S_max, c.D) and v.is_contiguous()
        assert tuple(seq_lens.shape) == (c.B,) and seq_lens.is_contiguous()
        assert tuple(out.shape) == (c.B, c.Hq, c.D) and out.is_contiguous()
        if lse is not None:
            assert lse.is_cuda and lse.dtype == torch.float32 and tuple(lse.shape) == (c.B, c.Hq) and lse.is_contiguous()

    def decode(self, q, k, v, seq_lens, n_splits: int, out=None, lse=None, bsp: bool = False,
               stream: Optional[int] = None, want_lse: bool = True, waits: bool = False):
        import torch
        c = self.cfg
        if out is None:
            out = torch.empty(c.B, c.Hq, c.D, device=q.device, dtype=torch.float32)
        if lse is None and want_lse:
            lse = torch.empty(c.B, c.Hq, device=q.device, dtype=torch.float32)
        self._check_tensors(q, k, v, seq_lens, out, lse)
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        fn = fd_decode_waits if waits else fd_decode_bsp if bsp else fd_decode
        fn(self.h, q, k, v, seq_lens, out, lse, n_splits, stream)
        return out, lse

    def decode_paged(self, q, k_pages, v_pages, block_table, page_size: int, seq_lens, n_splits: int,
                     out=None, lse=None, bsp: bool = False, stream: Optional[int] = None, want_lse: bool = True):
        import torch
        c = self.cfg
        if out is None:
            out = torch.empty(c.B, c.Hq, c.D, device=q.device, dtype=torch.float32)
        if lse is None and want_lse:
            lse = torch.empty(c.B, c.Hq, device=q.device, dtype=torch.float32)
        assert k_pages.is_cuda and v_pages.is_cuda and block_table.is_cuda and q.is_cuda and seq_lens.is_cuda
        want = torch.float16 if c.dtype == FD_DTYPE_FP16 else torch.bfloat16
        want_kv = torch.float8_e4m3fn if c.dtype == FD_DTYPE_FP8_KV else want
        assert k_pages.dtype == want_kv and v_pages.dtype == want_kv and block_table.dtype == torch.int32
        assert k_pages.shape == v_pages.shape and k_pages.is_contiguous() and v_pages.is_contiguous()
        assert tuple(k_pages.shape[1:]) == (c.Hkv, page_size, c.D)
        assert block_table.dim() == 2 and block_table.shape[0] == c.B and block_table.is_contiguous()
        assert tuple(q.shape) == (c.B, c.Hq, c.D) and q.is_contiguous() and q.dtype == want
        assert tuple(seq_lens.shape) == (c.B,) and seq_lens.dtype == torch.int32 and seq_lens.is_contiguous()
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        fd_decode_paged(self.h, q, k_pages, v_pages, block_table, page_size, seq_lens, out, lse, n_splits,
                        stream, bsp=bsp)
        return out, lse
