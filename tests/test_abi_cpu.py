"""CPU-only checks of the C ABI: the built library loads, exports every symbol
include/fd.h declares, and rejects bad arguments on the host before any device
work (no compute calls are made here)."""
import ctypes
import os
import re

import pytest

from paper_2511_02168_amd import binding as fd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fd_[a-z_]+)\s*\(", text)))


def test_library_is_built_and_loads():
    assert os.path.exists(fd.LIB_PATH), "run `python -m paper_2511_02168_amd.build` first"
    assert fd.fd_version() == 150


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert "fd_decode" in names and "fd_decode_bsp" in names and len(names) >= 12
    raw = ctypes.CDLL(fd.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in fd.h but not exported"
    assert sorted(fd.EXPORTS) == names, "binding's export list and fd.h disagree"


def good_cfg(**kw):
    base = dict(B=2, Hq=8, Hkv=2, D=128, S_max=4096, max_splits=16, kv_layout=0, scale=0.0, dtype=0, k_scale=0.0, v_scale=0.0)
    base.update(kw)
    return fd.fd_config(*[base[k] for k in ("B", "Hq", "Hkv", "D", "S_max", "max_splits", "kv_layout", "scale", "dtype", "k_scale", "v_scale")])


def test_workspace_bytes_formula():
    cfg = good_cfg()
    tiles, G, n = 4, 4, 16
    groups = 1                                                        # ceil(16 splits / 16 partials per first-level group)
    expect = (tiles * n * G * 128 * 4 + tiles * n * 128                # partials, one 128-byte line of LSEs per slot
              + tiles * groups * G * 128 * 4 + tiles * groups * 128    # second-level partials and their LSE lines
              + 256 + tiles * 64 * 4 + 256 + 256)                      # tile counters, 64 group counters per tile, direct marks, status word
    assert fd.fd_workspace_bytes(cfg) == expect
    assert fd.fd_workspace_bytes(good_cfg(D=64)) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), fd.FD_ERR_INVALID_ARG),
    (dict(Hq=7), fd.FD_ERR_INVALID_ARG),
    (dict(S_max=-5), fd.FD_ERR_INVALID_ARG),
    (dict(max_splits=0), fd.FD_ERR_INVALID_ARG),
    (dict(max_splits=100000), fd.FD_ERR_INVALID_ARG),
    (dict(scale=-1.0), fd.FD_ERR_INVALID_ARG),
    (dict(scale=float("nan")), fd.FD_ERR_INVALID_ARG),
    (dict(D=64), fd.FD_ERR_UNSUPPORTED),
    (dict(kv_layout=1), fd.FD_ERR_UNSUPPORTED),
    (dict(B=1 << 20, Hq=16, Hkv=8, max_splits=1024), fd.FD_ERR_UNSUPPORTED),
    (dict(dtype=3), fd.FD_ERR_UNSUPPORTED),
    (dict(dtype=2, k_scale=-1.0), fd.FD_ERR_INVALID_ARG),
    (dict(dtype=-1), fd.FD_ERR_UNSUPPORTED),
    (dict(Hq=68, Hkv=2), fd.FD_ERR_UNSUPPORTED),
])
def test_create_rejects_bad_config_before_touching_the_device(kw, code):
    with pytest.raises(fd.FdError) as e:
        fd.fd_create(good_cfg(**kw))
    assert e.value.code == code
    assert fd.fd_last_error() != ""


def test_null_handles_and_pointers():
    L = fd.lib()
    assert L.fd_destroy(None) == fd.FD_ERR_INVALID_ARG
    assert L.fd_reset(None, None) == fd.FD_ERR_INVALID_ARG
    assert L.fd_decode(None, None, None, None, None, None, None, 1, None) == fd.FD_ERR_INVALID_ARG
    assert L.fd_decode_bsp(None, None, None, None, None, None, None, 1, None) == fd.FD_ERR_INVALID_ARG
    assert L.fd_set_option(None, 1, 0) == fd.FD_ERR_INVALID_ARG
    assert L.fd_create(None, None) == fd.FD_ERR_INVALID_ARG
    assert "handle" in fd.fd_last_error() or "NULL" in fd.fd_last_error()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2511_02168_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "fd_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2511_02168_amd" not in text and "libfd.so" not in text, f


def test_host_computed_division_constants(tmp_path):
    """csrc/fd_fastdiv.hpp (the multiply-high division of the kernels' work-list arithmetic), compiled for the
    host and checked against the machine's own division: exhaustively for small operands, on boundary numerators
    (multiples of the divisor and their neighbours, the top of the 31-bit range) for 200 000 seeded divisors."""
    import subprocess
    exe = tmp_path / "fastdiv_check"
    src = os.path.join(ROOT, "tests", "fastdiv_check.cpp")
    subprocess.run(["g++", "-O2", "-o", str(exe), src], check=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True)
    assert res.returncode == 0 and res.stdout.startswith("OK"), res.stdout[-500:]


def test_host_half_under_address_and_undefined_behaviour_sanitizers():
    """The host half of libfd.so built with ASan + UBSan (device code untouched) and driven by
    tests/abi_host_check.c through every refusal path of the ABI, from two threads.  No kernel is launched.
    The sanitized library is cached in the temp directory under a hash of the sources (the device code takes
    about a minute to compile)."""
    import hashlib
    import subprocess
    import tempfile
    csrc = os.path.join(ROOT, "paper_2511_02168_amd", "csrc")
    files = sorted(os.path.join(csrc, f) for f in os.listdir(csrc)) + [os.path.join(ROOT, "include", "fd.h")]
    digest = hashlib.sha256(b"".join(open(f, "rb").read() for f in files)).hexdigest()[:16]
    work = os.path.join(tempfile.gettempdir(), f"fd_host_san_{digest}")
    os.makedirs(work, exist_ok=True)
    lib = os.path.join(work, "libfd_host_san.so")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    if not os.path.exists(lib):
        cmd = ["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O2", "-std=c++17", "-fPIC", "-shared", *san,
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
               "-Wno-inline-asm", "-o", lib + ".tmp", os.path.join(csrc, "fd_lib.hip")]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
        os.replace(lib + ".tmp", lib)
    exe = os.path.join(work, "abi_host_check")
    cmd = ["/opt/rocm/lib/llvm/bin/clang", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(ROOT, "tests", "abi_host_check.c"),
           "-L", work, "-lfd_host_san", f"-Wl,-rpath,{work}", "-lpthread"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0 and res.stdout.startswith("OK"), (res.stdout + res.stderr)[-3000:]
