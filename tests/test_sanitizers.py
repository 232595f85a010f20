"""Sanitizer passes over the host code (CPU only).

1. The oracle, built with AddressSanitizer + UndefinedBehaviorSanitizer, runs its brute-force, fixture and
   closed-form pins again: an out-of-bounds read or an overflow in the checker would otherwise go unnoticed
   as long as the answers happen to match.
2. The host side of libdct (argument checks, workspace sizing: everything that runs before a launch), built
   host-only with the same sanitizers, is driven through its error paths.  No kernel is launched.

Each pass runs in a child process with the sanitizer runtime preloaded (the interpreter is not instrumented).
"""
import ctypes
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ASAN_ENV = {"ASAN_OPTIONS": "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=86",
            "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1:exitcode=87"}


def _runtime(cmd):
    try:
        path = subprocess.run(cmd, capture_output=True, text=True, check=True).stdout.strip()
    except (OSError, subprocess.CalledProcessError):
        return None
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _run(preload, extra_env, args, timeout=600):
    env = dict(os.environ, **ASAN_ENV, **extra_env)
    env["LD_PRELOAD"] = preload + (" " + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    r = subprocess.run([sys.executable, *args], cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    return out


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    import oracle
    libasan = _runtime(["gcc", "-print-file-name=libasan.so"])
    if libasan is None:
        pytest.skip("gcc's libasan is not installed")
    lib = oracle.build_sanitized(str(tmp_path / "libdct_oracle_san.so"))
    pins = ("rank_counting or golden or closed_form or capacity_prefix or invalid_arguments or alternating_sign "
            "or k_equals_n or row_stride or hand_worked or rounding or eventually_delivered or idx16 or packbits")
    out = _run(libasan, {"DCT_ORACLE_LIB": lib},
               ["-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider", "-k", pins])
    assert " passed" in out and "failed" not in out, out[-2000:]


HOST_DRIVER = r"""
import ctypes, sys
ctypes.CDLL(sys.argv[2], mode=ctypes.RTLD_GLOBAL)  # stand-ins for the device code objects
lib = ctypes.CDLL(sys.argv[1])
vp, u64, u32, i32, sz = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_size_t
def fn(name, res, *args):
    f = getattr(lib, name); f.restype = res; f.argtypes = list(args); return f
P = 0x7000000000  # a device address as far as the host code is concerned: never dereferenced on the host
INVALID, WORKSPACE = 1, 2
ws_sel = fn("dct_select_threshold_workspace_bytes", sz, i32, u64)
ws_cmp = fn("dct_threshold_compact_workspace_bytes", sz, i32, u64)
assert ws_sel(0, 0) == 0 and ws_sel(7, 100) == 0 and ws_sel(0, 1 << 31) == 0 and ws_sel(0, 1 << 20) > 0
assert ws_sel(1, (1 << 31) - 1) > ws_sel(0, 1 << 22) > 0
assert ws_cmp(0, 0) == 0 and 0 < ws_cmp(1, (1 << 31) - 1) < (1 << 20)
sel = fn("dct_select_threshold", i32, vp, i32, u64, u64, vp, vp, sz, vp)
for args, want in [((None, 0, 10, 1, P, P, 1 << 20, None), INVALID), ((P, 0, 0, 1, P, P, 1 << 20, None), INVALID),
                   ((P, 0, 10, 0, P, P, 1 << 20, None), INVALID), ((P, 0, 10, 11, P, P, 1 << 20, None), INVALID),
                   ((P, 5, 10, 1, P, P, 1 << 20, None), INVALID), ((P + 2, 0, 10, 1, P, P, 1 << 20, None), INVALID),
                   ((P, 0, 10, 1, P + 4, P, 1 << 20, None), INVALID), ((P, 0, 1 << 31, 1, P, P, 1 << 40, None), INVALID),
                   ((P, 0, 10, 1, P, None, 1 << 20, None), WORKSPACE), ((P, 0, 10, 1, P, P + 8, 1 << 20, None), WORKSPACE),
                   ((P, 0, 1 << 24, 1, P, P, 1024, None), WORKSPACE)]:
    assert sel(*args) == want, (args, sel(*args))
efs = fn("dct_ef_select_threshold", i32, vp, vp, i32, u64, u64, vp, vp, sz, vp)
assert efs(P, None, 0, 10, 1, P, P, 1 << 20, None) == INVALID and efs(P, P + 4, 0, 10, 1, P, P, 1 << 20, None) == INVALID
assert efs(P, P + 64, 1, 10, 1, P, P, 1 << 20, None) == INVALID
cmp_ = fn("dct_threshold_compact", i32, vp, i32, u64, vp, i32, vp, vp, u64, vp, vp, sz, vp)
for args, want in [((None, 0, 10, P, 0, P, P, 10, P, P, 1 << 20, None), INVALID), ((P, 0, 10, None, 0, P, P, 10, P, P, 1 << 20, None), INVALID),
                   ((P, 0, 10, P, 2, P, P, 10, P, P, 1 << 20, None), INVALID), ((P, 0, 10, P, 0, None, P, 10, P, P, 1 << 20, None), INVALID),
                   ((P, 0, 10, P + 8, 0, P, P, 10, P, P, 1 << 20, None), INVALID), ((P, 0, 10, P, 0, P, P, 10, P + 4, P, 1 << 20, None), INVALID),
                   ((P, 0, 10, P, 0, P, P, 10, P, None, 1 << 20, None), WORKSPACE), ((P, 0, 10, P, 0, P, P, 10, P, P, 16, None), WORKSPACE)]:
    assert cmp_(*args) == want, (args, cmp_(*args))
wsi = fn("dct_threshold_compact_workspace_init", i32, vp, sz, vp)
assert wsi(None, 1 << 20, None) == WORKSPACE and wsi(P, 8, None) == WORKSPACE and wsi(P + 1, 1 << 20, None) == WORKSPACE
efc = fn("dct_ef_threshold_compact", i32, vp, vp, vp, i32, u64, vp, i32, vp, vp, u64, vp, vp, sz, vp)
big = 1 << 20
for args in [(P, None, P + big, 0, 10, P, 0, P, P, 10, P, P, big, None), (P, P + big, None, 0, 10, P, 0, P, P, 10, P, P, big, None),
             (P, P + big, P + 2 * big, 1, 10, P, 0, P, P, 10, P, P, big, None),      # bf16: no error feedback
             (P, P + big, P + 16, 0, 10, P, 0, P, P, 10, P, P, big, None),           # g overlaps e_out
             (P, P + big, P + big + 16, 0, 10, P, 0, P, P, 10, P, P, big, None),     # e_in overlaps e_out without being it
             (P, P + big + 4, P + 2 * big, 0, 10, P, 0, P, P, 10, P, P, big, None)]: # different offsets within 16 bytes
    assert efc(*args) == INVALID, args
static = fn("dct_threshold_compact_static", i32, vp, i32, u64, vp, i32, vp, vp, u64, vp, vp)
assert static(P, 0, 0, P, 0, P, P, 10, P, None) == INVALID and static(P, 0, 1 << 31, P, 0, P, P, 10, P, None) == INVALID
fwd = fn("dct_rowtopk_fwd", i32, vp, i32, u32, u32, u64, u32, vp, vp, vp, vp)
for args in [(None, 0, 4, 8, 8, 2, P, P, None, None), (P, 0, 0, 8, 8, 2, P, P, None, None), (P, 0, 4, 8, 7, 2, P, P, None, None),
             (P, 0, 4, 8, 8, 0, P, P, None, None), (P, 0, 4, 8, 8, 9, P, P, None, None), (P, 3, 4, 8, 8, 2, P, P, None, None),
             (P, 0, 4, 8, 8, 2, None, P, None, None), (P + 2, 0, 4, 8, 8, 2, P, P, None, None)]:
    assert fwd(*args) == INVALID, args
bwd = fn("dct_rowtopk_bwd", i32, vp, i32, u32, u32, u64, u32, vp, vp, vp)
assert bwd(None, 0, 4, 8, 8, 2, P, P, None) == INVALID and bwd(P, 0, 4, 8, 8, 9, P, P, None) == INVALID
i16 = fn("dct_rowtopk_fwd_idx16", i32, vp, i32, u32, u32, u64, u32, vp, vp, vp, vp)
assert i16(P, 1, 4, 65537, 65537, 2, P, P, None, None) == INVALID
sc = fn("dct_scatter", i32, vp, vp, vp, u64, i32, vp, u64, i32, vp)
assert sc(P, P, None, 10, 0, None, 100, 0, None) == INVALID and sc(P, P, None, 10, 1, P, 100, 1, None) == INVALID
assert sc(P, P, None, 10, 0, P, 0, 0, None) == INVALID and sc(P, P, None, 10, 0, P, 100, 5, None) == INVALID
class Seg(ctypes.Structure):
    _fields_ = [(n, u64) for n in ("offset", "n", "k", "out_offset", "capacity")]
bws = fn("dct_batched_workspace_bytes", sz, i32, vp, u32)
segs = (Seg * 3)(Seg(0, 1000, 10, 0, 20), Seg(1000, 64, 1, 20, 2), Seg(2000, 1 << 20, 100, 22, 200))
assert bws(0, ctypes.cast(segs, vp), 3) > 0 and bws(0, ctypes.cast(segs, vp), 0) == 0 and bws(0, None, 3) == 0
bad = (Seg * 1)(Seg(0, 10, 11, 0, 20))
bsel = fn("dct_select_threshold_batched", i32, vp, i32, vp, u32, vp, vp, sz, vp)
assert bsel(P, 0, ctypes.cast(bad, vp), 1, P, P, 1 << 24, None) == INVALID
assert bsel(P, 0, ctypes.cast(segs, vp), 3, P, P, 64, None) == WORKSPACE
st = fn("dct_status_string", ctypes.c_char_p, i32)
assert st(0) == b"DCT_OK" and b"unknown" in st(99)
fn("dct_set_wait_limit", None, u32)(5)
fn("dct_set_wait_limit", None, u32)(0)
print("host checks ok")
"""


def test_libdct_host_side_under_asan_and_ubsan(tmp_path):
    clang = "/opt/rocm/lib/llvm/bin/clang"
    rt = _runtime([clang, "-print-file-name=libclang_rt.asan-x86_64.so"]) if os.path.exists(clang) else None
    if rt is None:
        pytest.skip("the ROCm clang AddressSanitizer runtime is not installed")
    from paper_2010_08899_amd import build
    lib = str(tmp_path / "libdct_hostsan.so")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    # host pass only: the kernels are stubs, which is all the argument checks need
    cmd = [hipcc, "--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", "-shared", "-fPIC",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libsan",
           "-I", os.path.join(ROOT, "include"), "-I", build.CSRC, "-o", lib, *build.sources()]
    subprocess.run(cmd, check=True, capture_output=True)
    # The host pass refers to the device code objects by symbol (__hip_fatbin_<hash>); there are none in a
    # host-only build.  Empty stand-ins satisfy the loader; they are never parsed, because the HIP runtime only
    # looks at a code object when a kernel of it is first launched.
    undefined = subprocess.run(["nm", "-u", lib], capture_output=True, text=True, check=True).stdout.split()
    fatbins = sorted({u for u in undefined if u.startswith("__hip_fatbin_")})
    stub_c = tmp_path / "fatbin_stubs.c"
    stub_c.write_text("".join(f"const char {name}[64] __attribute__((aligned(4096))) = {{0}};\n" for name in fatbins))
    stub = str(tmp_path / "libfatbin_stubs.so")
    subprocess.run(["gcc", "-shared", "-fPIC", "-o", stub, str(stub_c)], check=True, capture_output=True)
    driver = tmp_path / "host_driver.py"
    driver.write_text(HOST_DRIVER)
    out = _run(rt, {}, [str(driver), lib, stub])
    assert "host checks ok" in out
