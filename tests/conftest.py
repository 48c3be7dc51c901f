import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def host_hooks():
    """The host-only test hooks (tests/host_hooks.cpp: replay of the kernels' index code, schedule
    checks), compiled with g++ into tests/_build/ on first use.  Test infrastructure; the product
    library exports none of it."""
    import ctypes
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    src = os.path.join(here, "host_hooks.cpp")
    out_dir = os.path.join(here, "_build")
    lib = os.path.join(out_dir, "libhosthooks.so")
    csrc = os.path.join(ROOT, "paper_2505_13060_amd", "csrc")
    deps = [src] + [os.path.join(csrc, h) for h in ("table.h", "walk.h", "internal.h")] + \
           [os.path.join(ROOT, "include", "ampsens.h")]
    if not os.path.exists(lib) or any(os.path.getmtime(d) > os.path.getmtime(lib) for d in deps):
        os.makedirs(out_dir, exist_ok=True)
        subprocess.run(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-D__HIP_PLATFORM_AMD__",
                        "-I/opt/rocm/include", src, "-o", lib], check=True)
    L = ctypes.CDLL(lib)
    i64, u64, vp = ctypes.c_int64, ctypes.c_uint64, ctypes.c_void_p
    L.hooks_replay_unit.restype = i64
    L.hooks_replay_unit.argtypes = [u64, u64, vp, i64, vp, i64, ctypes.POINTER(u64)]
    L.hooks_replay_unit_rows.restype = i64
    L.hooks_replay_unit_rows.argtypes = [u64, u64, vp, i64, i64, vp, i64, ctypes.POINTER(u64)]
    L.hooks_check_linear_schedule.restype = i64
    L.hooks_check_linear_schedule.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.POINTER(u64), ctypes.POINTER(u64)]
    return L
