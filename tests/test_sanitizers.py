"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU-side code: the fp64 oracle, and the
HOST side of the HIP library (validation, workspace sizing, kernel planning).  GPU code is not
sanitised (not available for gfx950 here); the sanitised library copy is built beside the normal
one, only when its sources are newer, and no test ever launches a kernel through it."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
ENV = {**os.environ, "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1",
       "OMP_NUM_THREADS": "4"}
# the sanitizer runtime wants to be the first library of the process: nothing may be preloaded before it
ENV.pop("LD_PRELOAD", None)


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", *SAN, "-std=c11", "-Wall", "-o", exe,
                    os.path.join(ROOT, "oracle", "oracle.c"), os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"],
                   check=True)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "geometries ok" in r.stdout


def _build_sanitized_host_library():
    from paper_1810_01993_amd import build
    out = os.path.join(build.HERE, "_build_san")
    os.makedirs(out, exist_ok=True)
    lib = os.path.join(out, "libdlconv_hostsan.so")
    srcs = [os.path.join(build.CSRC, s) for s in build.SOURCES]
    deps = srcs + [os.path.join(build.CSRC, h) for h in os.listdir(build.CSRC) if h.endswith(".h")] + \
        [os.path.join(ROOT, "include", "dlconv.h")]
    if os.path.exists(lib) and os.path.getmtime(lib) >= max(os.path.getmtime(d) for d in deps):
        return lib
    host_san = []
    for f in SAN:
        host_san += ["-Xarch_host", f]

    def cc(src):
        obj = os.path.join(out, os.path.basename(src).replace(".hip", ".o"))
        # -O1 for the device pass too: this copy is never launched, only its host code runs
        flags = [f for f in build.FLAGS if f != "-O3"] + ["-O1", "-g"]
        subprocess.run(["hipcc", *flags, *host_san, "-c", src, "-o", obj], check=True, capture_output=True)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(cc, srcs))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *SAN, "-o", lib, *objs], check=True,
                   capture_output=True)
    return lib


def test_library_host_path_under_asan_ubsan(tmp_path):
    lib = _build_sanitized_host_library()
    exe = str(tmp_path / "cabi_san")
    # the same compiler family as the library's host pass: the two sanitizer runtimes do not mix
    subprocess.run(["amdclang", "-O1", "-g", *SAN, "-std=c11", "-Wall", "-o", exe, os.path.join(ROOT, "tests", "cabi_sanitize_driver.c"),
                    lib, f"-Wl,-rpath,{os.path.dirname(lib)}"], check=True)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "0 wrong status codes" in r.stdout
