"""The CPU oracle and the library's host logic under AddressSanitizer and UndefinedBehaviorSanitizer.

tests/host_sanitize.cpp is linked with oracle/mgg_oracle.c and the library's host translation units
(partition build, entry points, search), all compiled with -fsanitize=address,undefined on the host side
(`-Xarch_host`, so the device code is left alone); the kernels' translation units are linked as they are.
The executable builds partitions host-only, compares every integer structure with the oracle's and runs the
oracle's arithmetic; any sanitizer report makes it exit non-zero.  No GPU is needed.
"""
import os
import shutil
import subprocess

import pytest

from paper_2209_06800_amd import build as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]
HOST_SOURCES = ["partition.cpp", "api.cpp", "tuner.cpp"]


def _xarch_host(flags):
    out = []
    for f in flags:
        out += ["-Xarch_host", f]
    return out


def test_oracle_and_host_library_run_clean_under_asan_and_ubsan(tmp_path):
    clang = os.path.join(os.path.dirname(os.path.realpath(b.HIPCC)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = shutil.which("clang") or clang
    if not os.path.exists(b.HIPCC) or not os.path.exists(clang):
        pytest.skip("hipcc / clang not found")
    out = str(tmp_path)
    objs = []
    # the library's host translation units, instrumented on the host side only
    for src in HOST_SOURCES:
        obj = os.path.join(out, src + ".o")
        subprocess.check_call([b.HIPCC, *b.FLAGS, *_xarch_host(SAN), "-c", os.path.join(b.CSRC, src), "-o", obj], stderr=subprocess.DEVNULL)
        objs.append(obj)
    # the kernels' translation units as the library build leaves them (built now if they are not there)
    os.makedirs(b.OBJ, exist_ok=True)
    for src in b.SOURCES:
        if src in HOST_SOURCES:
            continue
        obj = os.path.join(b.OBJ, os.path.splitext(src)[0] + ".o")
        if not os.path.exists(obj):
            b._compile(src)
        objs.append(obj)
    # the oracle (plain C) and the driver, instrumented
    ora = os.path.join(out, "mgg_oracle.o")
    subprocess.check_call([clang, "-O1", "-std=c99", *SAN, "-c", os.path.join(ROOT, "oracle", "mgg_oracle.c"), "-o", ora])
    objs.append(ora)
    drv = os.path.join(out, "host_sanitize.o")
    subprocess.check_call([clang + "++", "-O1", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
                           os.path.join(ROOT, "tests", "host_sanitize.cpp"), "-o", drv])
    exe = os.path.join(out, "host_sanitize")
    subprocess.check_call([b.HIPCC, "--offload-arch=gfx950", *_xarch_host(SAN[:2]), drv, *objs, "-lm", "-o", exe], stderr=subprocess.DEVNULL)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-6000:]
    assert "all checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-6000:]
