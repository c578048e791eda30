"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The five sources are compiled host-only (no device code is generated, so this takes seconds) with
-fsanitize=address,undefined and linked with tests/abi_host_check.cpp, which drives every entry point
through its planning and validation paths: workspace sizes and layouts over the paper's shapes and
the edges of the supported range, invalid shapes, NULL and undersized arguments, empty inputs, error
strings, the profiling bookkeeping.  Any report of either sanitizer aborts the program."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2506_18145_amd", "csrc")
OUT = os.path.join(ROOT, "_build", "abi_sanitized")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _tool(name):
    for cand in (os.path.join("/opt/rocm/bin", name), os.path.join("/opt/rocm/llvm/bin", name), shutil.which(name)):
        if cand and os.path.exists(cand):
            return cand
    return None


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, " ".join(cmd) + "\n" + r.stdout[-4000:]
    return r.stdout


def test_host_side_under_asan_and_ubsan():
    hipcc, clang, nm = _tool("hipcc"), _tool("clang++"), _tool("llvm-nm") or shutil.which("nm")
    if not (hipcc and clang and nm):
        pytest.skip("needs hipcc, clang++ and nm")
    from paper_2506_18145_amd.build import SOURCES
    os.makedirs(OUT, exist_ok=True)
    objs = []
    for src in SOURCES:
        obj = os.path.join(OUT, src.replace(".hip", ".o"))
        host_san = [x for flag in SAN for x in ("-Xarch_host", flag)]
        _run([hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-omit-frame-pointer", *host_san,
              "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    driver = os.path.join(OUT, "abi_host_check.o")
    _run([clang, "-O1", "-g", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
          os.path.join(ROOT, "tests", "abi_host_check.cpp"), "-o", driver])
    # a host-only object refers to the device image it would have carried: define those symbols as zeros
    images = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", _run([nm, "-u", *objs]))))
    exe = os.path.join(OUT, "abi_host_check")
    _run([clang, *SAN[:2], driver, *objs, *[f"-Wl,--defsym={s}=0" for s in images], "-L/opt/rocm/lib", "-lamdhip64",
          "-Wl,-rpath,/opt/rocm/lib", "-o", exe])
    env = dict(os.environ)
    # leak checking would report the HIP runtime's own start-up allocations; the link-order check
    # objects to any preloaded library, which is not what this test is about
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "all checks passed" in r.stdout, r.stdout[-4000:]
