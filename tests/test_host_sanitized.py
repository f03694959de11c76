"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer: isa_api.hip (argument checks,
count derivation, workspace carve-up, launch sequencing) is compiled with the sanitizers on its host pass only, linked
with the other objects of the regular build and a C++ driver that walks every host-only path of the C ABI.  Runs
without a GPU; no kernel is launched."""
import os
import subprocess

import pytest

from paper_2605_04569_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
       "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = B._hipcc()
    objdir = os.path.join(B.HERE, "_build")
    others = [os.path.join(objdir, s.replace(".hip", ".o")) for s in B.SOURCES if s != "isa_api.hip"]
    if not all(os.path.exists(o) for o in others):
        B.build()
    api_o, drv_o, exe = (str(tmp_path / n) for n in ("isa_api_san.o", "host_sanitize.o", "host_sanitize"))
    for src, obj in ((os.path.join(B.CSRC, "isa_api.hip"), api_o), (os.path.join(ROOT, "tests", "host", "host_sanitize.cpp"), drv_o)):
        r = subprocess.run([hipcc, *B.FLAGS, *SAN, "-x", "hip", "-c", src, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-4000:]
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        api_o, drv_o, *others, "-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "host checks ok" in r.stdout, (r.stdout[-3000:], r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
