"""The library's host code (argument checks, layout and size functions: csrc/taq_api.hip and the headers it includes)
built with AddressSanitizer and UBSan and driven through the C ABI by tests/host/abi_sanitize.cpp. No GPU: every call is
host-only or is rejected before a launch. The device code and the other translation units are the normal build's."""
import os
import shutil
import subprocess

import pytest

from paper_2603_22943_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_under_asan_and_ubsan(tmp_path):
    hipcc = B.hipcc_path()
    objdir = os.path.join(B.HERE, "_build")
    others = [os.path.join(objdir, s.replace(".hip", ".o")) for s in B.SOURCES if s != "taq_api.hip"]
    if not all(os.path.exists(o) for o in others):
        B.build_lib(verbose=False)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
           "-Xarch_host", "-fno-omit-frame-pointer"]
    common = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-ffp-contract=off",
              "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-honor-nans", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-I", os.path.join(ROOT, "include")]
    api_o = str(tmp_path / "taq_api_san.o")
    drv_o = str(tmp_path / "abi_sanitize.o")
    exe = str(tmp_path / "abi_sanitize")
    for cmd in ([hipcc] + common + san + ["-c", os.path.join(B.CSRC, "taq_api.hip"), "-o", api_o],
                [hipcc] + common + san + ["-c", os.path.join(ROOT, "tests", "host", "abi_sanitize.cpp"), "-o", drv_o],
                [hipcc, "--offload-arch=gfx950"] + san + [drv_o, api_o] + others + ["-o", exe]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
    # (verify_asan_link_order=0: the environment may preload a library of its own ahead of the sanitizer runtime)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and "abi_sanitize: ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
