"""AddressSanitizer + UndefinedBehaviorSanitizer pass over the host side of the C ABI (CPU only, no kernel runs).

csrc/thrift_api.hip is compiled once more with the sanitizers on its HOST code only, linked with the kernel objects of
the regular build and with tests/sanitize_abi_driver.cpp, which calls every entry point with arguments that must be
refused before a launch (invalid enum codes, sizes whose products overflow, missing buffers) and sweeps the host
helpers.  The sanitizers abort on the first finding."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_23081_amd", "csrc")
from paper_2605_23081_amd.build import SOURCES

# every object of the library except the C ABI itself, which this test compiles with the sanitizers on its host side
KERNEL_OBJECTS = [src.replace(".hip", ".o") for src in SOURCES if src != "thrift_api.hip"]
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"


def test_abi_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    if shutil.which("hipcc") is None or not os.path.exists(CLANGXX):
        pytest.skip("no ROCm toolchain")
    if not all(os.path.exists(os.path.join(CSRC, o)) for o in KERNEL_OBJECTS):
        from paper_2605_23081_amd import build
        build.build()
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    san_host = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    api = str(tmp_path / "api_san.o")
    drv = str(tmp_path / "driver.o")
    exe = str(tmp_path / "abi_san")
    steps = [
        ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         *san_host, *inc, "-c", os.path.join(CSRC, "thrift_api.hip"), "-o", api],
        [CLANGXX, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", *inc,
         "-c", os.path.join(ROOT, "tests", "sanitize_abi_driver.cpp"), "-o", drv],
        ["hipcc", "--offload-arch=gfx950", drv, api, *[os.path.join(CSRC, o) for o in KERNEL_OBJECTS], "-o", exe, "-fno-gpu-sanitize", "-fsanitize=address,undefined"],
    ]
    for cmd in steps:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0 and ("asan" in r.stderr.lower() or "ubsan" in r.stderr.lower()) and "cannot find" in r.stderr.lower():
            pytest.skip("no sanitizer runtime for this toolchain")
        assert r.returncode == 0, r.stderr[-3000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "abi sanitizer pass: ok" in run.stdout
