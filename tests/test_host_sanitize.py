"""Host-side hardening on the CPU: the library's host code (validation, launch planner,
scheduling helpers; csrc/medha.hip with its headers) and the C oracle are compiled with
-fsanitize=address,undefined and driven by tests/host_sanitize/driver.cpp -- planner fuzz with
batches up to 10^4 sequences and prefixes up to 2^31-1, every entry point's refusal paths, the
policy helpers against their own invariants, tiny and empty cases through every oracle entry.
No kernel runs (the device code is compiled without sanitizers and never launched)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/lib/llvm/bin/clang"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)),
                    reason="needs the ROCm compilers")
def test_host_code_and_oracle_under_address_and_ub_sanitizers(tmp_path):
    inc = ["-I", os.path.join(ROOT, "include"), "-I",
           os.path.join(ROOT, "paper_2409_17264_amd", "csrc")]
    lib_o, ora_o, drv_o = (str(tmp_path / n) for n in ("medha.o", "oracle.o", "driver.o"))
    exe = str(tmp_path / "host_san")
    host_san = []
    for f in SAN:
        host_san += ["-Xarch_host", f]
    steps = [
        [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san, *inc, "-c",
         os.path.join(ROOT, "paper_2409_17264_amd", "csrc", "medha.hip"), "-o", lib_o],
        [CLANG, "-O1", "-g", "-std=c99", *SAN, "-c", os.path.join(ROOT, "oracle", "medha_oracle.c"),
         "-o", ora_o],
        [CLANG + "++", "-O1", "-g", "-std=c++17", *SAN, *inc, "-c",
         os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"), "-o", drv_o],
        [HIPCC, "-fsanitize=address,undefined", lib_o, ora_o, drv_o, "-o", exe, "-lm"],
    ]
    for cmd in steps:
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, " ".join(cmd) + "\n" + res.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1", HIP_VISIBLE_DEVICES="")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-6000:]
    for part in ("planner fuzz ok", "validation paths ok", "policy paths ok", "oracle paths ok"):
        assert part in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr
    shutil.rmtree(tmp_path, ignore_errors=True)
