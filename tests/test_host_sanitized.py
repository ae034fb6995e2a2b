"""The plan code of the library (csrc/mdbf_api.hip: plan layout, work-item tables, balancing, last-round pieces,
workspace layouts) compiled with AddressSanitizer and UndefinedBehaviorSanitizer on the host side, linked into
a standalone driver (tests/host_sanitized_driver.cpp) with the other translation units as the regular build left
them, and run on the CPU.  No GPU, no Python in the sanitized process."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BUILD = os.path.join(ROOT, "_build")
CSRC = os.path.join(ROOT, "paper_2512_24545_amd", "csrc")
OTHERS = ["mdbf_pack", "mdbf_precise", "mdbf_stage_mfma", "mdbf_stage_mx", "mdbf_stage_gemm", "mdbf_stage_generic", "mdbf_msvid"]


def test_plan_code_under_host_sanitizers(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    objs = [os.path.join(BUILD, n + ".o") for n in OTHERS]
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no ROCm toolchain")
    if not all(os.path.exists(o) for o in objs):
        pytest.skip("the regular build's objects are not there (run __graft_entry__.build() first)")
    api = str(tmp_path / "api_san.o")
    drv = str(tmp_path / "drv.o")
    exe = str(tmp_path / "plan_driver")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    subprocess.run([hipcc, "-O1", "-g", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature",
                    "-Xclang", "-packed-fp32-ops", "-w", *san, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
                    os.path.join(CSRC, "mdbf_api.hip"), "-o", api], check=True, capture_output=True)
    subprocess.run([clang, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-I",
                    os.path.join(ROOT, "include"), "-c", os.path.join(ROOT, "tests", "host_sanitized_driver.cpp"), "-o", drv],
                   check=True, capture_output=True)
    subprocess.run([clang, "-fsanitize=address,undefined", drv, api, *objs, "-L/opt/rocm/lib", "-lamdhip64",
                    "-Wl,-rpath,/opt/rocm/lib", "-o", exe], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    report = r.stdout[-3000:] + r.stderr[-6000:]
    assert r.returncode == 0, report
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, report
    assert r.stdout.strip().endswith("ok"), report
