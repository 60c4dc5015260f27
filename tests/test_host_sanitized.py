"""The library's host code (planners, segment merging, latency model, and the C ABI's argument
checking and launch splitting against recording stand-ins for the HIP runtime and the kernel
launchers) and the oracle, compiled with AddressSanitizer + UBSan into one CPU program and run on
exact-size buffers. No GPU, no HIP runtime."""
import os
import subprocess

from conftest import ROOT

CSRC = os.path.join(ROOT, "paper_2506_10911_amd", "csrc")
ROCM_INCLUDE = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "include")   # HIP API declarations only


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "host_sanitize_driver"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-I", ROCM_INCLUDE,
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), os.path.join(CSRC, "api.cpp"),
           os.path.join(CSRC, "planner.cpp"), os.path.join(CSRC, "launch_plan.cpp"),
           os.path.join(CSRC, "latency_model.cpp"), os.path.join(ROOT, "oracle", "noloco_oracle.cpp"),
           "-o", str(exe)]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "host sanitize driver: ok" in run.stdout
