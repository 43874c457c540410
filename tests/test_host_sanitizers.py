"""The host-only code of the library (csrc/psx_host.cpp, csrc/psx_cpu.cpp) under sanitizers, on the CPU:
AddressSanitizer + UndefinedBehaviorSanitizer, then ThreadSanitizer for the worker pool.  The driver
(tests/host_sanitizer_driver.cpp) compares layout and host-core Adam with the oracle on the way."""
import os
import subprocess

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2108_05818_amd", "csrc")
HIP_INCLUDE = "/opt/rocm/include"          # psx_internal.h includes the HIP runtime header for its types only


def build(tmp_path, name, sanitize):
    obj = tmp_path / "oracle.o"
    # the oracle keeps its own flags (no contraction, no fast-math) and is not instrumented
    subprocess.run(["gcc", "-c", *[f for f in oracle.CFLAGS if f not in ("-shared",)], os.path.join(ROOT, "oracle", "psx_oracle.c"),
                    "-o", str(obj)], check=True)
    exe = tmp_path / name
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", f"-fsanitize={sanitize}", "-fno-sanitize-recover=all",
           "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I", HIP_INCLUDE, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"), os.path.join(CSRC, "psx_host.cpp"),
           os.path.join(CSRC, "psx_cpu.cpp"), str(obj), "-o", str(exe), "-lpthread", "-lm"]
    subprocess.run(cmd, check=True)
    return exe


def run(exe, iters, env_extra):
    env = dict(os.environ, **env_extra)
    r = subprocess.run([str(exe), str(iters)], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, f"rc {r.returncode}\n{r.stdout[-2000:]}\n{r.stderr[-4000:]}"
    assert "host sanitizer driver ok" in r.stdout
    assert "ERROR" not in r.stderr and "WARNING: ThreadSanitizer" not in r.stderr, r.stderr[-4000:]


@pytest.mark.skipif(not os.path.exists(os.path.join(HIP_INCLUDE, "hip", "hip_runtime.h")), reason="HIP headers not installed")
def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = build(tmp_path, "drv_asan", "address,undefined")
    run(exe, 20000, {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", "UBSAN_OPTIONS": "print_stacktrace=1"})


@pytest.mark.skipif(not os.path.exists(os.path.join(HIP_INCLUDE, "hip", "hip_runtime.h")), reason="HIP headers not installed")
def test_worker_pool_under_thread_sanitizer(tmp_path):
    exe = build(tmp_path, "drv_tsan", "thread")
    run(exe, 2000, {"TSAN_OPTIONS": "halt_on_error=1:second_deadlock_stack=1"})
