"""The host side of libmpic (planner, argument checks, plan accessors, cache library) under
AddressSanitizer and UBSan: g++ build of plan.cpp + api.hip (as plain C++) with the kernel
launchers stubbed, run on random layouts.  No GPU is touched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_01960_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"),
                    reason="needs g++ and the ROCm headers")
def test_planner_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "plan_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "plan.cpp"), "-x", "c++", os.path.join(CSRC, "api.hip"),
           os.path.join(ROOT, "tests", "native", "plan_sanitize.cpp"),
           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=600)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitized planner run ok" in r.stdout


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"),
                    reason="needs g++ and the ROCm headers")
@pytest.mark.parametrize("sanitizer", ["thread", "address,undefined"])
def test_store_and_layer_pipeline_under_sanitizers(tmp_path, sanitizer):
    """store.cpp (tiers, files, reader threads, ring, fall-back paths) with the HIP runtime
    replaced by plain-memory stand-ins: ThreadSanitizer for the reader pool, ASan/UBSan for the
    buffers."""
    exe = str(tmp_path / "store_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=" + sanitizer, "-fno-sanitize-recover=undefined",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "store.cpp"),
           os.path.join(ROOT, "tests", "native", "store_sanitize.cpp"), "-lpthread", "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=600)
    disk = tmp_path / "disk"
    disk.mkdir()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", TSAN_OPTIONS="halt_on_error=1",
               LD_PRELOAD="")
    r = subprocess.run([exe, str(disk)], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitized store run ok" in r.stdout
