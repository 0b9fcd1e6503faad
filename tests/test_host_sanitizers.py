"""The library's pure host code (planner, page table, scheduling primitives) under AddressSanitizer /
UBSan: compiled with g++ from the library's own sources (no GPU code involved) and run on random
inputs."""

import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2605_10195_amd", "csrc")


def build_with_sanitizers(exe, sources):
    build = subprocess.run(
        ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-static-libasan", "-static-libubsan"] + sources + ["-o", exe], capture_output=True, text=True)
    if build.returncode != 0 and "cannot find" in build.stderr and any(w in build.stderr for w in ("asan", "ubsan", "sanitize")):
        pytest.skip("the sanitizer runtime is not installed")
    assert build.returncode == 0, build.stderr[-2000:]


def test_c_abi_host_side_under_address_sanitizer(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("needs hipcc")
    exe = str(tmp_path / "api_fuzz")
    sources = [os.path.join(CSRC, f) for f in ("api.cpp", "planner.cpp", "page_table.cpp", "sched.cpp", "kernels.hip")]
    build = subprocess.run(
        [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-x", "hip"] + sources +
        [os.path.join(HERE, "api_fuzz.cpp"), "-o", exe], capture_output=True, text=True)
    if build.returncode != 0 and any(w in build.stderr for w in ("asan", "sanitizer")):
        pytest.skip("the sanitizer runtime of the HIP compiler is not installed")
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([exe, "120"], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert run.stdout.startswith("ok:"), run.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_scheduling_fuzz_under_sanitizers(tmp_path):
    exe = str(tmp_path / "sched_fuzz")
    build_with_sanitizers(exe, [os.path.join(HERE, "sched_fuzz.cpp"), os.path.join(CSRC, "sched.cpp")])
    run = subprocess.run([exe, "3000"], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert run.stdout.startswith("ok:"), run.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_fuzz_under_sanitizers(tmp_path):
    exe = str(tmp_path / "planner_fuzz")
    build_with_sanitizers(exe, [os.path.join(HERE, "planner_fuzz.cpp"), os.path.join(CSRC, "planner.cpp"),
                                os.path.join(CSRC, "page_table.cpp")])
    run = subprocess.run([exe, "120"], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert run.stdout.startswith("ok:"), run.stdout
    patched_with_pages = int(run.stdout.split("(")[1].split()[0])
    assert patched_with_pages > 1000
