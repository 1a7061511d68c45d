"""The planner under AddressSanitizer and UndefinedBehaviorSanitizer, host code only (no GPU): the
library's host source is compiled with g++ -fsanitize=address,undefined against stubbed kernel
launchers and driven with random pools and batches; the placement routine with random demands."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIP_INCLUDE = "/opt/rocm/include"
HIP_LIB = "/opt/rocm/lib"


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(HIP_INCLUDE), reason="needs g++ and the HIP headers")
def test_planner_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "planner_sanitizer_driver")
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__", "-I" + HIP_INCLUDE,
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2511_22880_amd", "csrc"),
           "-o", exe, os.path.join(ROOT, "tests", "planner_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2511_22880_amd", "csrc", "lora_host.cpp"),
           os.path.join(ROOT, "paper_2511_22880_amd", "csrc", "lora_place.cpp"),
           "-L" + HIP_LIB, "-lamdhip64", "-Wl,-rpath," + HIP_LIB]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "asan" in (build.stderr or "").lower() and "cannot find" in build.stderr:
        pytest.skip("the sanitizer runtime is not installed")
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "planner sanitizer run ok" in run.stdout


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir(HIP_INCLUDE), reason="needs g++ and the HIP headers")
def test_planner_from_several_threads_under_thread_sanitizer(tmp_path):
    """Four threads create pools, plan, export and destroy at once, each on objects of its own: what the
    header allows.  ThreadSanitizer reports any state they share without saying so."""
    exe = str(tmp_path / "planner_thread_driver")
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=thread", "-fno-omit-frame-pointer", "-pthread",
           "-D__HIP_PLATFORM_AMD__", "-I" + HIP_INCLUDE,
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2511_22880_amd", "csrc"),
           "-o", exe, os.path.join(ROOT, "tests", "planner_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2511_22880_amd", "csrc", "lora_host.cpp"),
           os.path.join(ROOT, "paper_2511_22880_amd", "csrc", "lora_place.cpp"),
           "-L" + HIP_LIB, "-lamdhip64", "-Wl,-rpath," + HIP_LIB]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "tsan" in (build.stderr or "").lower() and "cannot find" in build.stderr:
        pytest.skip("the sanitizer runtime is not installed")
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1:report_signal_unsafe=0")
    run = subprocess.run([exe, "threads"], capture_output=True, text=True, env=env, timeout=300)
    if run.returncode != 0 and "unexpected memory mapping" in (run.stdout + run.stderr):
        pytest.skip("ThreadSanitizer cannot map its shadow memory in this container")
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "planner thread run ok" in run.stdout
