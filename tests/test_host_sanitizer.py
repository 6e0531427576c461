"""The library's pure host logic (balancer, partition, pipeline step plan, the
Evaluator's record ring on a scripted event layer) compiled with g++ under
AddressSanitizer and UndefinedBehaviorSanitizer and run on the CPU.  No HIP."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_logic_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2510_15882_amd", "csrc")
    exe = str(tmp_path / "host_check")
    subprocess.run(
        ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=all", "-static-libasan", "-I", os.path.join(ROOT, "include"), "-I", csrc,
         os.path.join(ROOT, "tests", "host_sanitizer", "host_check.cpp"), os.path.join(csrc, "balancer.cpp"),
         "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "host check passed" in run.stdout
