"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, never on a GPU): the host half of
libepara (csrc/epara_host.cpp: planner, scheduler, handler, placement, simulator) and the C oracle
(oracle/dense_oracle.c) are compiled with -fsanitize=address,undefined together with tests/sanitize_driver.cpp
and run over seeded inputs; a report from either sanitizer fails the test."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_planner_and_oracle_are_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_driver")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan", "-g", "-O1"]
    obj = str(tmp_path / "oracle.o")
    subprocess.check_call(["gcc"] + san + ["-c", os.path.join(ROOT, "oracle", "dense_oracle.c"), "-o", obj])
    subprocess.check_call(["g++", "-std=c++17"] + san + ["-I" + os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "sanitize_driver.cpp"),
                           os.path.join(ROOT, "paper_2511_00603_amd", "csrc", "epara_host.cpp"), obj, "-o", exe, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the process
    r = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "sanitize_driver: ok" in r.stdout and "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout, r.stdout[-4000:]
