"""CPU sanitizer build: the library's host-only translation unit and the C oracle, compiled with
AddressSanitizer and UndefinedBehaviorSanitizer (runtime linked statically, so that nothing is preloaded),
run through their entry points by tests/host_sanitize_main.cpp."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_and_oracle_under_the_sanitizers(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1", "-ffp-contract=off"]
    oracle_o = str(tmp_path / "oracle.o")
    subprocess.check_call(["gcc", "-std=c11", "-fopenmp", *san, "-c", "-o", oracle_o, os.path.join(ROOT, "oracle", "sop_oracle.c")])
    subprocess.check_call(["g++", "-std=c++17", *san, "-static-libasan", "-static-libubsan", "-fopenmp", "-o", exe,
                           os.path.join(ROOT, "tests", "host_sanitize_main.cpp"),
                           os.path.join(ROOT, "paper_2605_14929_amd", "csrc", "sop_host.cpp"), oracle_o, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and "sanitize ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
