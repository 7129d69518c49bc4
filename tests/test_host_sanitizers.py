"""AddressSanitizer + UndefinedBehaviorSanitizer run of all host-side code that has no device calls: the C
oracle, the library's host bookkeeping (csrc/pool_host.h) and its split controller (csrc/alpha_ctl.h).
tests/host_san/replay.cpp replays random KV / split traces on the bookkeeping and the oracle side by side and
drives the oracle's cache and layer routines over small, ragged and invalid inputs; the test builds it with
-fsanitize=address,undefined (errors are fatal) and expects a clean exit."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1",
           "-fopenmp"]
    objs = []
    for src in ("pool_oracle.c", "hstu_oracle.c"):
        obj = str(tmp_path / (src + ".o"))
        subprocess.check_call(["gcc", "-std=c11", "-Wall"] + san + ["-c", os.path.join(ROOT, "oracle", src), "-o", obj])
        objs.append(obj)
    exe = str(tmp_path / "replay")
    subprocess.check_call(["g++", "-std=c++17", "-Wall"] + san +
                          [os.path.join(ROOT, "tests", "host_san", "replay.cpp")] + objs +
                          ["-static-libasan", "-lm", "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    run = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    sys.stdout.write(run.stdout[-4000:])
    assert run.returncode == 0, run.stdout[-4000:]
    assert "host sanitizer replay: ok" in run.stdout
