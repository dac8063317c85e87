"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

tests/oracle_sanitize_main.c calls every exported function of oracle/scmoe_oracle.c on small
inputs that reach the ends of its arrays (empty inputs, an empty expert segment, capacity 0,
expert indices outside [0, E), k up to 4).  It is built twice, once with the sanitizers and
once with the flags of the ordinary oracle build, and run in child processes: the sanitized
run must finish clean, and both must print the same sums.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), os.path.join(ROOT, "oracle", "scmoe_oracle.c")]


def _build_and_run(tmp_path, name, flags, env=None):
    exe = str(tmp_path / name)
    subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra"] + flags + SRC + ["-o", exe, "-lm"])
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300,
                       env=dict(os.environ, **(env or {})))
    assert r.returncode == 0, "%s exited with %d\n%s\n%s" % (name, r.returncode, r.stdout[-2000:], r.stderr[-4000:])
    assert r.stderr.strip() == "", r.stderr[-4000:]
    lines = r.stdout.strip().splitlines()
    assert lines[-1] == "done"
    return lines


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path, oracle):
    san = _build_and_run(tmp_path, "oracle_san",
                         ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                          "-fno-sanitize-recover=all"],
                         env={"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1"})
    plain = _build_and_run(tmp_path, "oracle_plain", ["-O2"])
    assert len(san) >= 24
    assert san == plain
    # the scalar helpers of the same line, through the library the other tests use
    f = san[0].split()
    assert f[0] == "scalar"
    want = [oracle.round_to_bf16(1.00390625), oracle.round_to_bf16(-3.1415926), oracle.gelu(0.7, 0),
            oracle.gelu(-1.3, 1)]
    assert [float(v) for v in f[1:5]] == want
    assert [int(v) for v in f[5:8]] == [oracle.capacity(8192, 8, 1, 1.25), oracle.capacity(100, 7, 2, 1.0),
                                       oracle.capacity(0, 3, 1, 2.0)]
