"""The C oracles under AddressSanitizer and UndefinedBehaviorSanitizer (host only, no GPU): both files are compiled
with ``-O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all`` into a temporary directory and the pins that
drive them hardest (hand-worked traces, brute force over tiny instances, window edges, order-statistic definition,
invariants, children rows, the agentic schedules) run again in a child interpreter that loads those builds.  Any
finding aborts the child."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
       "-fno-omit-frame-pointer"]


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    replay = str(tmp_path / "libap_oracle_san.so")
    agentic = str(tmp_path / "libagentic_oracle_san.so")
    subprocess.run(["gcc", *SAN, "-pthread", os.path.join(ROOT, "oracle", "ap_oracle.c"), "-o", replay], check=True)
    subprocess.run(["gcc", *SAN, os.path.join(ROOT, "oracle", "agentic_oracle.c"), "-o", agentic], check=True)
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()
    env = dict(os.environ, AP_ORACLE_LIB=replay, AP_AGENTIC_ORACLE_LIB=agentic, LD_PRELOAD=runtime,
               ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    # the statistical M/D/1 pin replays a million requests and is left to the plain build
    run = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_agentic_pins.py"),
                          "-k", "not pollaczek and not md1"],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = run.stdout + run.stderr
    assert run.returncode == 0, out[-4000:]
    assert "passed" in out and "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
