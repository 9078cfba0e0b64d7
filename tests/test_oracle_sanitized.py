"""The oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host code, CPU only):
every pin is run against that build in a child process, so an out-of-bounds access, a signed
overflow or a misaligned load inside the oracle ends the test instead of quietly producing the
expected values every parity claim rests on."""

import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = """
import sys
sys.path[:0] = [%(root)r, %(tests)r]
import oracle, oracle_pins
lib = oracle.load(%(lib)r)
for pin in oracle_pins.ALL_PINS:
    pin(lib)
print("pins passed:", len(oracle_pins.ALL_PINS))
"""


def test_all_pins_pass_on_the_sanitized_oracle(tmp_path):
    lib_path = oracle.build(oracle.SOURCE, str(tmp_path / "libpx_oracle_san.so"), oracle.SANITIZE_FLAGS)
    runtime = subprocess.run(["g++", "-print-file-name=libasan.so"], capture_output=True, text=True,
                             check=True).stdout.strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime), "g++ has no AddressSanitizer runtime"
    env = dict(os.environ)
    # the sanitizer runtime has to be the first library of the process; whatever is preloaded already stays
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=99"        # the interpreter itself leaks at exit
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=98"
    code = CHILD % {"root": ROOT, "tests": os.path.join(ROOT, "tests"), "lib": lib_path}
    res = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=900)
    assert res.returncode == 0, "sanitized oracle run failed (%d):\n%s\n%s" % (
        res.returncode, res.stdout[-2000:], res.stderr[-6000:])
    assert "pins passed:" in res.stdout
