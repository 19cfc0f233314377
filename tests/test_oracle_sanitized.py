"""The oracle's pins once more with the oracles compiled under AddressSanitizer + UndefinedBehaviorSanitizer
(oracle/build.py --sanitize): a child pytest process with the ASan runtime preloaded loads lib*_san.so instead of the
regular builds and runs the rule, invariant, sampler, superko, brute-force and Hex pins (the three exhaustive
enumerations, whose time goes to the Python side, are left to the regular run).  No GPU."""
import os
import subprocess
import sys

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["test_oracle_rules.py", "test_oracle_invariants.py", "test_oracle_sampler.py", "test_oracle_superko.py",
        "test_oracle_bruteforce.py", "test_hex_oracle.py"]


def test_oracle_pins_under_asan_and_ubsan():
    oracle_build.build(force=True, sanitize=True)
    oracle_build.build_hex(force=True, sanitize=True)
    env = dict(os.environ)
    env["ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = ":".join(x for x in (oracle_build.asan_runtime(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"     # the interpreter's own leaks are not the subject
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", "not exhaustive",
           *[os.path.join(ROOT, "tests", f) for f in PINS]]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
    assert " passed" in out and "failed" not in out
    # the child really ran the sanitized builds
    probe = subprocess.run([sys.executable, "-c", "import oracle; from oracle import hex as hx; oracle.lib(); hx.lib(); "
                            "print(open('/proc/self/maps').read().count('_oracle_san.so') > 0)"], cwd=ROOT, env=env, capture_output=True, text=True)
    assert probe.stdout.strip() == "True", probe.stdout + probe.stderr
