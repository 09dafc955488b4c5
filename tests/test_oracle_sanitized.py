"""The oracle's pins once more against a build of graft_oracle.c with AddressSanitizer and
UndefinedBehaviorSanitizer (every report fatal): the pins stay green and no out-of-bounds access,
overflow or misaligned load is reported on any of their inputs, error paths included."""
import glob
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    oracle.build(sanitize=True)
    files = sorted(f for f in glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py"))
                   if not f.endswith("test_oracle_sanitized.py"))
    assert len(files) >= 7
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=oracle.sanitizer_env(), stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True, timeout=900)
    tail = r.stdout[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in tail and "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, tail
    # the child really ran the sanitized library
    probe = subprocess.run([sys.executable, "-c",
                            "import oracle, os; oracle.retrieve([[1, 2, 1, 2]], [4], 1, 2, 1, 1); "
                            "print(os.path.basename(oracle._load()._name))"],
                           cwd=ROOT, env=oracle.sanitizer_env(), stdout=subprocess.PIPE, text=True, timeout=120)
    assert probe.stdout.strip() == "libgraft_oracle_san.so", probe.stdout
