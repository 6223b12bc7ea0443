"""The oracle's pins once more, against the build of the oracle under AddressSanitizer and
UndefinedBehaviorSanitizer: its index arithmetic over the message arrays ([2t+1][k][count],
[k][n][count], pooling windows) must stay inside its buffers and free of undefined behaviour on every
case the pins run.  A finding aborts the child process, which fails this test."""
import os
import subprocess
import sys

import pytest

from oracle import build as orc_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(not orc_build.sanitizer_runtime(), reason="this toolchain has no libasan")
def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    orc_build.build_sanitized()
    env = orc_build.sanitizer_env()
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=1200)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    # the child really ran on the sanitized library
    probe = subprocess.run([sys.executable, "-c",
                            "import oracle.ssnet_oracle as o; print(o._lib._name)"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert probe.stdout.strip().endswith("libssnet_oracle_san.so"), probe.stdout + probe.stderr
