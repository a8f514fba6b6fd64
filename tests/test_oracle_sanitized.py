"""The oracle's pins once more with the oracle compiled under -fsanitize=address,undefined
(oracle/build.py, sanitize=True): a child process loads the sanitized library instead of the
plain one and runs the oracle test files; an access out of bounds, a signed overflow or a use
of freed memory anywhere in the oracle aborts it.  Host code only -- nothing here touches a GPU."""
import os
import subprocess
import sys

import pytest

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILES = ["test_oracle_fps.py", "test_oracle_mdps.py", "test_oracle_ball_query.py", "test_oracle_knn.py",
         "test_oracle_excl_lists.py", "test_oracle_mlp.py"]


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    lib = oracle_build.build(sanitize=True)
    assert os.path.exists(lib)
    runtime = oracle_build.asan_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("no AddressSanitizer runtime next to gcc")
    env = dict(os.environ)
    env["FASTPOINT_ORACLE_SANITIZE"] = "1"
    # the sanitizer's runtime has to come first among the preloaded libraries; whatever is
    # preloaded already stays behind it.  Python's own allocations are not the oracle's: no leak report.
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + \
          [os.path.join(ROOT, "tests", f) for f in FILES]
    res = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=900)
    out = res.stdout.decode(errors="replace")
    if res.returncode != 0 and "ASan runtime does not come first" in out:
        pytest.skip("the AddressSanitizer runtime cannot be preloaded first on this machine")
    assert res.returncode == 0, out[-4000:]
    assert "passed" in out and "libfastpoint_ref_san" not in out
