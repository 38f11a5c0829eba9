"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only).

`oracle/sanitize_check.c` includes the oracle's source and drives every exported function on small flows
whose buffers have exactly their stated sizes; any out-of-bounds access, misaligned access, signed
overflow or leak ends the run with a non-zero status.  It also re-checks the invariants the paper fixes
(eq. 4 / eq. 5 mutual inverses, Prop. 3.2) so that the instrumented build is known to compute the same
thing as the one the tests use.  Both arithmetic types are built and run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sanitize_check.c")


@pytest.mark.parametrize("ctype", ["double", "float"])
def test_oracle_runs_clean_under_address_and_undefined_sanitizers(tmp_path, ctype):
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the image"
    exe = str(tmp_path / f"sanitize_check_{ctype}")
    cmd = [gcc, "-O1", "-g", "-std=gnu99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           f"-DREAL={ctype}", "-Wall", "-Wextra", SRC, "-o", exe, "-lm"]
    subprocess.run(cmd, check=True, cwd=ROOT)
    env = dict(os.environ)
    # other preloaded libraries may precede the sanitizer runtime in the link order; that is harmless here
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "sanitize_check: ok" in r.stdout
