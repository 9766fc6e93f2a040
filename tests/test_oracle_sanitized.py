"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

A child process preloads the sanitizer runtime, makes ``oracle`` load its ``-fsanitize=address,undefined`` build and
runs the small forward / backward pins again: ragged lengths, causal masks, grouped-query heads, sampled rows and keys,
the P dump, the MX and two-level variants and the block mask all index buffers in their own way, and an access outside
them, a signed overflow or a misaligned access aborts the child.  The pins' own assertions hold as well, so the
sanitized build also computes the same numbers."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PINS = ["tests/test_oracle_fwd.py", "tests/test_oracle_bwd.py", "tests/test_oracle_twolevel.py",
        "tests/test_oracle_blocksparse.py", "tests/test_oracle_ablation.py", "tests/test_oracle_smoothk.py"]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not on PATH")
def test_oracle_pins_pass_under_asan_and_ubsan():
    import oracle
    oracle.build_sanitized()
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no libasan.so next to gcc")
    env = dict(os.environ)
    env["LD_PRELOAD"] = (asan + " " + env.get("LD_PRELOAD", "")).strip()
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["ATTNQAT_ORACLE_SANITIZED"] = "1"
    env["OMP_NUM_THREADS"] = "4"
    probe = subprocess.run([sys.executable, "-c", "import oracle; print(oracle.e4m3_value(0x7e))"], cwd=ROOT, env=env,
                           capture_output=True, text=True, timeout=300)
    if probe.returncode != 0 and "ASan runtime does not come first" in probe.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from coming first")
    assert probe.returncode == 0 and probe.stdout.strip() == "448.0", probe.stderr[-2000:]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=1500)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "passed" in r.stdout and "failed" not in r.stdout
