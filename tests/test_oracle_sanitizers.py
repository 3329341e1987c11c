"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle's pins are run once more in a child
process against a sanitizer build of oracle/fk_oracle.c (host code only; nothing here touches a GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["test_oracle_attention.py", "test_oracle_scorer.py", "test_oracle_select_compact.py", "test_oracle_protocol.py",
        "test_oracle_sampled.py", "test_oracle_features.py"]


def test_oracle_pins_under_asan_and_ubsan():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc's AddressSanitizer runtime is not installed"
    env = dict(os.environ)
    env["FK_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")   # the runtime first, whatever was preloaded stays
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"     # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *[os.path.join(ROOT, "tests", f) for f in PINS]]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0, out[-4000:]
    assert " passed" in out
