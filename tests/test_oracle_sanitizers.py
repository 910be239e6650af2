"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle is built a second
time with both (any finding aborts) and its whole pin suite runs against that build in a child
process.  Host code only; nothing here touches a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _libasan():
    p = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return p if os.path.isabs(p) and os.path.exists(p) else None


@pytest.mark.skipif(_libasan() is None, reason="no libasan beside this gcc")
def test_oracle_pins_pass_under_asan_and_ubsan(tmp_path):
    from oracle import lococo_oracle as orc
    lib = orc.build_sanitized(str(tmp_path / "liblococo_oracle_san.so"))
    env = dict(os.environ)
    env["LOCOCO_ORACLE_LIB"] = lib
    # the sanitizer runtime has to come first among the preloaded libraries; whatever is already
    # preloaded stays behind it
    env["LD_PRELOAD"] = ":".join(x for x in (_libasan(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"     # the interpreter's own leaks are not ours
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_backward_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert " passed" in r.stdout, tail
