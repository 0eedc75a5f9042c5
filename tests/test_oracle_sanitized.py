"""The oracle's pins once more on a sanitizer-instrumented build of the same C source (undefined behaviour, strict array
bounds, float-to-integer overflow: any report aborts the run), in a child process."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_on_an_instrumented_oracle(tmp_path):
    from oracle import build as obuild
    san = obuild.build(out=str(tmp_path / "liblq_oracle_san.so"), sanitize=True)
    env = dict(os.environ, LQ_ORACLE_LIB=san, UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-2000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in r.stdout + r.stderr, tail
