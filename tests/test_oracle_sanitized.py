"""The oracle's pins once more, against a build of oracle_attn.c instrumented with the host compiler's address and
undefined-behaviour sanitizers (CPU only): an out-of-bounds read of a pool, table or output row, a misaligned access or
a signed overflow in the index arithmetic aborts the child process."""
import os
import subprocess
import sys

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    oracle_build.build(force=True, sanitize=True)
    env = dict(os.environ)
    env["ORACLE_SANITIZED"] = "1"
    # the sanitizer runtime must come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = ":".join(x for x in (oracle_build.sanitizer_runtime(), env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"          # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    # the child really maps the instrumented library and its runtime
    probe = "import oracle; oracle.lib(); m = open('/proc/self/maps').read(); print('liboracle_attn_san.so' in m, 'libasan' in m)"
    r = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.split() == ["True", "True"], r.stdout + r.stderr
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
