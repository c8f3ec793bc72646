"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

The pins' small cases are run a second time, in a child process, against a build of
oracle/hq_oracle.c with -fsanitize=address,undefined: an out-of-bounds access, a signed overflow
or a misaligned access in the oracle ends that process with a report, which fails this test."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# every pin except the ones that only time out under instrumentation (exhaustive sweeps over
# millions of values keep a reduced range through HQ_ORACLE_SANITIZE, see test_oracle_pins.py)
SELECT = ("linear or conv or depthwise or minmax or qparams or idempotent or clip_counts or range_update "
          "or static_with_current or in_hindsight_sequence or weight_quantizer or weight_gradient_scale "
          "or accumulator_unit or real_tensor_quantizer or stochastic_rounding_against or saturation or logarithm")


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    sys.path.insert(0, ROOT)
    from oracle import build_sanitized
    build_sanitized.build(force=True)
    env = dict(os.environ)
    preload = [build_sanitized.runtime()] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env.update(HQ_ORACLE_SANITIZE="1", LD_PRELOAD=":".join(preload), OMP_NUM_THREADS="4",
               ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:abort_on_error=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-k", SELECT],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, tail
