"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): a
driver calls every entry point on exactly sized heap buffers; a stray access aborts it."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_c_code_is_clean_under_asan_and_ubsan():
    src = [os.path.join(ROOT, "oracle", f) for f in ("rglru_oracle.c", "sanitize_driver.c")]
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_sanitize")
        subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined",
                               "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", exe] + src + ["-lm"])
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1", OMP_NUM_THREADS="3")
        r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
        assert r.returncode == 0 and r.stdout.strip().endswith("ok"), r.stdout[-4000:]
