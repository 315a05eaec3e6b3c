"""Host sanitizer build of the two plain-C sources (CPU oracle, input generator): AddressSanitizer and
UndefinedBehaviorSanitizer over a tiny model that goes through every exported routine.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_generator_are_clean_under_asan_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "san_driver")
    cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-DPV_REAL=double", "-o", exe, os.path.join(ROOT, "tests", "san_driver.c"),
           os.path.join(ROOT, "oracle", "ref_decoder.c"), os.path.join(ROOT, "pv_inputs", "synth.c"), "-lm"]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)            # the sanitizer runtime has to come first in the library list
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "san_driver ok" in r.stdout, r.stdout + r.stderr
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
