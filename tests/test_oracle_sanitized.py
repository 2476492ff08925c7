"""The oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a C
driver calls every entry point on small pseudo-random problems; both the sanitized and the plain
build must run clean and print the same checksum."""
import os
import shutil
import subprocess

import pytest

from conftest import ROOT


def build_and_run(tmp_path, name, flags):
    exe = str(tmp_path / name)
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-I", os.path.join(ROOT, "oracle")] + flags + [
        os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "ppo.c"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)  # the sanitizer's runtime must come first in the library list
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    return res


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    plain = build_and_run(tmp_path, "plain", [])
    assert plain.returncode == 0, plain.stderr
    san = build_and_run(tmp_path, "sanitized", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                                                "-fno-omit-frame-pointer"])
    assert san.returncode == 0, san.stderr[-4000:]
    assert "runtime error" not in san.stderr and "ERROR: AddressSanitizer" not in san.stderr, san.stderr[-4000:]
    assert plain.stdout == san.stdout and plain.stdout.startswith("checksum ")
