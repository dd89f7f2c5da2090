"""The C part of the CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): a small C
driver runs both entry points over several shapes, edge sizes included; the sanitized binary must finish clean
and print exactly what the ordinary build prints."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = [os.path.join(HERE, "sanitize_accept_driver.c"), os.path.join(os.path.dirname(HERE), "oracle", "accept.c")]


def _build_and_run(tmp, name, flags):
    exe = os.path.join(tmp, name)
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra", *flags, "-o", exe,
                    *SRC, "-lm"], check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)             # the sanitizer runtime has to be the first library of the process
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_accept_c_is_clean_under_asan_and_ubsan(tmp_path):
    plain = _build_and_run(str(tmp_path), "plain", [])
    assert plain.returncode == 0, plain.stdout + plain.stderr
    try:
        san = _build_and_run(str(tmp_path), "san", ["-fsanitize=address,undefined", "-fno-omit-frame-pointer"])
    except subprocess.CalledProcessError as e:
        pytest.skip("this gcc cannot link the sanitizer runtimes: " + e.stderr[-200:])
    assert san.returncode == 0, san.stdout[-2000:] + san.stderr[-4000:]
    assert "runtime error" not in san.stderr and "AddressSanitizer" not in san.stderr, san.stderr[-4000:]
    assert san.stdout == plain.stdout and "done bad 0" in san.stdout
