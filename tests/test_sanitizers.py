"""The oracle's C code and the library's host-only logic under AddressSanitizer and UndefinedBehaviorSanitizer, on the
CPU (a sanitizer never goes near the GPU): tests/sanitize/driver.cc is built with -fsanitize=address,undefined
against oracle/kvcomp_oracle.c and paper_2509_00579_amd/csrc/host_logic.h and run; it repeats the codebook and codec
pins that need no device, and checks the library's host codebook against the oracle's."""
import pathlib
import shutil
import subprocess

import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="needs gcc and g++")
def test_oracle_and_host_logic_under_asan_and_ubsan(tmp_path):
    obj = tmp_path / "oracle.o"
    exe = tmp_path / "driver"
    subprocess.run(["gcc", "-std=c99", *SAN, "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-c",
                    str(ROOT / "oracle" / "kvcomp_oracle.c"), "-o", str(obj)], check=True)
    subprocess.run(["g++", "-std=c++17", *SAN, "-ffp-contract=off", "-Wall", "-Wextra",
                    str(ROOT / "tests" / "sanitize" / "driver.cc"), str(obj), "-o", str(exe), "-lm"], check=True)
    r = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600,
                       env={"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
                            "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1"})
    assert r.returncode == 0, r.stdout[-4000:]
    assert "sanitizer driver: ok" in r.stdout
