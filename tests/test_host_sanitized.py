"""The library's host code and both oracles under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

tests/host_sanitizer_driver.cpp is compiled together with the packer / validator, the error-bound code, the encode
side's host functions and the two C oracles, and run: pack -> validate -> unpack round trips in exactly-sized heap
buffers, a seeded mutation fuzz of the blob (byte flips, truncations, boundary values written into header, index and
layer-record fields) that validate_blob must answer with RINR_OK or an error code without reading outside the buffer,
and the host functions and oracles on small inputs.  Any sanitizer report aborts the driver."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2306_16699_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs g++ and gcc")
def test_host_code_under_asan_ubsan(tmp_path):
    san = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    objs = []
    for src in ("inr_oracle.c", "fit_oracle.c"):
        o = str(tmp_path / (src + ".o"))
        subprocess.run(["gcc", "-std=c11", "-fopenmp", *san, "-c", os.path.join(ROOT, "oracle", src), "-o", o], check=True)
        objs.append(o)
    exe = str(tmp_path / "driver")
    subprocess.run(["g++", "-std=c++17", "-fopenmp", *san, os.path.join(ROOT, "tests", "host_sanitizer_driver.cpp"),
                    os.path.join(CSRC, "rinr_pack.cpp"), os.path.join(CSRC, "rinr_bounds.cpp"), os.path.join(CSRC, "rinr_encode.cpp"),
                    *objs, "-o", exe, "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([exe, "40", "400"], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "sanitizer driver: ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
