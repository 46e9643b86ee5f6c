"""CPU sanitizer build (no GPU): the plain C oracle and the library's two host planners,
compiled with AddressSanitizer and UndefinedBehaviorSanitizer and run over small ragged and
degenerate inputs by tests/san_driver.cpp.  The GPU machines offer no device sanitizer, so this
is where out-of-bounds indexing in the host-side code would show."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1"]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_oracle_and_host_planners_under_asan_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2510_19366_amd", "csrc")
    objs = []
    jobs = [(["gcc", "-std=gnu11", "-ffp-contract=off"], os.path.join(ROOT, "oracle", "moe_prism_oracle.c")),
            (["g++", "-std=c++17", "-x", "c++"], os.path.join(csrc, "batcher.hip")),
            (["g++", "-std=c++17", "-x", "c++"], os.path.join(csrc, "partition.hip")),
            (["g++", "-std=c++17"], os.path.join(ROOT, "tests", "san_driver.cpp"))]
    for cc, src in jobs:
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([*cc, *SAN, "-c", src, "-o", obj], check=True, capture_output=True, text=True)
        objs.append(obj)
    exe = str(tmp_path / "san_driver")
    subprocess.run(["g++", *SAN, "-o", exe, *objs, "-lm"], check=True, capture_output=True, text=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "sanitizer run clean" in r.stdout
