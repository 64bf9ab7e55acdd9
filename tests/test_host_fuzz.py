"""CPU differential fuzz of the library's host logic under ASan + UBSan.

tests/host_fuzz.cpp drives the library's block table (eager block rotation,
paper Section 4.3.2) and its VLT / LVF scheduler (Section 4.2, Algorithm 1)
next to the oracle's with long random operation sequences, and compares every
return code, mapping, state, counter and byte after every operation.  It is
built here with the host sanitizers, with a host stand-in for the two engine
calls the table makes, so it needs no GPU.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-O1", "-g"]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_table_and_scheduler_agree_with_oracle_under_sanitizers(tmp_path):
    oracle_o = tmp_path / "oracle.o"
    exe = tmp_path / "host_fuzz"
    subprocess.run(["gcc", "-std=c11", *SAN, "-pthread", "-c", os.path.join(ROOT, "oracle", "duplexkv_oracle.c"),
                    "-o", str(oracle_o)], check=True)
    csrc = os.path.join(ROOT, "paper_2601_20309_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", *SAN,
                    # the engine's internal header names HIP types; nothing of HIP is called or linked
                    "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                    os.path.join(ROOT, "tests", "host_fuzz.cpp"), os.path.join(csrc, "kv_table.cpp"),
                    os.path.join(csrc, "kv_sched.cpp"), str(oracle_o), "-static-libasan", "-pthread",
                    "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")
    run = subprocess.run([str(exe), "20000", "20000"], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-4000:]
    assert "host fuzz ok" in run.stdout
