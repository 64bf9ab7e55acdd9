"""The plain-C example: the library is usable through its C ABI alone, with no
Python and no PyTorch in the process."""
import os
import re
import subprocess

import pytest

from paper_2601_20309_amd import build as hipbuild


def test_example_compiles_against_the_public_header(tmp_path):
    out = hipbuild.build_example(str(tmp_path / "duplex_demo"))
    assert os.path.exists(out)


@pytest.mark.gpu
def test_example_rotates_and_verifies_on_the_gpu():
    exe = hipbuild.EXAMPLE_BIN
    assert os.path.exists(exe), "examples/duplex_demo is built by __graft_entry__.build()"
    run = subprocess.run([exe, "128"], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-2000:]
    assert "rotation verified on the CPU: 128 blocks out, 128 in" in run.stdout
    assert "kv_rotate_static verified on the CPU" in run.stdout
    m = re.search(r"duplex rotation: ([0-9.]+) ms, ([0-9.]+) GB/s", run.stdout)
    assert m and float(m.group(2)) > 60.0, run.stdout
