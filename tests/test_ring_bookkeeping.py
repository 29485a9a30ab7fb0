"""Host logic of the flash kernels: the scalar bookkeeping of the K/V block stream and of the ring
of LDS slots (csrc/ape_ring.h) compiles for the host, and tests/ring_sim.cpp drives it through
~52 000 streams (prefix + causal segments of every length up to several tiles, ragged chunk tables,
splits that start and end inside chunks, every wavefront's causal limit) in place of the MFMA work.
No GPU is needed."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs a host C++ compiler")
def test_ring_bookkeeping_simulation(tmp_path):
    exe = str(tmp_path / "ring_sim")
    cmd = ["g++", "-O1", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-o", exe, os.path.join(HERE, "ring_sim.cpp")]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, (run.stdout[-4000:], run.stderr[-4000:])
    last = run.stdout.strip().splitlines()[-1]
    assert " 0 failed" in last, last
    # the fast path is exercised, not only the generic one
    n_fast = int(last.split(";")[1].split()[0])
    assert n_fast > 1000, last
    # ... and so are the groups of bodies whose ring slots are compile-time constants (wide prefill tile)
    n_static = int(last.split(";")[2].split()[0])
    assert n_static > 1000 and n_static % 6 == 0, last
