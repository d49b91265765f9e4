"""Host-only checks of logic that decides launch shapes and barrier schedules: small C++ programs compiled with the
system compiler under the address and undefined-behaviour sanitizers (no GPU, no HIP)."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def build_and_run(src, tmp_path):
    exe = os.path.join(tmp_path, os.path.basename(src) + ".bin")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", src, "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-4000:]
    return run.stdout


def test_decoder_stack_schedule(tmp_path):
    """Compute waves and helper waves of the decoder stack kernel arrive at the same barriers, in the same order, for
    every worker of many shapes; the compute waves consume exactly the worker's tiles; LDS regions fit."""
    out = build_and_run(os.path.join(HERE, "host", "stack_sched_check.cpp"), str(tmp_path))
    assert "0 violations" in out, out


def test_layout_and_dispatch_rules(tmp_path):
    """Workspace layout, staging size, split factors and the tile rule on thousands of random configurations
    (bpd_host_logic.h compiled for the host)."""
    out = build_and_run(os.path.join(HERE, "host", "host_logic_check.cpp"), str(tmp_path))
    assert " 0 violations" in out, out
