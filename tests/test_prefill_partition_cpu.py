"""The work partition of the 8-wave prefill kernel, checked on the host: tests/partition_check.cpp includes the
library's own partition arithmetic (csrc/hi_prefill_part.h, csrc/hi_internal.h: plain integer code shared by the
kernel, the merge kernel and the launcher) and replays the launches of prefill units on sets of tile ids.  Every
block of query positions must see each past tile and each own tile at or below its causal boundary exactly once
(Eq. 3: row p attends to keys 0..p), whatever the kernel variant, split, pairing and number of launches; images are
loaded only after they were stored, never by two workgroups; and the carry the plan sizes covers every launch."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_tile_is_counted_exactly_once(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "partition_check")
    subprocess.run([gxx, "-O2", "-std=c++17", "-I", os.path.join(ROOT, "include"),
                    "-I", os.path.join(ROOT, "paper_2502_12574_amd", "csrc"),
                    os.path.join(ROOT, "tests", "partition_check.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    assert " 0 failures" in r.stdout, r.stdout[-2000:]
