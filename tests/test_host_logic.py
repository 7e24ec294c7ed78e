"""Host logic of the library that no GPU is needed for, compiled from the library's own header and
run on the CPU."""
import os
import shutil
import subprocess

import pytest

from conftest import ROOT


def _build_and_run(tmp_path, name):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = tmp_path / name
    src = os.path.join(ROOT, "tests", "host", name + ".hip")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", os.path.join(ROOT, "include"),
                    "-I", os.path.join(ROOT, "paper_2605_11744_amd", "csrc"), src, "-o", str(exe)],
                   check=True, capture_output=True, timeout=600)
    return subprocess.run([str(exe)], capture_output=True, text=True, timeout=600).stdout


def test_item_mapping_is_one_to_one_and_longest_first(tmp_path):
    """item_coords (the integer part of the kernels' block-index resolution) over some 10,000 launch
    shapes -- dense, packed, retrieved-prefix and split-prefix forms, every sub-group count -- maps
    the item indices one-to-one onto (segment, block, head, sequence, sub-group, piece), lists the
    full-history heads first and longest first, and gives the same answer with the host-prepared
    divisors as with plain divisions."""
    out = _build_and_run(tmp_path, "item_coords_check")
    assert out.startswith("ok "), out
    launches, items = (int(x) for x in out.split()[1:3])
    assert launches > 5000 and items > 10_000_000


def test_launch_divisors_are_exact(tmp_path):
    """The multiply-shift pairs the launchers prepare (FastDiv) give n / d and n % d exactly for every
    divisor up to 70000, the neighbours of every power of two, 200000 random divisors, and for each
    the edge values and random n below 2^31."""
    out = _build_and_run(tmp_path, "fastdiv_check")
    assert out.startswith("ok "), out
    assert int(out.split()[1]) > 10_000_000
