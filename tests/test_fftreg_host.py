"""The in-register transforms on the CPU: csrc/circ_fftreg.h is plain C++ apart from its device
markers, so tests/fftreg_host/check_fftreg.cpp runs every sub-transform size (radix-2 and odd-prime
butterflies, forward and inverse) and the two-pass split of every block size with a fast transform
against the definition of the DFT in double precision (Sec. 4.1)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "fftreg_host", "check_fftreg.cpp")
INC = os.path.join(ROOT, "paper_1708_08917_amd", "csrc")


@pytest.fixture(scope="module")
def lines(tmp_path_factory):
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path_factory.mktemp("fftreg") / "check_fftreg")
    subprocess.run([cxx, "-std=c++17", "-O1", "-I", INC, "-o", exe, SRC], check=True, capture_output=True, text=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    return [l.split() for l in out.splitlines()]


def test_every_sub_transform_matches_the_definition(lines):
    reg = [l for l in lines if l[0] == "reg"]
    assert {int(l[2]) for l in reg} >= {3, 5, 6, 8, 10, 12, 16, 20, 24, 25, 32} and len(reg) == 34
    for _, direction, size, err in reg:
        assert float(err) < 2e-6, (direction, size, err)


def test_two_pass_split_matches_the_definition(lines):
    two = [l for l in lines if l[0] == "two-pass"]
    assert {int(l[2]) for l in two} >= {64, 128, 256, 96, 100, 384, 400} and len(two) == 46
    for _, direction, size, err in two:
        assert float(err) < 4e-6, (direction, size, err)
