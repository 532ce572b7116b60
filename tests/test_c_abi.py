"""The library driven from a plain C program (tests/c_abi/abi_smoke.c, compiled with gcc by
paper_2602_16839_amd.build): raw hipMalloc pointers through include/ptenc.h, closed-form expectations."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
BIN = os.path.join(HERE, "c_abi", "abi_smoke")


def test_c_program_is_built_and_links_the_library():
    assert os.path.exists(BIN), "run `python -m paper_2602_16839_amd.build` first"
    out = subprocess.run(["ldd", BIN], stdout=subprocess.PIPE, text=True).stdout
    assert "libptenc.so" in out and "not found" not in out.split("libptenc.so")[1].splitlines()[0]


@pytest.mark.gpu
def test_c_program_runs_the_decode_path():
    res = subprocess.run([BIN], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode == 0 and "abi_smoke ok" in res.stdout, res.stdout
