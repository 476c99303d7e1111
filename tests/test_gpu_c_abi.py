"""The boundary without Python in the way: a plain C program (tests/abi_c_gpu.c, built by
__graft_entry__.build()) allocates with the HIP runtime, inserts a batch through the C ABI, looks it
up again and checks slots, shared duplicates, untouched rows of sensitive tokens and every byte."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_c_gpu.bin")


def test_round_trip_from_plain_c():
    assert os.path.exists(EXE), "run __graft_entry__.build() first: tests/abi_c_gpu.bin is missing"
    run = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(run.stdout, run.stderr, flush=True)
    assert run.returncode == 0, (run.returncode, run.stdout[-2000:], run.stderr[-2000:])
    assert run.stdout.strip().startswith("c abi ok")
