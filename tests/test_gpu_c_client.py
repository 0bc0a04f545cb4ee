"""The C ABI used from plain C on the GPU: tests/c_abi_gpu_client.c (HIP runtime + the library +
the oracle, no Python in the loop) must report the state bit-identical to the oracle's."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi_gpu_client")


@pytest.mark.parametrize("n", [1_000_003, 257, 20_000_001])
def test_plain_c_program_matches_the_oracle(n):
    if not os.path.exists(EXE):
        import __graft_entry__
        __graft_entry__.build_c_gpu_client()
    run = subprocess.run([EXE, str(n)], capture_output=True, text=True, timeout=110)
    assert run.returncode == 0, (run.stdout, run.stderr[-1000:])
    lines = run.stdout.strip().splitlines()
    first = dict(zip(lines[0].split()[::2], lines[0].split()[1::2]))
    assert first["flag"] == "0" and first["state_bit_identical"] == "1", run.stdout
    assert float(first["sqnorm_rel_err"]) <= 1e-5
    if n <= 5_000_000:                      # far below any device's limit for the one-launch step
        small = dict(zip(lines[1].split()[1::2], lines[1].split()[2::2]))
        assert small["flag"] == "0" and small["state_bit_identical"] == "1", run.stdout
        assert float(small["sqnorm_rel_err"]) <= 1e-5
    else:
        assert lines[1].startswith("small_block skipped"), run.stdout
    assert lines[2] == "overflow_flag 1 untouched 1", run.stdout
