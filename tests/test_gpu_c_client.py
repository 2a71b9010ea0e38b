"""The C ABI from plain C: tests/c_client/abi_client.c (C99, adaspark.h and the HIP runtime API only, no Python, no
torch) runs pool, selection, sparse and dense attention on a small seeded problem and checks them against brute-force
loops of its own.  The package's build step compiles it; this test runs it on the GPU and reads its verdict."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

CLIENT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_client", "abi_client")


def test_plain_c_client_runs_the_path():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    assert os.path.exists(CLIENT), "tests/c_client/abi_client is not built: python -m paper_2604_08077_amd.build"
    r = subprocess.run([CLIENT], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert "abi_client: OK" in r.stdout
