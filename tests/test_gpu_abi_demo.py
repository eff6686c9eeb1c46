"""The boundary is a C ABI: a plain C program (hipMalloc, no Python, no
PyTorch) linked against libgsgd.so runs pull-gossip SGD on the quadratic and
checks the method's promises itself."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DEMO = os.path.join(ROOT, "paper_1611_04581_amd", "abi_demo")


@pytest.mark.parametrize("block_columns", ["16384", "0"])
def test_plain_c_program_runs_the_path(block_columns):
    """Blocked matrices (the gossip steps run as two ascending sweeps) and row-major ones (walks along the peer map)."""
    assert os.path.exists(DEMO), "abi_demo is not built: run `python -c 'import __graft_entry__ as g; g.build()'`"
    print("running", DEMO, block_columns, flush=True)
    done = subprocess.run([DEMO, block_columns], capture_output=True, text=True, timeout=100)
    print(done.stdout, done.stderr, flush=True)
    assert done.returncode == 0, done.stderr
    assert "abi_demo ok" in done.stdout
