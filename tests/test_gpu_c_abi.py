"""The C ABI used from plain C: tests/c_abi_check.c allocates with hipMalloc, calls
tuna_alltoallv and the persistent form through include/tuna.h, and compares with the oracle."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "c_abi_check")


@pytest.mark.parametrize("P,radix,rpn", [(12, 3, 0), (16, 2, 4), (40, 40, 0), (1, 2, 0)])
def test_c_program(P, radix, rpn):
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if not os.path.exists(EXE):
        pytest.skip("tests/c_abi_check is not built (run __graft_entry__.build())")
    print("c_abi_check", P, radix, rpn, flush=True)
    out = subprocess.run([EXE, str(P), str(radix), str(rpn)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=100)
    assert out.returncode == 0 and out.stdout.startswith("ok "), out.stdout
