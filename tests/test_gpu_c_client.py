"""The C ABI without Python or torch in the way: tests/c_abi_client.cpp (built by
__graft_entry__.build()) allocates with hipMalloc, calls la_causal_fwd + la_causal_bwd through
include/la.h and compares with the fp64 oracle, all inside one native process."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

CLIENT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi_client")


@pytest.mark.parametrize("N", [1, 1234, 20000])
def test_native_client_forward_backward(N):
    assert os.path.exists(CLIENT), "build first: python -c 'import __graft_entry__ as g; g.build()'"
    r = subprocess.run([CLIENT, str(N)], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)


def test_operand_split_is_exact_on_the_gpu():
    """tests/split_exact.hip (built by __graft_entry__.build()) runs the kernels' own split3 /
    split2 device functions on 4M values: x = h + m + l exactly, parts shrinking by 2^-8."""
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "split_exact")
    assert os.path.exists(exe), "build first: python -c 'import __graft_entry__ as g; g.build()'"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
