"""The C ABI used from plain C: csrc/abi_check.c (built by build.py as `abi_check`) allocates with the
HIP runtime, calls the library and checks two closed forms. No Python objects cross the boundary."""
import os
import subprocess

import pytest

import paper_2404_11912_amd as tf

pytestmark = pytest.mark.gpu


def test_plain_c_client_of_the_abi():
    exe = os.path.join(os.path.dirname(tf.LIB_PATH), "abi_check")
    if not os.path.exists(exe):
        pytest.fail("abi_check has not been built (python -m paper_2404_11912_amd.build)")
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    print(res.stdout, flush=True)
    assert res.returncode == 0, res.stdout
