"""The C ABI driven without PyTorch: a host-only C++ program (tests/c_abi/selftest.cpp)
allocates with hipMalloc (or co2_buffer_set_create), calls libco2.so directly for four consecutive rounds --
through co2_outer_step, co2_outer_step_static or co2_outer_step with the variant switches -- and compares every
element with the oracle source linked into it."""
import importlib.util
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def _exe():
    spec = importlib.util.spec_from_file_location("c_abi_build", os.path.join(HERE, "c_abi", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod.EXE if os.path.exists(mod.EXE) else mod.build_selftest()


@pytest.mark.parametrize("n,K,buffer_set,mode", [
    (100003, 3, 0, 0), (4099, 16, 0, 0), (1 << 20, 8, 0, 0), (1 << 20, 8, 1, 0),
    (100003, 3, 0, 1), (1 << 20, 8, 1, 1),          # the entry point that allocates nothing
    (100003, 3, 0, 2), (4099, 1, 0, 2), (1 << 20, 8, 1, 2),   # all three variant switches
])
def test_c_abi_selftest(n, K, buffer_set, mode):
    out = subprocess.run([_exe(), str(n), str(K), str(buffer_set), str(mode)], capture_output=True, text=True,
                         timeout=120)
    print(out.stdout, out.stderr, flush=True)
    assert out.returncode == 0 and "PASS" in out.stdout
