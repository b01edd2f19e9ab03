"""The C ABI used from a plain C++ program (no Python, no torch: hipMalloc'd buffers, Alg. 1 through
cdsgd_trainer_*, the formal phase also layer by layer on a stream of its own), checked by that program
bit for bit against the oracle.  The program is tests/native/abi_client.cpp.  (The file's name puts it
near the end of the collection order: it starts a second process on the GPU.)"""
import importlib.util
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


def test_native_client_matches_oracle():
    spec = importlib.util.spec_from_file_location("native_client_build", os.path.join(HERE, "native", "build.py"))
    native_build = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(native_build)
    exe = native_build.ensure_built()
    print("running", exe, flush=True)
    r = subprocess.run([exe, "2106"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=110)
    print(r.stdout[-3000:], flush=True)
    assert r.returncode == 0, r.stdout[-3000:]
    assert "abi client ok" in r.stdout
