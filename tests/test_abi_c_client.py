"""The C ABI from a caller written in plain C (tests/abi_client/client.c): the header is valid C, the
library links from C, and on the GPU the client's own checks pass without Python or PyTorch in the process."""
import importlib.util
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _client_build():
    spec = importlib.util.spec_from_file_location("abi_client_build", os.path.join(ROOT, "tests", "abi_client", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_header_is_valid_c99():
    res = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c",
                          os.path.join(ROOT, "include", "taco.h")], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout


def test_c_client_compiles_and_links():
    exe = _client_build().build()
    assert os.access(exe, os.X_OK)


@pytest.mark.gpu
def test_c_client_runs_on_the_gpu():
    exe = _client_build().ensure_built()
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=110)
    print(res.stdout)
    assert res.returncode == 0, res.stdout
    assert "abi_client: ok" in res.stdout
