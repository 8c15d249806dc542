"""The product path (package + C ABI) must not lean on the oracle, and must fail loudly when the
HIP library is missing instead of falling back to anything on the CPU."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2604_24088_amd")


def product_sources():
    for base, _, files in os.walk(PKG):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                yield os.path.join(base, f)
    yield os.path.join(ROOT, "include", "taco.h")


def test_product_never_references_the_oracle():
    for path in product_sources():
        text = open(path).read()
        assert not re.search(r"^\s*(from|import)\s+oracle|taco_ref|libtaco_ref", text, flags=re.M), path


def test_oracle_never_references_the_product():
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".cpp", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2604_24088_amd" not in text and "hip/" not in text and "taco.h" not in text, f


def test_missing_library_raises(monkeypatch, tmp_path):
    from paper_2604_24088_amd import build, taco
    monkeypatch.setattr(build, "LIB", str(tmp_path / "libtaco_hip.so"))
    monkeypatch.setattr(taco, "_LIB", None)
    with pytest.raises(ImportError):
        taco.lib()
    with pytest.raises(ImportError):
        taco.taco_payload_bytes(1024, 128)
