"""The C-ABI library loads and exports every symbol include/dq.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1805_10111_amd", "libdq.so")
HEADER = os.path.join(ROOT, "include", "dq.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dq_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} not built: run python paper_1805_10111_amd/build.py")
    return ctypes.CDLL(LIB)


def test_header_symbols_are_exported(lib):
    names = _declared()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), n


def test_binding_covers_the_header():
    import paper_1805_10111_amd as dq
    assert sorted(dq.EXPORTS) == _declared()
    for n in dq.EXPORTS:
        assert callable(getattr(dq, n)), n
    assert "gfx950" in dq.dq_version()


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_1805_10111_amd as dq
    v = torch.zeros(16)
    with pytest.raises(ValueError):
        dq.dq_absmax(v, torch.zeros(1))
