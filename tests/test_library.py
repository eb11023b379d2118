"""CPU-only: the C-ABI library is built, loads, and exports every declared symbol."""
import ctypes
import os
import re

from paper_2412_04788_amd import guide

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "guide.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(guide_[a-z_]+)\s*\(", text)))


def test_header_symbols_exported():
    names = _declared()
    assert set(names) == set(guide.EXPORTS)
    lib = ctypes.CDLL(guide.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_structs_match_header_sizes():
    assert ctypes.sizeof(guide.CModel) == 32 and ctypes.sizeof(guide.CHw) == 40
    assert ctypes.sizeof(guide.CAxis) == 24 and ctypes.sizeof(guide.CGrid) == 9 * 24
    assert ctypes.sizeof(guide.CSelectSpec) == 4 + 4 + 3 * 8 + 8 + 4 * 16 + 8 + 8
    assert ctypes.sizeof(guide.CSpace) == 12 * 8 + 5 * 4 + 4 + 8
    assert ctypes.sizeof(guide.CExtras) == 5 * 8


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2412_04788_amd", "guide.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")


def test_context_creation_fails_loudly_without_a_gpu():
    import pytest
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(guide.GuideError) as e:
        guide.Context(0)
    assert e.value.code == guide.E_DEVICE
