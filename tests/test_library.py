"""CPU-only: the C-ABI library is built, loads, and exports every declared symbol."""
import ctypes
import os
import re

from paper_2412_04788_amd import guide

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(guide_[a-z_]+)\s*\(", text))
    return sorted(names)


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
    assert ctypes.sizeof(guide.CExtras) == 9 * 8 + 8 + 3 * 8


def test_binding_structs_match_the_c_compiler(tmp_path):
    """sizeof of every struct of the header, as gcc lays it out, against the ctypes mirror."""
    import subprocess
    pairs = [("guide_model", guide.CModel), ("guide_hw", guide.CHw), ("guide_axis", guide.CAxis),
             ("guide_grid", guide.CGrid), ("guide_eff", guide.CEff), ("guide_metrics", guide.CMetrics),
             ("guide_stats", guide.CStats), ("guide_extras", guide.CExtras), ("guide_space", guide.CSpace),
             ("guide_sampled_out", guide.CSampledOut), ("guide_trace", guide.CTrace), ("guide_sim_out", guide.CSimOut),
             ("guide_constraint", guide.CConstraint), ("guide_select_spec", guide.CSelectSpec),
             ("guide_select_out", guide.CSelectOut), ("guide_column_constraint", guide.CColumnConstraint),
             ("guide_column_select", guide.CColumnSelect)]
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include "guide.h"\nint main(void) {\n' +
                   "".join(f'    printf("%zu\\n", sizeof({c}));\n' for c, _ in pairs) + "    return 0;\n}\n")
    exe = tmp_path / "sizes"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert got == [ctypes.sizeof(t) for _, t in pairs], list(zip([c for c, _ in pairs], got))


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
