"""The C-ABI library loads on a machine without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

from paper_1711_07227_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lcrwmd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lcrwmd_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert "lcrwmd_phase1_mindist" in names and "lcrwmd_phase2_spmm" in names and "lcrwmd_rwmd" in names
    lib = ctypes.CDLL(str(binding.LIB_PATH))
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in lcrwmd.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_struct_layouts_match_header():
    # int64 x3 + 4 pointers; pointer + int64 x3 + enum (padded); int x2 + int64 x2
    assert ctypes.sizeof(binding.CsrStruct) == 56
    assert ctypes.sizeof(binding.EmbStruct) == 40
    assert ctypes.sizeof(binding.OptionsStruct) == 32
    assert ctypes.sizeof(binding.ProfileStruct) == 152


def test_no_oracle_in_product_path():
    """Nothing in the package may import or call the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_1711_07227_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "rwmd_oracle" not in src
