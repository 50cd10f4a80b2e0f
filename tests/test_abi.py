"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

from paper_2603_28768_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "craft.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(craft_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_named_calls():
    names = _declared_functions()
    for must in ("craft_expert_load", "craft_plan", "craft_moe_rank_forward"):
        assert must in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_binding_covers_every_declared_symbol():
    assert sorted(binding.EXPORTS) == _declared_functions()


def test_status_strings():
    lib = binding.lib()
    assert lib.craft_status_str(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert lib.craft_status_str(code) not in (b"ok", b"unknown status")
    assert lib.craft_status_str(7) == b"unknown status"
