"""CPU-only checks of the boundary: the built library loads and exports every entry point the
header declares (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "agzo.h")
LIB = os.path.join(ROOT, "paper_2601_17261_amd", "libagzo.so")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(agzo_[a-z0-9_]+)\s*\(", src)))


def test_header_declares_the_five_hot_path_calls():
    names = _declared()
    for want in ("agzo_layer_forward_sketch", "agzo_basis", "agzo_perturbed_forward", "agzo_update", "agzo_step"):
        assert want in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail("libagzo.so is not built; run python -m paper_2601_17261_amd.build")
    lib = ctypes.CDLL(LIB)
    for name in _declared():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_entry_points():
    from paper_2601_17261_amd import binding
    assert sorted(binding.EXPORTS) == _declared()
    lib = binding.load()
    for name in binding.EXPORTS:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_header_sizes():
    from paper_2601_17261_amd import binding
    assert ctypes.sizeof(binding.AgzoLayer) == 3 * 8 + 4 * 4 + 3 * 8
    assert ctypes.sizeof(binding.AgzoLossSpec) == 4 + 4 + 8 + 8


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2601_17261_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
