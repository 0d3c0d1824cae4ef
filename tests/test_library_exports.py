"""The C-ABI library builds, loads, and exports every entry point that
include/seesaw_rt.h declares (no compute calls: CPU only)."""
import ctypes
import os
import re

import paper_2503_06433_amd as ss
from paper_2503_06433_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "seesaw_rt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z_0-9]+)\s*\(", text)))


def _library():
    if not os.path.exists(ss.library_path()):
        from paper_2503_06433_amd.build import build
        build()
    return ss.load_library()


def test_header_declares_the_four_calls_of_the_boundary():
    names = _declared()
    for must in ("ss_layer_prefill", "ss_layer_decode", "ss_kv_reshard", "ss_kv_swap"):
        assert must in names


def test_every_declared_symbol_is_exported_and_bound():
    lib = _library()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
        assert isinstance(getattr(lib, n), ctypes._CFuncPtr)
    assert sorted(binding.EXPORTED) == names


def test_no_torch_types_in_the_boundary():
    text = open(os.path.join(ROOT, "include", "seesaw_rt.h")).read()
    assert "torch" not in text and "at::" not in text and "#include <hip" not in text


def test_struct_sizes_match_the_header_layout():
    assert ctypes.sizeof(ss.ModelCfg) == 11 * 4
    assert ctypes.sizeof(ss.RuntimeCfg) == 3 * 8 + 2 * 4
    assert ctypes.sizeof(ss.ShardDesc) == 5 * 4
