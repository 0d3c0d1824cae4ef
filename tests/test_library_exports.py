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


def test_stored_form_folds_the_gains_with_one_rounding():
    """The expected bits of the weight inspection tests (gains folded into the matrices behind a norm) on values
    worked out by hand: bf16 keeps 8 significant bits, so (1 + 2^-7)^2 = 1 + 2^-6 + 2^-14 rounds to 1 + 2^-6;
    1.5 * 2 = 3 exactly; rows are scaled by their own gain, the other tensors stay as they are."""
    import numpy as np
    import workloads as wl
    from paper_2503_06433_amd.harness import stored_form
    one_eps = np.float32(1 + 2.0 ** -7)
    bits = lambda a: wl.bf16_bits(np.asarray(a, dtype=np.float32))
    ref = {"g1": bits([one_eps, 2.0]), "g2": bits([1.0, 0.5]),
           "wq": bits([[one_eps, 1.0], [1.5, -3.0]]), "wk": bits([[1.0], [1.0]]), "wv": bits([[0.0], [0.25]]),
           "wo": bits([[7.0, 9.0]]), "wg": bits([[3.0], [3.0]]), "wu": bits([[5.0], [5.0]]), "wd": bits([[11.0, 13.0]])}
    got = stored_form(ref, wl.BF16)
    f = lambda name: wl.bf16_to_f32(got[name])
    assert np.array_equal(f("wq"), np.array([[1 + 2.0 ** -6, one_eps], [3.0, -6.0]], dtype=np.float32))
    assert np.array_equal(f("wk"), np.array([[one_eps], [2.0]], dtype=np.float32))
    assert np.array_equal(f("wv"), np.array([[0.0], [0.5]], dtype=np.float32))
    assert np.array_equal(f("wg"), np.array([[3.0], [1.5]], dtype=np.float32))
    assert np.array_equal(f("wu"), np.array([[5.0], [2.5]], dtype=np.float32))
    for name in ("g1", "g2", "wo", "wd"):
        assert np.array_equal(got[name], ref[name])
    # fp32: one IEEE multiplication
    ref32 = {k: wl.bf16_to_f32(v) * np.float32(1.1) for k, v in ref.items()}
    got32 = stored_form(ref32, wl.F32)
    assert np.array_equal(got32["wq"], (ref32["wq"] * ref32["g1"].reshape(-1, 1)).astype(np.float32))
