"""Checks on the compiler's listing of the persistent GEMM (CPU only: hipcc cross-compiles gfx950 here).

The kernel issues its ring loads from inline assembly and counts them by hand; the compiler does not know of them, so
any `s_waitcnt vmcnt` it places inside the K loop (in front of a spill reload, or where a register that a load left
pending is written again) also waits for the ring and turns the pipeline into a synchronous one.  The listing is
checked for that, for spills inside the loop, and for the loads' scalar base operand.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2503_06433_amd import build as bld

SRC = os.path.join(bld.CSRC, "k_gemm_mfma.hip")


def _blocks(lines):
    """[(label, [instructions])] of one function's listing"""
    out, name, cur = [], "entry", []
    for l in lines:
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m:
            out.append((name, cur))
            name, cur = m.group(1), []
            continue
        x = l.strip()
        if x and not x.startswith(";") and not x.startswith("."):
            cur.append(x)
    out.append((name, cur))
    return out


@pytest.fixture(scope="module")
def listing(tmp_path_factory):
    if not shutil.which("hipcc"):
        pytest.skip("hipcc not on PATH")
    out = str(tmp_path_factory.mktemp("listing") / "k_gemm_mfma.s")
    r = subprocess.run(["hipcc", *bld.FLAGS, "--cuda-device-only", "-S", SRC, "-o", out], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    with open(out) as f:
        return f.read().split("\n")


def _stream_kernels(lines):
    starts = [i for i, l in enumerate(lines) if re.match(r"^_ZN\w*gemm_mfma_stream_kernel\w*:", l)]
    assert len(starts) >= 4, "expected the four instances of the persistent kernel in the listing"
    for i in starts:
        end = next(j for j in range(i, len(lines)) if "s_endpgm" in lines[j])
        yield lines[i].split(":")[0], lines[i:end]


def test_k_loop_of_the_persistent_gemm_has_no_compiler_wait_on_memory_and_no_spill(listing):
    for name, body in _stream_kernels(listing):
        with_loads, without = [], []
        for label, ins in _blocks(body):
            n_mfma = sum("v_mfma" in x for x in ins)
            if n_mfma < 32:
                continue
            n_dma = sum("global_load_lds_dwordx4" in x for x in ins)
            dirty = [x for x in ins if ("s_waitcnt" in x and "vmcnt" in x) or x.startswith("scratch_")]
            (with_loads if n_dma else without).append((label, dirty))
        assert with_loads and without, name
        # a half-slice that issues ring loads never waits on memory and never touches scratch
        for label, dirty in with_loads:
            assert not dirty, (name, label, dirty)
        # the other half-slice has a steady-state copy that is clean (a peeled first or last copy may wait)
        assert any(not dirty for _, dirty in without), (name, without)


def test_direct_to_lds_loads_take_a_scalar_base(listing):
    loads = [l.strip() for l in listing if "global_load_lds_dword" in l and not l.strip().startswith(";")]
    assert len(loads) > 100
    for l in loads:
        assert re.search(r"global_load_lds_dword(x4)?\s+v\d+,\s+s\[\d+:\d+\]", l), l
