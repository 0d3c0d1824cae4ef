"""Builds libseesaw_rt.so (HIP kernels + C-ABI runtime) for gfx950 with hipcc.

Run as `python -m paper_2503_06433_amd.build`; the library lands next to this
file so that it travels with the source tree.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libseesaw_rt.so")
HOST_SOURCES = ["ss_runtime.hip", "ss_offline.hip"]
# the kernel files are built twice: brain-float (namespace ssk) and, with SS_HALF_F16, IEEE half (ssk16)
KERNEL_SOURCES = ["k_elementwise.hip", "k_gemm_generic.hip", "k_gemm_mfma.hip", "k_attn_generic.hip", "k_attn_mfma.hip",
                  "k_kv_repack.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src, obj, defines=()):
    cmd = ["hipcc", *FLAGS, *defines, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    return err


def build(verbose=False, jobs=8):
    out_dir = os.path.join(HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    units = [(s, os.path.join(out_dir, s.replace(".hip", ".o")), ()) for s in HOST_SOURCES + KERNEL_SOURCES]
    units += [(s, os.path.join(out_dir, s.replace(".hip", "_f16.o")), ("-DSS_HALF_F16",)) for s in KERNEL_SOURCES]
    objs = [u[1] for u in units]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for (src, _, _), msg in zip(units, ex.map(lambda u: _compile(*u), units)):
            if verbose and msg.strip():
                print(src, msg, file=sys.stderr)
    # the HSA runtime (the one HIP itself runs on) carries the swap-out's device-to-host copies on the DMA engines
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs, "-lpthread", "-L/opt/rocm/lib",
           "-lhsa-runtime64"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
