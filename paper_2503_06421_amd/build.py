"""Build libtidal.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2503_06421_amd.build [--force] [--tuning]

--tuning builds a second library, libtidal_tuning.so, that reads walk lengths and kernel variants
from TIDAL_MFMA_* / TIDAL_APPLY_* environment variables (sweeps); the default library ignores the
environment.

hipcc cross-compiles without a GPU.  Objects go to paper_2503_06421_amd/_build/ (ignored by
git), the library next to this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtidal.so")

SOURCES = ["tidal.cpp", "tidal_lora.cpp", "tidal_apply.cpp", "plan.cpp", "convert_kernels.hip", "lora_kernels.hip", "lora_lds_kernel.hip",
           "lora_apply_kernels.hip", "convert_merge_kernel.hip"]
# per-file extras: the LDS swap kernel wants its MFMA results in VGPRs (see the file's header)
EXTRA_FLAGS = {"lora_lds_kernel.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}
HEADERS = [os.path.join(ROOT, "include", "tidal.h"), os.path.join(CSRC, "tidal_internal.h"), os.path.join(CSRC, "tidal_host.h"),
           os.path.join(CSRC, "plan.h"), os.path.join(CSRC, "lora_device.h"), os.path.join(CSRC, "host_trace.h")]

# -packed-fp32-ops off: packed fp32 VALU forms are not to be generated on this target.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


TUNING_LIB = os.path.join(HERE, "libtidal_tuning.so")


def _compile(src: str, force: bool, tuning: bool = False) -> str:
    obj = os.path.join(OBJ + ("_tuning" if tuning else ""), os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path, *HEADERS]):
        extra = ["-DTIDAL_TUNING_KNOBS"] if tuning else []
        cmd = ["hipcc", *FLAGS, *extra, *EXTRA_FLAGS.get(src, []), "-c", path, "-o", obj]
        p = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass does not know the gfx feature name and says so; that is expected
        err = "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
        if err.strip():
            sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False, verbose: bool = False, tuning: bool = False) -> str:
    LIB = TUNING_LIB if tuning else globals()["LIB"]
    os.makedirs(OBJ + ("_tuning" if tuning else ""), exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, tuning), SOURCES))
    if force or _stale(LIB, objs):
        tmp = LIB + ".tmp%d" % os.getpid()
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", tmp, *objs]
        p = subprocess.run(cmd, capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError("link failed:\n" + p.stderr)
        os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv, verbose=True, tuning="--tuning" in sys.argv)
