"""Builds tests/native/abi_gpu_check: a plain HIP host program that drives libtidal through its C ABI and
checks it against the oracle library (test infrastructure; needs both libraries built first).

    python -m tests.native.build_native
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "abi_gpu_check")


def build() -> str:
    lib_dir = os.path.join(ROOT, "paper_2503_06421_amd")
    orc_dir = os.path.join(ROOT, "oracle")
    for need in (os.path.join(lib_dir, "libtidal.so"), os.path.join(orc_dir, "libtidal_oracle.so")):
        if not os.path.exists(need):
            raise FileNotFoundError("%s is missing: build it first" % need)
    cmd = ["hipcc", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "include"), os.path.join(HERE, "abi_gpu_check.cpp"),
           "-L", lib_dir, "-l:libtidal.so", "-L", orc_dir, "-l:libtidal_oracle.so",
           "-Wl,-rpath,$ORIGIN/../../paper_2503_06421_amd:$ORIGIN/../../oracle", "-o", EXE]
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed for abi_gpu_check.cpp:\n" + p.stderr[-4000:])
    return EXE


if __name__ == "__main__":
    print("built", build())
