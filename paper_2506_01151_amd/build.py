"""Builds the HIP library in-tree: paper_2506_01151_amd/libzapformat.so (gfx950 only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libzapformat.so")
SOURCES = ["zf_regex.cpp", "zf_compile.cpp", "zf_earley.cpp", "zf_automaton.cpp", "zf_api.cpp", "zf_kernels.hip", "zf_mask_walk.hip", "zf_mask_automaton.hip", "zf_mask_store.hip", "zf_scratch.hip"]
HEADERS = ["zf_device.h", "zf_internal.h", "zf_launch.h", "zf_kernel_common.h", "zf_aut_step.h"]


def build(force: bool = True) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS] + [os.path.join(HERE, "..", "include", "zapformat.h")]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-function", "-o", LIB] + srcs
    # hipcc's host pass warns once per translation unit that it does not know the packed-fp32
    # feature (it only applies to the device pass); drop those lines, keep everything else
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if err.strip():
        print(err, file=sys.stderr)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed")
    return LIB


if __name__ == "__main__":
    print(build())
