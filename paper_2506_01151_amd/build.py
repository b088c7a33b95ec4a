"""Builds the HIP library in-tree: paper_2506_01151_amd/libzapformat.so (gfx950 only)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libzapformat.so")
SOURCES = ["zf_regex.cpp", "zf_compile.cpp", "zf_earley.cpp", "zf_automaton.cpp", "zf_api.cpp", "zf_kernels.hip", "zf_mask_walk.hip",
           "zf_mask_automaton.hip", "zf_mask_store.hip", "zf_scratch.hip"]
HEADERS = ["zf_device.h", "zf_internal.h", "zf_launch.h", "zf_kernel_common.h", "zf_aut_step.h", "zf_host_automaton.h"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]
# hipcc's host pass warns once per translation unit that it does not know the packed-fp32
# feature (it only applies to the device pass); those lines are dropped, everything else is shown
NOISE = "'-packed-fp32-ops' is not a recognized feature"


def _run(cmd):
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    err = "\n".join(l for l in proc.stderr.splitlines() if NOISE not in l)
    return proc.returncode, err


SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def build(force: bool = True, extra_flags=(), sanitize: bool = False) -> str:
    """Compile every source to an object (in parallel; with force=False only what is older than its sources) and link.
    sanitize=True builds libzapformat_asan.so instead: the host code of every source under AddressSanitizer and
    UndefinedBehaviorSanitizer (the device code is built as always), for the CPU test suite:
        LD_PRELOAD=$(/opt/rocm/lib/llvm/bin/clang++ -print-file-name=libclang_rt.asan-x86_64.so) ASAN_OPTIONS=detect_leaks=0 \
        ZAPFORMAT_LIBRARY=paper_2506_01151_amd/libzapformat_asan.so python -m pytest tests -m "not gpu" -q"""
    global OBJ, LIB
    if sanitize:
        OBJ, LIB = os.path.join(HERE, "_build", "asan"), os.path.join(HERE, "libzapformat_asan.so")
        force, extra_flags = True, list(extra_flags) + SANITIZE
    os.makedirs(OBJ, exist_ok=True)
    deps = [os.path.join(CSRC, h) for h in HEADERS] + [os.path.join(HERE, "..", "include", "zapformat.h"), os.path.join(HERE, "..", "include", "zapformat_debug.h")]
    newest_dep = max(os.path.getmtime(d) for d in deps)
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s + ".o")
        if force or extra_flags or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_dep):
            jobs.append(["hipcc", "-x", "hip", "-c", src, "-o", obj] + FLAGS + list(extra_flags))
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        results = list(pool.map(_run, jobs))
    failed = False
    for rc, err in results:
        if err.strip():
            print(err, file=sys.stderr)
        failed |= rc != 0
    if failed:
        raise RuntimeError("hipcc failed")
    if jobs or not os.path.exists(LIB):
        link = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libasan"] if sanitize else []
        rc, err = _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + link + [os.path.join(OBJ, s + ".o") for s in SOURCES])
        if err.strip():
            print(err, file=sys.stderr)
        if rc != 0:
            raise RuntimeError("hipcc link failed")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, extra_flags=[a for a in sys.argv[1:] if a.startswith("-D")], sanitize="--sanitize" in sys.argv))
