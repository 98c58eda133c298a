"""Builds libkvp.so (HIP kernels + C-ABI host code) for gfx950 with hipcc.

Usage: ``python -m paper_2604_16734_amd.build``.  The library is written next
to this file; object files go to ``_build/`` at the repository root.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvp.so")
SOURCES = ["attention.hip", "colsum.hip", "rowstat.hip", "keydiff.hip", "decode.hip", "select.hip", "compact.hip", "probe.hip", "plan.cpp", "kvp.cpp"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 arithmetic is kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose=False):
    hipcc = _hipcc()
    obj_dir = os.path.join(ROOT, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    objs = []
    jobs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.rsplit(".", 1)[0] + ".o")
        objs.append(obj)
        cmd = [hipcc] + FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + \
              ["-c", os.path.join(CSRC, src), "-o", obj]
        jobs.append(cmd)
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        for out in ex.map(_run, jobs):
            if verbose and out:
                print(out)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


def build_host_sanitized(out_dir):
    """The host side alone (kvp.cpp and plan.cpp; kernel launchers and HIP runtime calls stubbed) with
    the driver of tests/host_asan, compiled by g++ with the address and undefined-behaviour
    sanitizers.  Returns the path of the executable."""
    rocm_inc = os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(_hipcc()))), "include")
    tests = os.path.join(ROOT, "tests", "host_asan")
    exe = os.path.join(out_dir, "kvp_host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-isystem", rocm_inc,
           os.path.join(CSRC, "kvp.cpp"), os.path.join(CSRC, "plan.cpp"),
           os.path.join(tests, "stubs.cpp"), os.path.join(tests, "driver.cpp"), "-o", exe]
    _run(cmd)
    return exe


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
