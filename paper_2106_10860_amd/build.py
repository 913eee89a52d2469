"""Builds libmaddness.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmaddness.so")
# a copy kernel of known traffic for bandwidth calibration, a library of its own (not part of the method)
CALIB_LIB = os.path.join(HERE, "libmaddness_calib.so")
CALIB_SOURCE = os.path.join("calib", "stream_copy.hip")
SOURCES = ["api.hip", "encode_scan.hip", "fused_rows.hip", "encode_cols.hip", "mfma_scan.hip", "fused_mfma.hip", "build_luts.hip",
           "learn.hip"]
# the learner's sums must round as written (a * b + c stays two operations): its split decisions are
# compared bit for bit with a CPU statement of the same algorithms
FILE_FLAGS = {"learn.hip": ["-ffp-contract=off"]}

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # the table-scan text writes M0 (base of ds_read_addtid) and says so in its clobber list;
    # the compiler only ever sets M0 itself right before an instruction that reads it
    "-Wno-inline-asm",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = False, extra_flags=(), out: str = LIB, jobs: int = 0) -> str:
    """Compiles every source (in parallel, one hipcc per file) and links the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(len(SOURCES), os.cpu_count() or 1, 8)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="maddness_build_") as tmp:
        def compile_one(src: str) -> str:
            obj = os.path.join(tmp, src + ".o")
            cmd = [hipcc, *compile_flags, *FILE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
            return obj
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.check_call(link)
        if out == LIB:
            calib = [hipcc, *FLAGS, os.path.join(CSRC, CALIB_SOURCE), "-o", CALIB_LIB]
            if verbose:
                print(" ".join(calib), flush=True)
            subprocess.check_call(calib)
    return out


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
