"""Builds libdsmoe.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdsmoe.so")
# the same sources with every hand-counted wait replaced by a full wait (what a GPU test compares the library with)
LIB_CHECKED = os.path.join(PKG, "libdsmoe_checked.so")
SOURCES = ["api.hip", "router.hip", "router_stats.hip", "dispatch.hip", "expert_ffn.hip", "decode.hip", "decode_dense.hip", "decode_tiny.hip", "dense.hip", "moa.hip", "moa_bwd.hip",
           "bench_kernels.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True, extra_flags=(), lib_path: str = LIB, obj_dir: str = CSRC, link_flags=()) -> str:
    """Compiles every source for gfx950 and links them into lib_path (default: the in-tree libdsmoe.so).
    obj_dir / lib_path / link_flags let a test build an instrumented copy elsewhere."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"[build] {src} FAILED\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"[build] {src}:\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *link_flags, "-o", lib_path, *objs])
    if verbose:
        sys.stderr.write(f"[build] wrote {lib_path}\n")
    return lib_path


def build_checked(verbose: bool = True) -> str:
    """The conservative-waits build of the same sources (objects under csrc/checked/)."""
    obj_dir = os.path.join(CSRC, "checked")
    os.makedirs(obj_dir, exist_ok=True)
    return build(verbose, extra_flags=("-DDSMOE_CONSERVATIVE_WAITS",), lib_path=LIB_CHECKED, obj_dir=obj_dir)


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
    if not sys.argv[1:]:
        build_checked()
