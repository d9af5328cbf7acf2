"""Builds the C-ABI library libsl.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsl.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU ops out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-result",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built")


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


# Host-side sanitizer build: AddressSanitizer + UndefinedBehaviorSanitizer on the host pass only
# (the validation layer, workspace carving, launch logic); device code is compiled as usual.  The
# result goes to libsl_san.so and is meant for CPU runs of programs that are themselves built with
# the sanitizers (tests/cabi/validate_from_c.c).
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
SAN_LIB = os.path.join(PKG, "libsl_san.so")


def build(verbose: bool = False, extra_flags: list[str] | None = None, sanitize: bool = False) -> str:
    """Compile every kernel translation unit and link libsl.so (sanitize: libsl_san.so). Always recompiles."""
    objs = []
    if sanitize:
        extra_flags = (extra_flags or []) + SAN_FLAGS
    bdir = os.path.join(PKG, "_build_san" if sanitize else "_build")
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for src in sources():
        obj = os.path.join(bdir, os.path.basename(src) + ".o")
        cmd = [hipcc_path()] + [f for f in HIPCC_FLAGS if f != "-shared"] + (extra_flags or []) + [
            "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if pr.returncode != 0:
            failed = True
            print(f"[build] FAILED {src}\n{out}", file=sys.stderr)
        elif verbose and out:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    lib = SAN_LIB if sanitize else LIB
    tmp = lib + ".tmp"
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    if sanitize:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, sanitize="--sanitize" in sys.argv))
