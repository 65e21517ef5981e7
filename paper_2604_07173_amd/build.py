"""Builds liblora.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "liblora.so")
SOURCES = ["api.hip", "pack.hip", "segments.hip", "segments_large.hip", "shrink.hip", "expand.hip",
           "shrink_decode.hip", "expand_decode.hip", "fused_decode.hip", "combine.hip", "provision.cpp"]
HEADERS = ["lora_internal.h", "lora_layout.h", "lora_device.h", "expand_common.h", "expand_item.h", "shrink_wave.h", "segments_common.h", "segments_inline.h", os.path.join("..", "..", "include", "lora.h"),
           os.path.join("..", "..", "include", "lora_provision.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall"]      # host-only translation units


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False, jobs: int = 7, extra_flags=(), out: str = LIB_PATH) -> str:
    """Compile every translation unit and link the shared library. Always compiles.

    extra_flags / out: a second build of the library next to the installed one, e.g.
    extra_flags=("-DLORA_TUNING",) for a build whose work-split constants can be set from the
    environment during parameter sweeps."""
    cc = hipcc()
    objdir = os.path.join(PKG_DIR, "_build" if out == LIB_PATH else "_build_" + os.path.basename(out))
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        flags = HIPCC_FLAGS if src.endswith(".hip") else HOST_FLAGS
        cmd = [cc, *flags, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    subprocess.check_call(cmd)
    return out


def _drain(procs):
    for src, pr in procs:
        out, _ = pr.communicate()
        text = out.decode(errors="replace")
        # the host pass does not know the target feature and says so; that is harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{text}")
        if text.strip():
            print(text, file=sys.stderr)
    procs.clear()


if __name__ == "__main__":
    if len(sys.argv) > 1 and sys.argv[1] == "--tuning":       # python -m ...build --tuning OUT.so
        print(build(verbose=True, extra_flags=("-DLORA_TUNING",), out=os.path.abspath(sys.argv[2])))
    else:
        print(build(verbose=True))
