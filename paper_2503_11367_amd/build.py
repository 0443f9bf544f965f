"""Build libmmattn.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2503_11367_amd.build

Every translation unit under csrc/ is compiled for gfx950 only and linked into
one shared library next to this file; nothing is JIT-compiled at import time.
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
LIB = os.path.join(HERE, "libmmattn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC,
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option", "-Wno-inline-asm"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def build_lib(verbose: bool = True, extra=(), out: str = LIB, objdir: str = OBJ) -> str:
    """Compile csrc/*.hip (extra: additional hipcc flags, e.g. -D tile knobs)
    and link them into `out`."""
    os.makedirs(objdir, exist_ok=True)

    def cc(src):
        obj = os.path.join(objdir, src[:-4] + ".o")
        cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        return src, obj, r

    objs = []
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        for src, obj, r in ex.map(cc, sources()):
            msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                             if "packed-fp32-ops" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{msgs}")
            if verbose and msgs.strip():
                print(msgs)
            objs.append(obj)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    if verbose:
        print("built", out)
    return out


if __name__ == "__main__":
    build_lib()
    sys.exit(0)
