"""Builds libpafu.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc."""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpafu.so")
SOURCES = ["api.hip", "score.hip", "select.hip", "compact.hip", "quant.hip", "attention.hip", "sse.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the attention step is one fully unrolled 32-slot block; above the default threshold the unroller keeps a partial
    # loop, the register arrays get indexed dynamically and spill
    "-mllvm", "-pragma-unroll-threshold=200000",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, extra_flags=(), out: str = "") -> str:
    """Compiles every translation unit and links libpafu.so; always recompiles.

    `out` names another library file next to libpafu.so (study builds with extra -D flags, loaded by name through
    bench.py --library); its objects go to a directory of their own so that the product build is left alone."""
    LIB = os.path.join(HERE, out) if out else globals()["LIB"]
    obj_dir = os.path.join(HERE, "_build" + ("_" + os.path.splitext(out)[0] if out else ""))
    os.makedirs(obj_dir, exist_ok=True)
    cc = hipcc()
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]

    def one(i):
        return _run([cc, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]])

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as ex:
        logs = list(ex.map(one, range(len(SOURCES))))
    logs.append(_run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]))
    if verbose:
        print("\n".join(l for l in logs if l.strip()))
    return LIB


if __name__ == "__main__":
    argv = sys.argv[1:]
    out_name = ""
    if "--out" in argv:
        i = argv.index("--out")
        out_name = argv[i + 1]
        del argv[i:i + 2]
    print(build(verbose=True, extra_flags=argv, out=out_name))
