"""Build the gfx950 shared library ``libtwa.so`` in-tree with hipcc (no JIT, no torch extension)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtwa.so")
SOURCES = ["twa_api.hip", "twa_project.hip", "twa_expand.hip", "twa_quantize.hip", "twa_basis.hip", "twa_layers.hip", "twa_centre.hip", "twa_minmax.hip"]
HEADERS = ["twa_device.h", "twa_host.h", os.path.join("..", "..", "include", "twa.h")]
# -packed-fp32-ops: keep the compiler from forming packed fp32 instructions
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False, jobs: int = 5) -> str:
    """Compile every HIP source for gfx950 and link ``libtwa.so``.  Returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hdrs = [os.path.normpath(os.path.join(CSRC, h)) for h in HEADERS]
    procs, objs = [], []

    def running():
        return [p for _, p, _ in procs if p.poll() is None]

    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(o)
        if force or _stale(o, [s] + hdrs):
            cmd = [hipcc] + FLAGS + ["-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), flush=True)
            # the compiler's output goes to a file: a pipe nobody reads while waiting can fill up and block it
            log = open(o + ".log", "w+")
            procs.append((src, subprocess.Popen(cmd, stdout=log, stderr=subprocess.STDOUT, text=True), log))
            while len(running()) >= jobs:
                running()[0].wait()
    for src, p, log in procs:
        p.wait()
        log.seek(0)
        out = log.read()
        log.close()
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError(f"hipcc failed on {src}")
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
