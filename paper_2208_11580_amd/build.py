"""Build libobc.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libobc.so")
OBJDIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes", "-Wno-pass-failed",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_lib(force: bool = False, verbose: bool = False) -> str:
    """Compile every .hip under csrc/ and link libobc.so.  Objects are rebuilt when a source
    or any header is newer (or always with ``force``)."""
    os.makedirs(OBJDIR, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    hdr_time = max(os.path.getmtime(h) for h in headers)
    objs, todo = [], []
    for src in sources():
        obj = os.path.join(OBJDIR, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        stale = force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), hdr_time)
        if stale:
            todo.append((src, obj))
    # at most JOBS compilers at a time, the long ones (the unrolled panel kernels) first
    jobs = max(1, int(os.environ.get("OBC_BUILD_JOBS", min(8, os.cpu_count() or 1))))
    todo.sort(key=lambda so: (0 if "panel_" in os.path.basename(so[0]) else 1, so[0]))
    procs, running = [], []
    for src, obj in todo:
        while len(running) >= jobs:
            running[0].wait()
            running = [r for r in running if r.poll() is None]
        cmd = [HIPCC] + FLAGS + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        log = open(obj + ".log", "wb")
        pr = subprocess.Popen(cmd, stdout=log, stderr=subprocess.STDOUT)
        log.close()
        procs.append((src, pr, obj + ".log"))
        running.append(pr)
    failed = False
    for src, p, logname in procs:
        p.wait()
        with open(logname, "rb") as f:
            out = f.read()
        os.remove(logname)
        text = out.decode(errors="replace")
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write("hipcc failed on %s:\n%s\n" % (src, text))
        elif verbose and text.strip():
            print(text)
    if failed:
        raise RuntimeError("libobc build failed")
    if procs or force or not os.path.exists(LIB):
        tmp = LIB + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(force="--force" in sys.argv, verbose=True))
