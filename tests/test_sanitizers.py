"""CPU sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer): the oracle's C code, and the
host side of libobc compiled without any device code.  GPU code is never built or run under a
sanitizer."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="3")
ENV.pop("LD_PRELOAD", None)


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, "%s\n%s\n%s" % (" ".join(cmd), r.stdout[-3000:], r.stderr[-3000:])
    return r


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-std=c11", "-fopenmp"] + SAN + ["-o", exe, os.path.join(ROOT, "oracle", "obc_oracle.c"),
                                                   os.path.join(ROOT, "tests", "sanitize", "oracle_main.c"), "-lm"])
    r = _run([exe], env=ENV)
    assert "oracle sanitizer run clean" in r.stdout


def test_libobc_host_side_under_address_and_ub_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    csrc = os.path.join(ROOT, "paper_2208_11580_amd", "csrc")
    objs, procs = [], []
    for src in sorted(glob.glob(os.path.join(csrc, "*.hip"))):
        obj = str(tmp_path / (os.path.basename(src)[:-4] + ".o"))
        objs.append(obj)
        # host pass only: no device code is generated, so nothing here can run on a GPU
        procs.append((src, subprocess.Popen([hipcc, "--offload-host-only", "-std=c++17", "-fPIC"] + SAN + ["-c", src, "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, "%s\n%s" % (src, out[-3000:])
    # every object refers to the device image the full build would embed next to it: stand-ins with
    # no code object in them (the runtime finds no kernel there, and none is launched)
    undef = set()
    for obj in objs:
        for ln in _run(["nm", "-u", obj]).stdout.split():
            if ln.startswith("__hip_fatbin_"):
                undef.add(ln)
    stub = str(tmp_path / "fatbin_stubs.c")
    with open(stub, "w") as f:
        for name in sorted(undef):
            f.write("const unsigned char %s[64] __attribute__((aligned(4096))) = {0};\n" % name)
    lib = str(tmp_path / "libobc_host.so")
    _run([hipcc, "--offload-host-only", "-shared", "-fPIC"] + SAN + ["-o", lib] + objs + ["-x", "c", stub])
    exe = str(tmp_path / "abi_host_san")
    # the driver is plain C++: the same clang, without hipcc's HIP mode
    clangxx = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clangxx):
        clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    _run([clangxx, "-std=c++17"] + SAN +
         ["-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "sanitize", "abi_host_main.cpp"),
          "-o", exe, "-L", str(tmp_path), "-lobc_host", "-Wl,-rpath," + str(tmp_path)])
    r = _run([exe], env=ENV)
    assert "libobc host sanitizer run clean" in r.stdout
