"""Builds librainfusion.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librainfusion.so")
SOURCES = ["rf_api.cpp", "rf_plan.cpp", "rf_attn.hip", "rf_arm.hip"]
HEADERS = ["rf_internal.h", "rf_device.h"]


def hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def compile_flags(extra_flags=()):
    # -Wno-inline-asm: the tile loads of rf_attn.hip set M0 in inline assembly and say so in their
    # clobber list, which clang flags because M0 is a reserved register; tests/test_build_checks.py
    # verifies on the generated assembly that nothing else in that file uses M0.
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"),
            "-I", CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
            "-Wno-unused-command-line-argument", "-Wno-inline-asm"] + list(extra_flags)


def device_assembly(source, extra_flags=()):
    """gfx950 assembly text of one HIP source, compiled with the library's flags."""
    cmd = [hipcc()] + compile_flags(extra_flags) + ["--cuda-device-only", "-S", os.path.join(CSRC, source), "-o", "-"]
    return subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True).stdout


def build_library(verbose=False, extra_flags=(), out=LIB):
    """Compile every source for gfx950 and link the shared library. Always rebuilds."""
    objs = []
    flags = compile_flags(extra_flags)
    procs = []
    for s in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        procs.append((s, subprocess.Popen([hipcc()] + flags + ["-c", os.path.join(CSRC, s), "-o", obj],
                                          stderr=subprocess.PIPE, text=True)))
    for s, p in procs:
        _, err = p.communicate()
        err = "\n".join(l for l in err.splitlines() if "not a recognized feature" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (s, err))
        if verbose and err.strip():
            sys.stderr.write(err + "\n")
    tmp = out + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
