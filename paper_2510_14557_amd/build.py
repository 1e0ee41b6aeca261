"""Build libmxp.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmxp.so")
PROBE_DIR = os.path.join(HERE, "probe")
PROBE_LIB = os.path.join(PROBE_DIR, "libmxp_probe.so")      # bench-only measurement aid, not part of the product ABI
SOURCES = ["mxp_quantize.hip", "mxp_convert.hip", "mxp_gemm.hip", "mxp_w4a16.hip", "mxp_wide.hip"]
HEADERS = [os.path.join(CSRC, "mxp_common.h"), os.path.join(CSRC, "mxp_decode.h"), os.path.join(ROOT, "include", "mxp.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def up_to_date():
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS + [os.path.abspath(__file__)]
    if not os.path.exists(PROBE_LIB):
        return False
    tp = os.path.getmtime(PROBE_LIB)
    pdeps = [os.path.join(PROBE_DIR, f) for f in ("mxp_probe.hip", "mxp_probe.h")] + HEADERS
    return all(os.path.getmtime(d) <= t for d in deps) and all(os.path.getmtime(d) <= tp for d in pdeps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and up_to_date():
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for s in SOURCES:
        o = os.path.join(objdir, s.replace(".hip", ".o"))
        objs.append(o)
        cmd = [_hipcc()] + FLAGS + ["-c", os.path.join(CSRC, s), "-o", o]
        if verbose:
            print(" ".join(cmd))
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    pcmd = [_hipcc()] + FLAGS + ["-I" + PROBE_DIR, "-shared", os.path.join(PROBE_DIR, "mxp_probe.hip"), "-o", PROBE_LIB]
    procs.append(("mxp_probe.hip", subprocess.Popen(pcmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (s, out))
        if out.strip() and verbose:
            print(out)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
