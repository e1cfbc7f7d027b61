"""Builds libfscnn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree, and beside it
libfscnn_bench_probe.so, the measurement helper that only bench.py loads.

    python -m paper_2212_08815_amd.build [--force] [--sanitize-host]

--sanitize-host builds a second copy, libfscnn_hostsan.so, whose HOST code (argument checks,
handles, plans: everything that is not a kernel) is instrumented with AddressSanitizer and
UndefinedBehaviorSanitizer; tests/README_sanitize.txt says how the tests run against it.

hipcc cross-compiles without a GPU.  Objects go to _build/ (not committed), the
shared library next to this file so that it travels with the source tree.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libfscnn.so")
SOURCES = ["api.hip", "compress.hip", "conv_sf.hip", "conv_si.hip", "transpose.hip"]
PROBE_LIB = os.path.join(HERE, "libfscnn_bench_probe.so")
PROBE_SRC = os.path.join(CSRC, "bench_probe.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         # packed-fp32 forms are switched off for every device function of the library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _newer(target, deps):
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(d) <= t for d in deps)


def _compile(src, obj, extra):
    cmd = [HIPCC] + FLAGS + extra + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    return src, r.returncode, r.stdout + r.stderr


SAN_LIB = os.path.join(HERE, "libfscnn_hostsan.so")
# each -fsanitize= directly behind -Xarch_host: device code is never instrumented
SAN_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def build_host_sanitized(verbose=True):
    """libfscnn_hostsan.so: the library with its host code under ASan + UBSan."""
    objdir = os.path.join(OBJDIR, "hostsan")
    os.makedirs(objdir, exist_ok=True)
    objs = []
    for s in SOURCES:
        obj = os.path.join(objdir, s.replace(".hip", ".o"))
        objs.append(obj)
        src, rc, out = _compile(os.path.join(CSRC, s), obj, SAN_FLAGS)
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if verbose and out.strip():
            print(out)
        if rc != 0:
            raise RuntimeError("hipcc failed on %s" % src)
    subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=address",
                           "-fsanitize=undefined", "-shared-libsan", "-o", SAN_LIB] + objs)
    return SAN_LIB


def build(force=False, extra_flags=(), verbose=True):
    os.makedirs(OBJDIR, exist_ok=True)
    headers = [os.path.join(CSRC, "internal.h"), os.path.join(CSRC, "lds_dma.h"),
               os.path.join(ROOT, "include", "fscnn.h"),
               os.path.abspath(__file__)]
    jobs, objs = [], []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJDIR, s.replace(".hip", ".o"))
        objs.append(obj)
        if force or not _newer(obj, [src] + headers):
            jobs.append((src, obj))
    if jobs:
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
            for src, rc, out in ex.map(lambda j: _compile(j[0], j[1], list(extra_flags)), jobs):
                # the host pass does not know the packed-fp32 feature name; that warning is harmless
                out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
                if verbose and out.strip():
                    print(out)
                if rc != 0:
                    raise RuntimeError("hipcc failed on %s" % src)
    if jobs or force or not _newer(LIB, objs):
        tmp = LIB + ".tmp%d" % os.getpid()
        subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
        os.replace(tmp, LIB)
    if force or not _newer(PROBE_LIB, [PROBE_SRC, os.path.abspath(__file__)]):
        tmp = PROBE_LIB + ".tmp%d" % os.getpid()
        r = subprocess.run([HIPCC] + FLAGS + ["-shared", "-o", tmp, PROBE_SRC], capture_output=True, text=True)
        if r.returncode != 0:
            print(r.stdout + r.stderr)
            raise RuntimeError("hipcc failed on %s" % PROBE_SRC)
        os.replace(tmp, PROBE_LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
    if "--sanitize-host" in sys.argv:
        print(build_host_sanitized())
