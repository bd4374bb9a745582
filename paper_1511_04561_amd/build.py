"""Builds libdq8.so (HIP kernels + C ABI) for gfx950 next to this file.

hipcc cross-compiles without a GPU.  Flags that matter for the results:
  -ffp-contract=off   the decode-and-average sum rounds product and sum separately;
  no fast-math        divisions are the correctly rounded ones;
  -packed-fp32-ops off (target feature) as required for the test machines.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdq8.so")
SOURCES = ["dq8.hip", "dq8_avg_short.hip", "dq8_avg_long.hip", "dq8_tables.cpp"]
HEADERS = ["dq8_internal.h", "dq8_launch.hpp", "dq8_tables.hpp", "dq8_device.hpp", "dq8_plan.hpp", "dq8_units.hpp", "dq8_arith.hpp", "dq8_kernels_codec.hpp", "dq8_kernels_avg.hpp",
           "dq8_kernels_avg_encode.hpp", "dq8_kernels_stats.hpp", "dq8_kernels_small.hpp", "dq8_kernels_segments.hpp", os.path.join(ROOT, "include", "dq8.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unknown-cuda-version"]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def command(out=LIB, extra=()):
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    return [hipcc()] + FLAGS + list(extra) + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", out] + srcs


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def _compile_and_link(out, extra=(), verbose=False):
    """Every source to an object file, all at once, then one link: the translation units are independent."""
    import shutil
    import tempfile
    tmpdir = tempfile.mkdtemp(prefix="dq8_build_")
    try:
        flags = [f for f in FLAGS if f != "-shared"]
        jobs = []
        for src in SOURCES:
            obj = os.path.join(tmpdir, src + ".o")
            cmd = [hipcc()] + flags + list(extra) + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, src),
                                                    "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            jobs.append((cmd, obj, subprocess.Popen(cmd)))
        for cmd, obj, proc in jobs:
            if proc.wait() != 0:
                for _, _, other in jobs:
                    if other.poll() is None:
                        other.kill()
                raise subprocess.CalledProcessError(proc.returncode, cmd)
        link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + [obj for _, obj, _ in jobs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.check_call(link)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)


def build(force=True, verbose=False, extra=()):
    """Compiles the library; with force=False only when it is missing or older than a source."""
    if not force and not stale():
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    _compile_and_link(tmp, extra, verbose)
    os.replace(tmp, LIB)
    return LIB


def build_tunable(out=None, verbose=False):
    """The same library with changeable launch shapes (-DDQ8_TUNABLE), for experiments: libdq8_tunable.so."""
    out = out or os.path.join(HERE, "libdq8_tunable.so")
    _compile_and_link(out, ["-DDQ8_TUNABLE"], verbose)
    return out


if __name__ == "__main__":
    if sys.argv[1:] == ["--tunable"]:
        print(build_tunable(verbose=True))
    else:
        build(force=True, verbose=True, extra=sys.argv[1:])
        print(LIB)
