"""Compile the HIP library for gfx950 into paper_2305_18627_amd/libgqsgd.so (in-tree)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgqsgd.so")
SOURCES = [os.path.join(CSRC, f) for f in ("common.hip", "norm.hip", "quantize.hip", "aggregate.hip", "reduce.hip",
                                           "sparse.hip", "pipeline.hip")]
HEADERS = [os.path.join(CSRC, "gq_device.hpp"), os.path.join(CSRC, "gq_host.hpp"),
           os.path.join(ROOT, "include", "gqsgd.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # the rounding decisions are single IEEE binary32 operations: no implicit fusing, exact division
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    # do not form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the packed-fp32 feature and says so; that is harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(force=True, verbose=False):
    """Compile every source (always, unless force=False and the library is newer than its sources),
    the translation units in parallel, then link them into one shared library."""
    if not force and not is_stale():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, os.path.basename(src)[:-4] + ".%d.o" % os.getpid()) for src in SOURCES]
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
            list(ex.map(lambda so: _run([HIPCC] + FLAGS + ["-c", "-o", so[1], so[0]], verbose), zip(SOURCES, objs)))
        tmp = LIB + ".tmp.%d" % os.getpid()
        _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs, verbose)
        os.replace(tmp, LIB)
    finally:
        for o in objs:
            if os.path.exists(o):
                os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
