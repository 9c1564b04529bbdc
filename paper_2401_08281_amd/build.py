"""Builds libvs.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvs.so")
# the benchmark's calibration kernels (read stream, matrix-core loop, named copy): a library of
# their own, so that libvs.so exports the search boundary and nothing else
CALIBRATE_LIB = os.path.join(HERE, "libvs_calibrate.so")
CALIBRATE_SOURCE = "calibrate.hip"
SOURCES = ["api.hip", "kernels_dist.hip", "kernels_select.hip", "kernels_ivfpq.hip", "kernels_mfma.hip",
           "kernels_refine.hip", "kernels_train.hip",
           "kernels_ivfflat.hip", "kernels_place.hip"]
HEADERS = ["common.hpp", "internal.hpp", os.path.join("..", "..", "include", "vs.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fvisibility=hidden",
    # packed-fp32 instructions are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def lib_path():
    return LIB


def calibrate_lib_path():
    return CALIBRATE_LIB


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return any(os.path.getmtime(p) > t for p in deps)


def build_calibrate_lib(verbose=False):
    """Compiles and links libvs_calibrate.so (one translation unit)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-shared", os.path.join(CSRC, CALIBRATE_SOURCE), "-o", CALIBRATE_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    _drain([(cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT))])
    return CALIBRATE_LIB


def build_lib(verbose=False, jobs=4, extra_flags=(), out=None, tag=""):
    """Compiles every translation unit and links libvs.so.  Always rebuilds.
    extra_flags / out / tag produce a differently-flagged variant next to it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs, procs = [], []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", tag + ".o"))
        cmd = [hipcc] + FLAGS + list(extra_flags) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    target = out or LIB
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", target] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    if out is None and not tag:
        build_calibrate_lib(verbose)
    return target


def _drain(procs):
    while procs:
        cmd, p = procs.pop(0)
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        # hipcc's host pass does not know the packed-fp32 target feature: harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), text))
        if text:
            print(text, flush=True)


if __name__ == "__main__":
    build_lib(verbose=True)
    print(LIB)
