"""Builds libbconv.so (hand-written HIP kernels for gfx950 + the C ABI) in-tree.

Every translation unit is compiled with hipcc for gfx950 only; packed-FP32
instruction selection is switched off for all device code.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbconv.so")
NUM_GROUPS = 24

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _units():
    units = [("bconv_api.hip", "bconv_api.o", []), ("aux_kernels.hip", "aux_kernels.o", []),
             ("fma_conv.hip", "fma_conv.o", []), ("hconv_first.hip", "hconv_first.o", [])]
    for lay in range(3):   # fp16 matrix-core tiles, one unit per activation-layout pair
        units.append(("hconv_mfma.hip", "hconv_mfma_l%d.o" % lay, ["-DHCONV_LAYOUT=%d" % lay]))
    for g in range(NUM_GROUPS):
        units.append(("tconv_instances.hip", "tconv_instances_g%d.o" % g, ["-DBCONV_GROUP=%d" % g]))
    return units


def _deps():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))] + \
           [os.path.join(HERE, "..", "include", "bconv.h")]


def _compile(unit, force):
    src, obj, extra = unit
    srcp, objp = os.path.join(CSRC, src), os.path.join(OBJ, obj)
    if not force and os.path.exists(objp) and \
            os.path.getmtime(objp) >= max(os.path.getmtime(d) for d in _deps()):
        return objp
    cmd = [HIPCC] + FLAGS + extra + ["-c", srcp, "-o", objp]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature name: harmless
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (obj, out))
    if "warning" in out:
        sys.stderr.write(out + "\n")
    return objp


def build(force=True, jobs=6):
    """Compile all HIP sources and link libbconv.so; returns its path."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda u: _compile(u, force), _units()))
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                   check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
