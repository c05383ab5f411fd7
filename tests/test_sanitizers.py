"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

Three pieces are compiled with ``-fsanitize=address,undefined``: the C oracle, the host
emulation of the tiled kernel (which includes the launch planner and the index functions
the device code shares), and the host half of the library's API translation unit
(validation, selection table and heuristic, planning, workspace queries, the bounds audit).
The instrumented API object is linked with the library's ordinary kernel objects; a driver
walks the host-only entry points and runs emulated launches against the oracle.  GPU code
is not instrumented (device sanitizers are not available) and no GPU is used.
"""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PKG = os.path.join(ROOT, "paper_1606_00094_amd")
OUT = os.path.join(HERE, "sanitize", "_san")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, "%s\n%s" % (" ".join(cmd), r.stdout[-4000:])
    return r.stdout


@pytest.mark.timeout(900)
def test_host_code_is_clean_under_asan_and_ubsan():
    from paper_1606_00094_amd import build as hip_build
    os.makedirs(OUT, exist_ok=True)
    # the kernel objects the instrumented API object is linked with
    objs = [os.path.join(hip_build.OBJ, o) for _, o, _ in hip_build._units() if o != "bconv_api.o"]
    if not all(os.path.exists(o) for o in objs):
        hip_build.build(force=False)
    # host pass instrumented, device pass untouched: each -fsanitize= follows its own -Xarch_host
    api = os.path.join(OUT, "bconv_api_san.o")
    _run([HIPCC] + hip_build.FLAGS + ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                                       "-Xarch_host", "-fno-sanitize-recover=undefined",
                                       "-c", os.path.join(PKG, "csrc", "bconv_api.hip"), "-o", api])
    emu = os.path.join(OUT, "emu_tconv_san.o")
    _run(["g++", "-std=c++17"] + SAN + ["-c", os.path.join(HERE, "host_emu", "emu_tconv.cpp"), "-o", emu])
    orc = os.path.join(OUT, "conv_oracle_san.o")
    _run(["gcc", "-std=c11", "-fopenmp"] + SAN + ["-c", os.path.join(ROOT, "oracle", "conv_oracle.c"), "-o", orc])
    drv = os.path.join(OUT, "san_driver.o")
    _run(["g++", "-std=c++17"] + SAN + ["-c", os.path.join(HERE, "sanitize", "san_driver.cpp"), "-o", drv])
    exe = os.path.join(OUT, "san_driver")
    _run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fopenmp",
          "-o", exe, drv, api, emu, orc] + objs)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    out = _run([exe], env=env, timeout=600)
    assert "san_driver: ok" in out, out[-4000:]
    assert "runtime error" not in out and "AddressSanitizer" not in out, out[-4000:]
