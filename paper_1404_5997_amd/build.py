"""Builds libowt.so (HIP, gfx950 only) in-tree with hipcc.

The implicit-GEMM kernels are instantiated once per (pass, storage type) in
separate objects so the six compile in parallel.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libowt.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 VALU forms are switched off on purpose (they have misbehaved on the test machines)
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _units():
    units = [("owt_api.o", "owt_api.hip", []), ("owt_pool.o", "owt_pool.hip", []), ("owt_update.o", "owt_update.hip", [])]
    for ps, pname in ((0, "fwd"), (1, "data"), (2, "filter")):
        for bf in (0, 1):
            units.append(("igemm_%s_%s.o" % (pname, "bf16" if bf else "f32"), "igemm_inst.hip",
                          ["-DOWT_INST_PASS=%d" % ps, "-DOWT_INST_BF16=%d" % bf]))
    for ps, pname in ((0, "fwd"), (1, "data")):
        for bf in (0, 1):
            units.append(("dconv_%s_%s.o" % (pname, "bf16" if bf else "f32"), "dconv_inst.hip",
                          ["-DOWT_INST_PASS=%d" % ps, "-DOWT_INST_BF16=%d" % bf]))
    for ps, pname in ((0, "fwd"), (1, "data")):
        units.append(("dconv16_%s.o" % pname, "dconv_bf16_inst.hip", ["-DOWT_INST_PASS=%d" % ps]))
    units.append(("fcgemm.o", "fcgemm_inst.hip", []))
    units.append(("dfilter2.o", "dfilter2_inst.hip", []))
    units.append(("dfilter16.o", "dfilter_bf16_inst.hip", []))
    units.append(("dfilter16b.o", "dfilter16b_inst.hip", []))
    units.append(("sconv16.o", "sconv_bf16_inst.hip", []))
    units.append(("sfilter16.o", "sfilter_bf16_inst.hip", []))
    for bf in (0, 1):
        units.append(("sconv_%s.o" % ("bf16" if bf else "f32"), "sconv_inst.hip", ["-DOWT_INST_BF16=%d" % bf]))
    for bf in (0, 1):
        units.append(("sfilter_%s.o" % ("bf16" if bf else "f32"), "sfilter_inst.hip", ["-DOWT_INST_BF16=%d" % bf]))
    for bf in (0, 1):
        units.append(("dfilter_%s.o" % ("bf16" if bf else "f32"), "dfilter_inst.hip", ["-DOWT_INST_BF16=%d" % bf]))
    return units


def _compile(unit):
    obj, src, defs = unit
    cmd = [HIPCC] + FLAGS + defs + ["-c", os.path.join(CSRC, src), "-o", os.path.join(BUILD, obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s\n%s" % (" ".join(cmd), r.stdout, r.stderr))
    return r.stderr


def build_lib(jobs=8, verbose=False):
    os.makedirs(BUILD, exist_ok=True)
    units = _units()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        logs = list(ex.map(_compile, units))
    if verbose:
        for u, l in zip(units, logs):
            if l.strip():
                print(u[0], l)
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + \
          [os.path.join(BUILD, u[0]) for u in units]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
