"""Builds libtjnvfp4.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtjnvfp4.so")
# (source, object name, extra flags): the product kernel's instantiations are compiled in twelve slices, in parallel
SOURCES = [("api.hip", "api.o", []), ("quant.hip", "quant.o", []), ("osci.hip", "osci.o", []), ("hp.hip", "hp.o", []), ("gemm.hip", "gemm.o", [])] + [
    ("gemm_inst.hip", "gemm_inst_ps%d_out%d_outer%d.o" % (ps, out, outer),
     ["-DTJ_GEMM_PS=%d" % ps, "-DTJ_GEMM_OUT=%d" % out, "-DTJ_GEMM_OUTER=%d" % outer])
    for outer in (0, 1) for ps in (1, 0) for out in (0, 2, 1)]
HEADERS = ["device_fmt.h", "internal.h", "gemm_args.h", "gemm_kernel.h", os.path.join("..", "..", "include", "tjnvfp4.h")]

# -ffp-contract=off: the quantizer arithmetic is one IEEE rounding per written operation.
# packed-fp32-ops is switched off: hipcc then never forms v_pk_{add,mul,fma}_f32 on its own.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every .hip file and link the shared library.  Raises on failure."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    headers = [os.path.join(CSRC, h) for h in HEADERS]
    jobs = []
    for s, o, extra in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(objdir, o)
        if force or _stale(obj, [src] + headers):
            jobs.append((src, obj, extra))

    def compile_one(job):
        src, obj, extra = job
        cmd = [hipcc] + FLAGS + extra + ["-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        if verbose and r.stderr:
            sys.stderr.write(r.stderr)
        return obj

    workers = max(1, min(len(jobs), os.cpu_count() or 4, 8))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(compile_one, jobs))
    objs = [os.path.join(objdir, o) for _, o, _ in SOURCES]
    if jobs or not os.path.exists(LIB):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
