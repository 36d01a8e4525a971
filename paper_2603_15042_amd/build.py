"""Builds libvte.so (HIP kernels + runtime, gfx950) and the input generator, in-tree.

    python -m paper_2603_15042_amd.build [--force] [--trace]

--trace also builds libvte_trace.so: the same library with the matrix-core GEMV (batch 3 to 16)
compiled with device-side time stamps (csrc/trace_stamps.h), for `experiments ramp`.
"""
import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libvte.so")
OUT_TRACE = os.path.join(HERE, "libvte_trace.so")
TRACED = "gemv_mfma.hip"            # the translation unit that carries stamps in the trace build
OBJ = os.path.join(HERE, "_build")

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-inline-asm",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument"]
SOURCES = ["norm_kernels.hip", "gemv_b1.hip", "gemv_b2.hip", "gemv_b4.hip", "gemv_b8.hip", "gemv_b16.hip", "gemv_mfma.hip", "gemv_mfma32.hip", "gemv_mfma64.hip", "gemv_rows.hip",
           "misc_kernels.hip", "noalloc.hip", "gemm_kernel.hip", "backend_hip.cpp", "backend_fake.cpp", "pool.cpp", "planner.cpp",
           "desc.cpp", "runtime.cpp"]


def _newer(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, force, defines=(), tag=""):
    obj = os.path.join(OBJ, src + tag + ".o")
    path = os.path.join(CSRC, src)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(HERE, "..", "include", "vte.h"))
    if not force and not _newer(obj, [path] + headers):
        return obj, ""
    cmd = ["hipcc"] + HIP_FLAGS + ["-D" + d for d in defines] + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    log = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, log))
    return obj, log


def _link(out, objs):
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs + ["-lpthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)


def build(force=False, jobs=None, trace=False):
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    with cf.ThreadPoolExecutor(jobs) as ex:
        results = list(ex.map(lambda s: _compile(s, force), SOURCES))
    objs = [o for o, _ in results]
    for _, log in results:
        if log.strip():
            sys.stderr.write(log + "\n")
    if force or _newer(OUT, objs):
        _link(OUT, objs)
    if trace:
        tobj, log = _compile(TRACED, force, defines=("VTE_TRACE_STAMPS",), tag=".trace")
        if log.strip():
            sys.stderr.write(log + "\n")
        tobjs = [tobj if o.endswith(os.sep + TRACED + ".o") else o for o in objs]
        if force or _newer(OUT_TRACE, tobjs):
            _link(OUT_TRACE, tobjs)
    from . import inputs
    inputs.build(force)
    return OUT


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, trace="--trace" in sys.argv))
