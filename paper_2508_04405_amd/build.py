"""Compile the HIP sources in csrc/ for gfx950 into two libraries next to this file:

libflexq.so      the product: the C ABI of include/flexq.h and nothing else;
libflexq_dev.so  the same sources compiled with FLEXQ_DEV plus the development entry
                 points of include/flexq_dev.h (per-call kernel overrides, ablation
                 variants, probes): test and measurement infrastructure.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libflexq.so")
DEV_LIB = os.path.join(HERE, "libflexq_dev.so")
SOURCES = ["quant_pack.hip", "producers.hip", "skinny.hip", "gemm.hip", "gemm_wlds.hip", "layer.hip", "noalloc.hip",
           "api.hip"]
DEV_SOURCES = SOURCES + ["probes.hip", "dev_api.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def sources_newer_than(lib):
    """True if `lib` is missing or older than any source it is built from."""
    if not os.path.exists(lib):
        return True
    built = os.path.getmtime(lib)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h"))]
    deps += [os.path.join(HERE, "..", "include", f) for f in ("flexq.h", "flexq_dev.h")]
    deps.append(os.path.abspath(__file__))
    return any(os.path.getmtime(d) > built for d in deps)


def build(verbose=False, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = []
    for lib, sources, defs, tag in ((LIB, SOURCES, [], ""), (DEV_LIB, DEV_SOURCES, ["-DFLEXQ_DEV"], ".dev")):
        objs = []
        for src in sources:
            obj = os.path.join(CSRC, src.replace(".hip", tag + ".o"))
            cmd = [hipcc, *FLAGS, *defs, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
            jobs.append(cmd)
            objs.append(obj)
        jobs.append(("link", lib, objs))
    compiles = [j for j in jobs if isinstance(j, list)]
    limit = max(1, min(16, os.cpu_count() or 1))
    running, failed = [], None
    queue = list(compiles)
    while queue or running:
        while queue and len(running) < limit:
            cmd = queue.pop(0)
            running.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        cmd, p = running.pop(0)
        out = p.communicate()[0].decode()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0 and failed is None:
            failed = "hipcc failed: " + " ".join(cmd) + "\n" + "\n".join(lines)
        if verbose and lines:
            print("\n".join(lines))
    if failed:
        raise RuntimeError(failed)
    for j in jobs:
        if not isinstance(j, list):
            _, lib, objs = j
            subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, extra=tuple(sys.argv[1:])))
