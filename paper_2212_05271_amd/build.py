"""Builds libgss.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2212_05271_amd.build            # compile everything, link
    python -m paper_2212_05271_amd.build --if-missing

Object files go to paper_2212_05271_amd/_build/ (git-ignored); the shared library is written next to
this file so it travels with the source tree.
"""

from __future__ import annotations

import argparse
import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgss.so")

ARCH = "gfx950"
# Packed-FP32 VALU instructions are switched off for every kernel of this library.
HIP_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


# Sources that are compiled several times, once per value of a macro, so that their template
# instantiations build in parallel.
MULTI = {
    "gss_em_inst.hip": [(("GSS_INST_D", d), ("GSS_INST_K", k)) for d in range(8, 0, -1) for k in range(8, 0, -1)],
    "gss_large_inst.hip": [(("GSS_INST_K", k),) for k in range(1, 9)],
}


def sources():
    """List of (source path, object name, extra flags), the slowest translation units first."""
    jobs = []
    names = sorted(os.listdir(CSRC), key=lambda n: (n not in MULTI, n))
    for f in names:
        if not f.endswith(".hip"):
            continue
        src = os.path.join(CSRC, f)
        if f in MULTI:
            for macros in MULTI[f]:
                tag = ".".join(f"{m}_{v}" for m, v in macros)
                jobs.append((src, f"{f}.{tag}.o", [f"-D{m}={v}" for m, v in macros]))
        else:
            jobs.append((src, f + ".o", []))
    return jobs


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(job, extra):
    src, objname, flags = job
    obj = os.path.join(BUILD, objname)
    cmd = [_hipcc(), *HIP_FLAGS, *flags, *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    return obj, warn


def build(verbose=True, jobs=None, extra=()):
    os.makedirs(BUILD, exist_ok=True)
    srcs = sources()
    jobs = jobs or min(8, len(srcs))
    for f in os.listdir(BUILD):
        if f.endswith('.o'):
            os.remove(os.path.join(BUILD, f))
    objs = []
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        for obj, warn in ex.map(lambda s: _compile(s, list(extra)), srcs):
            objs.append(obj)
            if verbose and warn:
                print(warn, file=sys.stderr)
    cmd = [_hipcc(), "-shared", "-fPIC", f"--offload-arch={ARCH}", "-fno-gpu-rdc", *objs, "-o", LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--if-missing", action="store_true")
    ap.add_argument("-j", type=int, default=None)
    a = ap.parse_args()
    if a.if_missing and os.path.exists(LIB):
        print(f"{LIB} exists")
        return
    build(jobs=a.j)


if __name__ == "__main__":
    main()
