"""Builds libkvcapsule.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvcapsule.so")
SOURCES = ["kvc_api.hip", "kvc_generic.hip", "kvc_fast_decode.hip", "kvc_fast_compress.hip",
           "kvc_full_decode.hip", "kvc_stream_decode.hip"]
# packed-fp32 code generation is switched off on purpose: some packed forms have given
# wrong results on this hardware, so the compiler must not emit them
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # leading scalar / pointer kernel arguments (up to 14 dwords) arrive in registers at wave start
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-function"]


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    inc = os.path.join(HERE, "..", "include")
    deps += [os.path.join(inc, f) for f in os.listdir(inc)]
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source into paper_2605_16439_amd/libkvcapsule.so."""
    if not force and not _stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        # extra compile flags for developer builds (e.g. -DKVC_TIMELINE: in-kernel timestamps)
        extra = os.environ.get("KVC_HIPCC_FLAGS", "").split()
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    for src, p in procs:
        out = p.communicate()[0].decode()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, "\n".join(lines)))
        if lines and verbose:
            print("\n".join(lines))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


PROBES = ["l2_fill_probe.hip", "lds_stride_probe.hip"]


def build_probes() -> list:
    """Compile the standalone measurement aids under csrc/probes/ into paper_2605_16439_amd/probes_bin/."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out_dir = os.path.join(HERE, "probes_bin")
    os.makedirs(out_dir, exist_ok=True)
    outs = []
    for src in PROBES:
        out = os.path.join(out_dir, src.replace(".hip", ""))
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", os.path.join(CSRC, "probes", src), "-o", out]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, r.stdout.decode()))
        outs.append(out)
    return outs


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
    if "--probes" in sys.argv:
        print("\n".join(build_probes()))
