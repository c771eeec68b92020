"""Compile the HIP library for gfx950 into paper_2605_00539_amd/libagoq.so.

hipcc cross-compiles without a GPU.  Flags: no FMA contraction and no fast-math (the
arithmetic contract is bit-exact IEEE binary32), packed-fp32 instruction selection off.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libagoq.so")
SOURCES = [os.path.join(CSRC, name) for name in
           ("agoq_act.hip", "agoq_grad.hip", "agoq_recompute.hip", "agoq_probe.hip", "agoq_host.cpp")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"),
]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature and says so once per file: noise
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel), then link libagoq.so."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    objs = [os.path.join(objdir, os.path.basename(src) + ".%d.o" % os.getpid()) for src in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        outs = list(pool.map(lambda so: _run([HIPCC, *compile_flags, "-c", "-o", so[1], so[0]]),
                             zip(SOURCES, objs)))
    tmp = LIB + ".tmp.%d" % os.getpid()
    outs.append(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]))
    for o in objs:
        os.remove(o)
    if verbose and any(o.strip() for o in outs):
        print("\n".join(o for o in outs if o.strip()))
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
