"""Build libsp24.so (hand-written HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2104_08378_amd.build

The shared library lands next to this file so that it travels with the source
tree; nothing is installed.  There is one code path and one target: no CUDA
shims, no fallback.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsp24.so")
PROBE = os.path.join(HERE, "sp24_probe")        # stand-alone measurement of the chip's ceilings (csrc/probe.hip)
SOURCES = ["api.hip", "prune_compress.hip", "permute.hip", "permute_search.hip", "splitk.hip", "mm_simple.hip", "mm_skinny.hip", "mm_tiled.hip"] + [
    "mm_tiled_%s_%s.hip" % (i, o) for i, o in
    [("f16", "f32"), ("f16", "f16"), ("f16", "bf16"), ("bf16", "f32"), ("bf16", "f16"), ("bf16", "bf16"),
     ("i8", "i32"), ("i8", "i8"), ("i8", "f32"), ("i8", "f16"), ("i8", "bf16"), ("f8", "f32"), ("f8", "f16"), ("f8", "bf16")]]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # hipcc must not form packed-fp32 instructions by itself on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose=False):
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    probe_cmd = ["hipcc", *[f for f in FLAGS if f != "-fPIC"], os.path.join(CSRC, "probe.hip"), "-o", PROBE]
    procs.append(("probe.hip", subprocess.Popen(probe_cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "is not a recognized feature for this target" not in l)
        if p.returncode != 0:
            failed = True
            print(f"hipcc failed for {src}:\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("libsp24 build failed")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
