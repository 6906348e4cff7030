"""Build the HIP library in-tree: paper_1909_05073_amd/libpconv.so (gfx950 only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpconv.so")
SOURCES = ["pconv_capi.cpp", "pconv_pack.cpp", "pconv_kernels.hip", "pconv_tiled.hip", "pconv_mfma.hip"]

# packed-FP32 instructions are switched off for every device compile of this project
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]


# The tiled kernel is full of wave-uniform branches (which piece of work, which staging unit, whether
# a wave stages at all).  By default the AMDGPU backend structurizes uniform control flow as well,
# with guarded blocks and register copies at every join; this option leaves uniform regions as the
# plain branches they are.
EXTRA_FLAGS = {"pconv_tiled.hip": ["-mllvm", "-structurizecfg-skip-uniform-regions"]}


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def _run(cmd):
    """Run a compile step; drop the host pass's harmless note about the device-only feature flag."""
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops' is not a recognized" not in l)
    if out.strip():
        print(out)
    if r.returncode != 0:
        raise RuntimeError("build step failed: " + " ".join(cmd))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    gen_dir = os.path.join(HERE, "_build", "gen")
    os.makedirs(gen_dir, exist_ok=True)
    # the record loop of the tiled kernel is generated assembly text
    subprocess.run([sys.executable, os.path.join(CSRC, "gen_tiled_compute.py"),
                    os.path.join(gen_dir, "pconv_tiled_compute.inc")], check=True)
    for src in sources():
        obj = os.path.join(HERE, "_build", os.path.basename(src) + ".o")
        os.makedirs(os.path.dirname(obj), exist_ok=True)
        cmd = [hipcc, *HIP_FLAGS, *EXTRA_FLAGS.get(os.path.basename(src), []),
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", gen_dir, "-c"]
        if src.endswith(".cpp"):
            cmd += ["-x", "hip"]
        cmd += [src, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        _run(cmd)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd))
    _run(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
