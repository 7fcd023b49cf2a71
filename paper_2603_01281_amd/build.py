"""Build libseka.so (HIP, gfx950 only) in-tree with hipcc.  Usage: python -m paper_2603_01281_amd.build"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libseka.so")
PROBES = ["mfma_rate_probe", "hbm_read_probe"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

SOURCES = ["api.hip", "route.hip", "edit.hip", "decode.hip", "learn.hip", "attn_f32.hip", "attn_bf16.hip", "attn_bf16_d128.hip", "attn_bf16_d64.hip",
           "attn_bf16_pipe_plain.hip", "attn_bf16_pipe_r32.hip", "attn_bf16_pipe_r64.hip", "attn_bf16_pipe_r128.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffast-math", "-fno-finite-math-only",
    "-Wno-inline-asm",                                                # m0 is clobbered on purpose by the direct-to-LDS loads
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # packed fp32 VALU forms are kept out on purpose
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _compile(src, extra):
    out = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return out


def build(verbose=False, extra=()):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra)), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    # stand-alone probes (they live beside bench.py, which runs them): the device's sustained MFMA-only rate, and
    # the time of a kernel that only reads a key/value cache of a given shape
    for probe in PROBES:
        exe = os.path.join(ROOT, probe + ".bin")
        cmd = [HIPCC, *[f for f in FLAGS if f != "-fPIC"], os.path.join(ROOT, probe + ".hip"), "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"build of {probe} failed:\n" + r.stderr)
        if verbose:
            print("built", exe)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
