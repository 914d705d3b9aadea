"""Build libbittrain.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "bittrain.hip")
LIB = os.path.join(HERE, "libbittrain.so")
# measurement aids for bench.py: the same kernels with per-tile time stamps compiled in, plus a plain stream
BENCH_SRC = os.path.join(HERE, "csrc", "bench_aids.hip")
BENCH_LIB = os.path.join(HERE, "libbittrain_bench.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
    # packed fp32 VALU forms are kept out of the device code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose=False, extra_flags=(), lib=LIB, src=SRC):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-I", os.path.join(ROOT, "include"), src, "-o", lib]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return lib


def build_bench_aids(verbose=False, extra_flags=()):
    return build(verbose=verbose, extra_flags=extra_flags, lib=BENCH_LIB, src=BENCH_SRC)


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_bench_aids(verbose=True))
