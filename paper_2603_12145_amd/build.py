"""Compile the HIP sources under csrc/ into libmi355env.so (gfx950 only), in-tree.

Flags: -ffp-contract=off so that no multiply-add is fused behind the source's back (the Pong path is
compared bit for bit with a scalar CPU implementation; where the body wants an FMA it asks for one
explicitly), and packed-FP32 instruction selection is disabled.  The instruction scheduler is told to
maximise instruction-level parallelism rather than occupancy: the rollout kernels run one wavefront
per SIMD at the headline size, so only independent instructions of the same wavefront can hide the
latency of a dependent chain (Pong N = 65536 x T = 1000: 0.47 ms instead of 0.53 ms per launch; the
other kernels are unaffected).
"""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmi355env.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
         "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-sched-strategy=max-ilp",
         "-Wall", "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(force=True, verbose=False, extra=(), out=None):
    """extra: additional hipcc flags (e.g. -D switches for measurement variants); out: alternative
    output path (the default in-tree library is what the binding loads)."""
    srcs = sources()
    deps = srcs + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(CSRC, "*.inc")) + glob.glob(
        os.path.join(HERE, "..", "include", "*.h"))
    lib = out or LIB
    if not force and os.path.exists(lib) and all(
            os.path.getmtime(lib) >= os.path.getmtime(d) for d in deps):
        return lib
    cmd = [HIPCC] + FLAGS + list(extra) + ["-o", lib] + srcs
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    args = sys.argv[1:]
    out = None
    if "--out" in args:
        k = args.index("--out")
        out = os.path.abspath(args[k + 1])
        del args[k:k + 2]
    print(build(force=True, verbose=True, extra=args, out=out))
