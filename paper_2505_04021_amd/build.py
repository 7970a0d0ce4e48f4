"""Build libprismkv.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libprismkv.so")
SOURCES = ["api.hip", "pool_kernels.hip", "attn_kernels.hip", "kv_kernels.hip", "policy.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         # keep single-lane atomics as written: the optimiser would broadcast their result at once,
         # which forces a full wait on all outstanding KV loads at every queue / arrival atomic
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]


def newest_source_mtime():
    t = 0.0
    for root, _, files in os.walk(CSRC):
        for f in files:
            t = max(t, os.path.getmtime(os.path.join(root, f)))
    t = max(t, os.path.getmtime(os.path.join(HERE, "..", "include", "prism_kv.h")))
    return t


def build(force: bool = True, verbose: bool = False, defines=(), out: str = LIB) -> str:
    """defines / out: build a variant with other compile-time kernel knobs beside the default library."""
    if not force and os.path.exists(out) and os.path.getmtime(out) >= newest_source_mtime():
        return out
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + [f for f in FLAGS if f] + [f"-D{d}" for d in defines] + ["-o", out] + \
          [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature flag and says so; harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err:
        print(err)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
