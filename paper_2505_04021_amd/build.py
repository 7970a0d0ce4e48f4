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
    for h in ("prism_kv.h", "prism_kv_tuning.h"):
        t = max(t, os.path.getmtime(os.path.join(HERE, "..", "include", h)))
    return t


def build(force: bool = True, verbose: bool = False, defines=(), out: str = LIB) -> str:
    """defines / out: build a variant with other compile-time kernel knobs beside the default library.
    The sources are compiled side by side (one hipcc process each), then linked."""
    if not force and os.path.exists(out) and os.path.getmtime(out) >= newest_source_mtime():
        return out
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in FLAGS if f != "-shared"] + [f"-D{d}" for d in defines]

    def quiet(text):
        # the host pass does not know the packed-fp32 feature flag and says so; harmless
        return "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l and l.strip())

    with tempfile.TemporaryDirectory(prefix="prismkv_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, src + ".o")
            cmd = [hipcc] + compile_flags + ["-c", "-o", obj, os.path.join(CSRC, src)]
            if verbose:
                print(" ".join(cmd))
            r = subprocess.run(cmd, capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n" + quiet(r.stderr))
            return obj, quiet(r.stderr)

        with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
            done = list(ex.map(compile_one, SOURCES))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", "-o", out] + [o for o, _ in done]
        if verbose:
            print(" ".join(link))
        r = subprocess.run(link, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc link failed:\n" + quiet(r.stderr))
        if verbose:
            for _, err in done:
                if err:
                    print(err)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
