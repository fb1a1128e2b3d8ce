"""Builds liblms.so (C-ABI library: graph rewriter, executor, gfx950 kernels) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "liblms.so")


def sources():
    c = os.path.join(HERE, "csrc")
    return sorted(os.path.join(c, f) for f in os.listdir(c) if f.endswith((".cpp", ".hip")))


def build(verbose=False, jobs=None):
    """Compiles every source to an object file (in parallel) and links them.  Always compiles."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
             # packed fp32 instructions are kept out of generated code on purpose
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument",
             "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    jobs = jobs or max(1, min(8, os.cpu_count() or 1))
    log = []

    def run(cmd):
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
        if out.strip():
            log.append(out)

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        run([hipcc] + flags + ["-c", src, "-o", obj])
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, sources()))
    run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared"] + objs + ["-o", LIB])
    if verbose and log:
        print("\n".join(log))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
