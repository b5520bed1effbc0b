"""Compile the HIP sources under csrc/ into librcp.so for gfx950 (hipcc cross-compiles without a GPU).

Every source file is compiled to an object of its own, several at a time, then the objects are linked;
no device code crosses translation units, so no relocatable device code is needed."""
import concurrent.futures
import glob
import os
import shutil
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librcp.so")

COMPILE_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # kernel arguments arrive in scalar registers with the wavefront launch instead of being
    # fetched by its first instructions (these kernels run for a few microseconds)
    "-mllvm", "-amdgpu-kernarg-preload-count=16",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    return res.returncode, out


def build(verbose: bool = False, jobs: int = 0) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(8, os.cpu_count() or 1, int(os.environ.get("MAX_JOBS", "8")))
    tmp = tempfile.mkdtemp(prefix="rcp_build_")
    try:
        srcs = sources()
        objs = [os.path.join(tmp, os.path.basename(s)[:-4] + ".o") for s in srcs]
        cmds = [[hipcc] + COMPILE_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", s, "-o", o]
                for s, o in zip(srcs, objs)]
        with concurrent.futures.ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            results = list(pool.map(_run, cmds))
        for cmd, (rc, out) in zip(cmds, results):
            if verbose and out.strip():
                print(out)
            if rc != 0:
                raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp"] + objs
        rc, out = _run(link)
        if rc != 0:
            raise RuntimeError("link failed:\n" + out)
        os.replace(LIB + ".tmp", LIB)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
