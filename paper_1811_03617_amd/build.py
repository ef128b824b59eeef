"""Build libgvq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgvq.so")
SOURCES = ["gvq_api.cpp", "gvq_codec.hip", "gvq_codec_long.hip", "gvq_codec_ws.hip", "gvq_fit.hip", "gvq_fit_large.hip", "gvq_eigen_block.hip", "gvq_layout.hip"]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 VALU ops are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source to an object file (in parallel), then link the shared library."""
    import concurrent.futures
    import shutil
    import tempfile

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    common = [hipcc, *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    tmp = tempfile.mkdtemp(prefix="gvq_build_")

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # the host pass says it does not know the packed-fp32 target feature: harmless
        log = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + log)
        if verbose and log.strip():
            print(log, flush=True)

    try:
        objs = [os.path.join(tmp, s + ".o") for s in SOURCES]
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(7, len(SOURCES))) as pool:
            jobs = [pool.submit(run, [*common, "-c", "-o", o, os.path.join(CSRC, s)]) for s, o in zip(SOURCES, objs)]
            for j in jobs:
                j.result()
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp", *objs])
        os.replace(LIB + ".tmp", LIB)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "gvq.h")]
    return any(os.path.getmtime(p) > t for p in deps)


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
