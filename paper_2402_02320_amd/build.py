"""Builds libspin.so (the C-ABI library of include/spin.h) for gfx950 with hipcc.

    python -m paper_2402_02320_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspin.so")
SOURCES = ["spin_api.hip", "elementwise.hip", "gemm_valu.hip", "gemm_limb.hip", "gemm_limb128.hip", "probe.hip"]
COMPILE_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                 "-Wall", "-Wno-unused-command-line-argument"]
LINK_FLAGS = ["--offload-arch=gfx950", "-fPIC", "-shared", "-Wno-unused-command-line-argument"]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the device-only target feature and says so on every file
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose=False, extra=(), jobs=None):
    """Compiles every source to an object file (in parallel, at most `jobs` at a time) and links them."""
    from concurrent.futures import ThreadPoolExecutor
    cc = hipcc()
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = jobs or min(len(SOURCES), os.cpu_count() or 1, 8)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        futures = [pool.submit(_run, [cc] + COMPILE_FLAGS + list(extra) + ["-c", os.path.join(CSRC, s), "-o", o],
                               verbose) for s, o in zip(SOURCES, objs)]
        for f in futures:
            f.result()
    _run([cc] + LINK_FLAGS + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
