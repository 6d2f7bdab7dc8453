"""Compile the HIP sources in csrc/ into libscc_hip.so (gfx950 only), in-tree."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libscc_hip.so")
MEMBW_SRC = os.path.join(CSRC, "membw", "membw.hip")
MEMBW_LIB = os.path.join(HERE, "libscc_membw.so")   # streaming kernels of the benchmark's copy ceiling; not the SCC ABI

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMPILE_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
                 # packed fp32 VALU forms are kept out of the generated code on purpose
                 "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                 "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]
LINK_FLAGS = ["--offload-arch=gfx950", "-fPIC", "-shared", "-fno-gpu-rdc", "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(INCLUDE, "*.h"))
    return any(os.path.getmtime(f) > t for f in deps)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and res.stdout.strip():
        print(res.stdout)


def build(force=True, verbose=False):
    """Build libscc_hip.so.  With force=False, only when a source is newer than the library.
    The translation units are compiled side by side (objects in a scratch directory), then linked."""
    if not force and not stale():
        return LIB
    import concurrent.futures
    import shutil
    import tempfile
    work = tempfile.mkdtemp(prefix="scc_build_")
    try:
        objs = []
        with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(sources()))) as pool:
            jobs = []
            for src in sources():
                obj = os.path.join(work, os.path.basename(src) + ".o")
                objs.append(obj)
                jobs.append(pool.submit(_run, [HIPCC] + COMPILE_FLAGS + ["-I", INCLUDE, "-I", CSRC, "-c", src, "-o", obj],
                                        verbose))
            for j in jobs:
                j.result()
        tmp = LIB + ".tmp.%d" % os.getpid()
        _run([HIPCC] + LINK_FLAGS + ["-o", tmp] + objs, verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIB


def build_membw(force=True, verbose=False):
    """Build libscc_membw.so, the plain copy / read kernels bench.py measures its copy ceiling with."""
    if not force and os.path.exists(MEMBW_LIB) and os.path.getmtime(MEMBW_LIB) >= os.path.getmtime(MEMBW_SRC):
        return MEMBW_LIB
    tmp = MEMBW_LIB + ".tmp.%d" % os.getpid()
    _run([HIPCC] + COMPILE_FLAGS + ["-shared", "-o", tmp, MEMBW_SRC], verbose)
    os.replace(tmp, MEMBW_LIB)
    return MEMBW_LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_membw(force=True, verbose=True))
