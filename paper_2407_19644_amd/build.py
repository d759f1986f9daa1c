"""Builds libubp.so (host packer + HIP kernels for gfx950) in-tree with hipcc."""
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libubp.so")
HOST_SOURCES = ["ubp_host.cpp", "ubp_layouts.cpp", "ubp_select.cpp"]
HIP_SOURCES = ["ubp_api.hip", "ubp_wros.hip", "ubp_stripe.hip", "ubp_blk.hip", "ubp_tile.hip", "ubp_gemm.hip"]
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result"]
# packed-fp32 VALU forms are switched off for every device function in this library
HIP_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose=False, jobs=None, defines=(), out=None):
    """Compile every source (in parallel) and link libubp.so (or `out`); always recompiles.  Returns the path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC] + ["-D" + d for d in defines]
    lib = out or LIB
    tmpdir = tempfile.mkdtemp(prefix="ubp_build_")
    try:
        cmds = []
        for s in HOST_SOURCES:
            obj = os.path.join(tmpdir, s + ".o")
            cmds.append((obj, [hipcc] + COMMON + inc + ["-x", "c++", "-c", os.path.join(CSRC, s), "-o", obj]))
        for s in HIP_SOURCES:
            obj = os.path.join(tmpdir, s + ".o")
            cmds.append((obj, [hipcc] + COMMON + HIP_FLAGS + inc + ["-x", "hip", "-c", os.path.join(CSRC, s), "-o", obj]))

        def run(item):
            obj, cmd = item
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            return obj, res.returncode, res.stdout

        jobs = jobs or min(8, len(cmds), os.cpu_count() or 1)
        with ThreadPoolExecutor(max_workers=jobs) as ex:
            results = list(ex.map(run, cmds))
        for obj, rc, out in results:
            if rc != 0:
                raise RuntimeError("hipcc failed:\n" + out)
            if verbose and out.strip():
                print(out)
        tmp = lib + ".tmp%d" % os.getpid()
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [o for o, _, _ in results]
        res = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            if os.path.exists(tmp):
                os.remove(tmp)
            raise RuntimeError("link failed:\n" + res.stdout)
        os.replace(tmp, lib)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return lib


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
