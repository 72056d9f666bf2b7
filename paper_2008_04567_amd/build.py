"""Build libwpk.so (HIP, gfx950 only) in-tree with hipcc.

``python -m paper_2008_04567_amd.build`` (add ``--changed`` to compile only what is stale) or
``build_library()``.  Translation units are compiled
in parallel: the host part, the API/dispatch part and eight instantiation parts of the tiled
kernel family.  Works without a GPU (hipcc cross-compiles).
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libwpk.so")
N_PARTS = 8

COMMON = ["-O3", "-fPIC", "-std=c++17", "-I" + INCLUDE, "-I" + CSRC, "-Wall", "-Wno-unused-function"]
# packed-FP32 instructions are switched off for all device code
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        lines = out.splitlines()
        if len(lines) > 60:
            lines = lines[:60] + ["... (%d more lines)" % (len(lines) - 60)]
        raise RuntimeError("build step failed: %s\n%s" % (" ".join(cmd), "\n".join(lines)))
    return out


def sources_newer_than_lib():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(INCLUDE, "wpk.h")]
    return any(os.path.getmtime(f) > t for f in files)


def _stale(obj, deps):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(f) > t for f in deps)


def build_library(force=True, verbose=False):
    """Compile and link libwpk.so.  Returns its path.  With ``force=False`` only the objects whose
    sources (or headers) are newer than they are get compiled again."""
    if not force and not sources_newer_than_lib():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    src = lambda f: os.path.join(CSRC, f)
    headers = [os.path.join(INCLUDE, "wpk.h"), src("wpk_internal.h")]
    kernel_headers = headers + [src("wpk_igemm.h"), src("wpk_wsplit.h"), src("wpk_variants.def")]
    jobs, objs = [], []

    def add(cmd, deps):
        objs.append(cmd[-1])
        if force or _stale(cmd[-1], deps):
            jobs.append(cmd)

    add([hipcc] + COMMON + ["-c", src("wpk_host.cpp"), "-o", os.path.join(OBJ, "wpk_host.o")],
        headers + [src("wpk_host.cpp"), src("wpk_variants.def")])
    add([hipcc] + COMMON + DEVICE + ["-c", src("wpk_api.hip"), "-o", os.path.join(OBJ, "wpk_api.o")],
        kernel_headers + [src("wpk_api.hip")])
    for part in range(N_PARTS):
        add([hipcc] + COMMON + DEVICE + ["-DWPK_PART=%d" % part, "-c", src("wpk_igemm_inst.hip"),
                                         "-o", os.path.join(OBJ, "wpk_igemm_%d.o" % part)],
            kernel_headers + [src("wpk_igemm_inst.hip")])
    if jobs:
        workers = min(len(jobs), max(1, (os.cpu_count() or 4)), 16)
        with concurrent.futures.ThreadPoolExecutor(workers) as ex:
            for out in ex.map(_run, jobs):
                if verbose and out.strip():
                    print(out)
    _run(_link_command(objs))
    return LIB


def _link_command(objs):
    """Link against the HIP runtime PyTorch ships, when there is one.

    The PyTorch-ROCm wheel bundles its own libamdhip64.so (file name without version, no
    SONAME).  A process must hold ONE HIP runtime: tensors and streams made by PyTorch are
    handed to this library.  Linking against the bundled file records the dependency under the
    same name PyTorch uses, so whichever of the two is loaded first, the loader reuses it for
    the other.  Without PyTorch the system runtime under /opt/rocm is used.
    """
    rocm_lib = "/opt/rocm/lib"
    torch_lib = None
    try:
        import importlib.util
        spec = importlib.util.find_spec("torch")
        if spec and spec.origin:
            cand = os.path.join(os.path.dirname(spec.origin), "lib")
            if os.path.exists(os.path.join(cand, "libamdhip64.so")):
                torch_lib = cand
    except Exception:
        torch_lib = None
    cmd = ["g++", "-shared", "-fPIC", "-o", LIB] + objs
    if torch_lib:
        cmd += ["-L" + torch_lib, "-l:libamdhip64.so",
                "-Wl,-rpath," + torch_lib + ":" + rocm_lib]
    else:
        cmd += ["-L" + rocm_lib, "-lamdhip64", "-Wl,-rpath," + rocm_lib]
    return cmd


if __name__ == "__main__":
    print(build_library(force="--changed" not in sys.argv, verbose="-v" in sys.argv))
