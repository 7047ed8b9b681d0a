"""Builds libwkv.so (gfx950) in-tree with hipcc.  Run as ``python -m paper_2503_17922_amd.build``."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libwkv.so")
SOURCES = ["wkv_host.cpp", "wkv_api.cpp", "wkv_score.hip", "wkv_resident.hip", "wkv_select.hip", "wkv_gather.hip",
           "wkv_decode.hip"]
HOST_SOURCES = ["wkv_host.cpp", "wkv_api.cpp"]          # no device code: also built for the CPU-only sanitizer test
NOISE = "is not a recognized feature for this target"


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("build step failed: " + " ".join(cmd) + "\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = True) -> str:
    """Compile every source for gfx950 (one hipcc process per file, side by side) and link the
    shared library; always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU ops
             "-x", "hip", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = [os.path.join(OBJ, s + ".o") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        list(pool.map(lambda so: _run([hipcc(), *flags, "-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose),
                      zip(SOURCES, objs)))
    _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    return LIB


def build_host_sanitized(out_dir: str, extra_sources, exe_name: str = "cabi_validation", verbose: bool = False) -> str:
    """The host half of the library (argument validation, derived sizes, launch planning: the
    files that hold no device code) compiled for the CPU with AddressSanitizer and
    UndefinedBehaviorSanitizer and linked with ``extra_sources`` (a test driver plus stand-ins for
    the kernel launchers) into an executable.  Used by the CPU-only test of the C ABI."""
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, exe_name)
    cmd = [clang, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in HOST_SOURCES], *extra_sources,
           "-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    _run(cmd, verbose)
    return exe


if __name__ == "__main__":
    print(build())
