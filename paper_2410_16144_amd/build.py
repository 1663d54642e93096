"""Compile the HIP library (csrc/*.hip -> libbitlinear.so) for gfx950 with hipcc.

Runs on a machine without a GPU (hipcc cross-compiles).  The shared object is kept in-tree
next to this file so that it travels with the source tree.
"""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libbitlinear.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
    "-I", INCLUDE, "-I", CSRC,
]


# Kernel-argument preload for the decode and quantization kernels: their first seven scalar arguments arrive in
# registers with the wave (see BL_FIRST_WG_PARAMS in csrc/bl_internal.hpp).  A compiler option per translation unit.
PER_FILE_FLAGS = {
    "bl_gemv.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=7"],
    "bl_decode_sk.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=7"],
    "bl_quant.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=7"],
}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _newest_input():
    files = sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(INCLUDE, "*.h"))
    return max(os.path.getmtime(f) for f in files)


def _hip_runtime_dir() -> str:
    """Directory of the HIP runtime to link against.  The process that uses this library also
    holds PyTorch, whose wheel ships its own libamdhip64.so (without a versioned SONAME); two
    HIP runtimes in one process do not share streams or allocations, so link against the very
    file PyTorch loads.  Without PyTorch, fall back to the ROCm installation."""
    try:
        import torch
        d = os.path.join(os.path.dirname(torch.__file__), "lib")
        if os.path.exists(os.path.join(d, "libamdhip64.so")):
            return d
    except ImportError:
        pass
    return "/opt/rocm/lib"


def build(force: bool = True, extra_flags=(), verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library.  Returns its path."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= _newest_input():
        return LIB
    os.makedirs(OBJ_DIR, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        cmd = [HIPCC, *FLAGS, *PER_FILE_FLAGS.get(os.path.basename(src), []), *extra_flags, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        # the host pass does not know the (device-only) packed-fp32 feature and says so once per line
        noise = "'-packed-fp32-ops' is not a recognized feature"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
        if err.strip():
            print(err, flush=True)
        if r.returncode != 0:
            raise subprocess.CalledProcessError(r.returncode, cmd)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, sources()))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp,
                           "-no-hip-rt", "-L", _hip_runtime_dir(), "-lamdhip64"])
    os.replace(tmp, LIB)
    return LIB


ABI_CHECK_SRC = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "abi_check.c")
ABI_CHECK_BIN = os.path.join(os.path.dirname(HERE), "tests", "c_abi", "abi_check")


def build_abi_check() -> str:
    """Compile the plain-C host program of tests/c_abi with gcc and link it against the library:
    proof that include/bitlinear.h is C, and a caller of the boundary with no Python in between.
    It runs without PyTorch, so it takes the HIP runtime of the ROCm installation (same SONAME as
    the one the library was linked against)."""
    tmp = ABI_CHECK_BIN + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
                           "-I", INCLUDE, ABI_CHECK_SRC, "-o", tmp, "-L", HERE, "-lbitlinear",
                           "-L", "/opt/rocm/lib", "-lamdhip64",
                           "-Wl,-rpath,$ORIGIN/../../paper_2410_16144_amd", "-Wl,-rpath,/opt/rocm/lib"])
    os.replace(tmp, ABI_CHECK_BIN)
    return ABI_CHECK_BIN


CEILINGS_SRC = os.path.join(os.path.dirname(HERE), "tests", "ceilings", "ceilings.hip")
CEILINGS_LIB = os.path.join(os.path.dirname(HERE), "tests", "ceilings", "libceilings.so")


def build_ceilings() -> str:
    """The measured-ceiling probes of bench.py (a register-only MFMA loop, a read-only streaming kernel): a library of
    their own under tests/, not linked into libbitlinear.so."""
    tmp = CEILINGS_LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Wno-unused-command-line-argument", CEILINGS_SRC, "-o", tmp,
                           "-no-hip-rt", "-L", _hip_runtime_dir(), "-lamdhip64"], stderr=subprocess.DEVNULL)
    os.replace(tmp, CEILINGS_LIB)
    return CEILINGS_LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_abi_check())
    print(build_ceilings())
