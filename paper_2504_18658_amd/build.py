"""Build libpccl_local.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import hashlib
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpccl_local.so")
SOURCES = ["pccl_api.hip", "reduce_kernels.hip", "permute_kernels.hip", "step_kernels.hip",
           "fused_kernels.hip", "cost_model.hip", "address_check.hip", "knobs.hip"]
HEADERS = ["device_utils.h", "kernels.h", "address_check.h", "knobs.h", "reduce_device.h", "permute_device.h", os.path.join("..", "..", "include", "pccl_local.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # IEEE adds only: no contraction, no fast-math, subnormals kept
    "-ffp-contract=off", "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc():
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the HIP library cannot be built")
    return exe


ID_MARKER = b"pccl-build-id:"


def source_id():
    """Identity of what a build is made from: the compiler flags and the bytes of every source and header."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for name in SOURCES + HEADERS:
        h.update(name.encode())
        with open(os.path.join(CSRC, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def built_id(path=LIB):
    """The source identity compiled into a built library (None when the file or the marker is missing)."""
    try:
        with open(path, "rb") as f:
            data = f.read()
    except OSError:
        return None
    k = data.find(ID_MARKER)
    return data[k + len(ID_MARKER):k + len(ID_MARKER) + 16].decode("ascii", "replace") if k >= 0 else None


def is_stale():
    """True when the library on disk was not built from the sources on disk (file times play no part)."""
    return built_id() != source_id()


def build(force=True, verbose=False):
    """Compile every HIP source into one shared library.  Returns its path."""
    if not force and not is_stale():
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, '-DPCCL_BUILD_ID="%s"' % source_id(),
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
