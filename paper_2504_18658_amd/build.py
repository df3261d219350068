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


RESOURCES = os.path.join(HERE, "libpccl_local.resources.json")


def _parse_resource_remarks(text):
    """{kernel: {"vgpr", "scratch_bytes", "vgpr_spill", "sgpr_spill", "occupancy"}} from the compiler's
    -Rpass-analysis=kernel-resource-usage remarks."""
    import re
    keys = {"VGPRs": "vgpr", "ScratchSize [bytes/lane]": "scratch_bytes", "VGPRs Spill": "vgpr_spill",
            "SGPRs Spill": "sgpr_spill", "Occupancy [waves/SIMD]": "occupancy"}
    res, cur = {}, None
    for line in text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = res.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][^:]*): (\d+) \[-Rpass-analysis", line)
        if m and cur is not None and m.group(1) in keys:
            cur[keys[m.group(1)]] = int(m.group(2))
    return res


def build(force=True, verbose=False):
    """Compile every HIP source into one shared library.  Returns its path.

    The compiler's per-kernel resource report is kept next to the library (RESOURCES), and a kernel
    that spills vector registers to memory fails the build: every kernel here is bandwidth-bound, and a spill (a tile
    body that no longer fits the 128 registers of a 1024-thread block, say) halves its speed without
    changing a single result."""
    if not force and not is_stale():
        return LIB
    import json
    import sys
    tmp = LIB + ".tmp.%d" % os.getpid()
    sid = source_id()
    cmd = [hipcc(), *HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", '-DPCCL_BUILD_ID="%s"' % sid,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE)
    err = proc.stderr.decode("utf-8", "replace")
    quiet = []   # everything but the remarks (each is the remark line, the source line and a caret line)
    lines = err.splitlines()
    i = 0
    while i < len(lines):
        if "[-Rpass-analysis=kernel-resource-usage]" in lines[i]:
            i += 1
            while i < len(lines) and (lines[i].lstrip().startswith("|") or " | " in lines[i][:12]):
                i += 1
            continue
        quiet.append(lines[i])
        i += 1
    if quiet:
        sys.stderr.write("\n".join(quiet) + "\n")
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    res = _parse_resource_remarks(err)
    # (scalar registers spilled into lanes of a vector register cost next to nothing and are not meant)
    spilled = {k: v for k, v in res.items() if v.get("vgpr_spill", 0)}
    if spilled:
        os.remove(tmp)
        raise RuntimeError("kernels that spill registers: %s" % ", ".join(
            "%s (%d VGPRs, %d spilled)" % (k, v.get("vgpr", -1), v.get("vgpr_spill", 0)) for k, v in spilled.items()))
    with open(RESOURCES + ".tmp", "w") as f:
        json.dump({"build_id": sid, "kernels": res}, f, indent=0, sort_keys=True)
    os.replace(RESOURCES + ".tmp", RESOURCES)
    os.replace(tmp, LIB)
    return LIB


def resources():
    """The resource report of the library on disk ({kernel: {...}}), or None when the report is missing
    or belongs to another build."""
    import json
    try:
        with open(RESOURCES) as f:
            data = json.load(f)
    except (OSError, ValueError):
        return None
    return data["kernels"] if data.get("build_id") == built_id() else None


if __name__ == "__main__":
    print(build(force=True, verbose=True))
