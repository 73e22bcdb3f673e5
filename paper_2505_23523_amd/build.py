"""Builds libstragglar.so in-tree with hipcc for gfx950 (no GPU needed)."""

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libstragglar.so")
STAMP = LIB + ".sources"      # digest of the sources the library was built from
SOURCES = ["api.cpp", "planner.cpp", "matching.cpp", "round_kernel.hip", "fused_kernel.hip", "delay_kernel.hip"]


def source_files():
    """Everything the library is built from."""
    import glob
    return ([os.path.join(CSRC, s) for s in SOURCES] + glob.glob(os.path.join(CSRC, "*.hpp")) +
            glob.glob(os.path.join(INCLUDE, "*.h")))


def source_digest():
    """SHA-256 over the names and contents of everything the library is built from."""
    import hashlib
    h = hashlib.sha256()
    for path in sorted(source_files()):
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def hipcc_path():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose=False):
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Wall", "-Wno-unused-command-line-argument",
           # keep the compiler from forming packed-fp32 instructions
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", INCLUDE, "-I", CSRC, "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if os.path.exists(STAMP):
        os.remove(STAMP)
    digest = source_digest()
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n%s\n%s" % (" ".join(cmd), res.stderr))
    if verbose and err.strip():
        print(err)
    with open(STAMP, "w") as f:
        f.write(digest + "\n")
    return LIB


def build_c_smoke():
    """The plain-C consumer of the ABI used by the GPU tests (tests/c_abi_smoke.c)."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "tests", "c_abi_smoke.c")
    out = os.path.join(root, "tests", "c_abi_smoke")
    cmd = [hipcc_path(), "-x", "c", "-O2", "-std=c11", "-D__HIP_PLATFORM_AMD__", "-I", INCLUDE, "-I", "/opt/rocm/include",
           src, "-o", out, "-L", HERE, "-lstragglar", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../paper_2505_23523_amd", "-Wl,-rpath,/opt/rocm/lib"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("building c_abi_smoke failed:\n%s\n%s" % (" ".join(cmd), res.stderr))
    return out


def build_probe():
    """The store-pattern diagnostic (csrc/store_streams_probe.hip), a stand-alone HIP program."""
    out = os.path.join(HERE, "store_streams_probe")
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-unused-command-line-argument",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", out, os.path.join(CSRC, "store_streams_probe.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("building store_streams_probe failed:\n%s\n%s" % (" ".join(cmd), res.stderr))
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_c_smoke())
    print(build_probe())
