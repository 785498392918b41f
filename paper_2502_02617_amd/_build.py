"""Builds libpolarquant.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libpolarquant.so")
SOURCES = ["pq_host.hip", "pq_encode.hip", "pq_decode.hip", "pq_attn.hip", "pq_fit.hip", "pq_general.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose=False):
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = ["hipcc"] + HIPCC_FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LIB_PATH


MEMBENCH_PATH = os.path.join(LIB_DIR, "pq_membench")


def build_membench():
    """Stand-alone HBM read-ceiling / counter-calibration probe (see csrc/pq_membench.hip)."""
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "pq_membench.hip"), "-o", MEMBENCH_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return MEMBENCH_PATH


ISSUEBENCH_PATH = os.path.join(LIB_DIR, "pq_issuebench")


def build_issuebench():
    """Stand-alone probe of instruction issue costs and matrix / vector overlap (see csrc/pq_issuebench.hip)."""
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "pq_issuebench.hip"), "-o", ISSUEBENCH_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return ISSUEBENCH_PATH


LDSBENCH_PATH = os.path.join(LIB_DIR, "pq_ldsbench")


def build_ldsbench():
    """Stand-alone probe of LDS table-gather costs (see csrc/pq_ldsbench.hip)."""
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "pq_ldsbench.hip"), "-o", LDSBENCH_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    return LDSBENCH_PATH


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_membench())
    print(build_issuebench())
    print(build_ldsbench())
