"""Compile the HIP sources into paper_1803_06333_amd/lib/libsnap.so for gfx950 with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC_DIR = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libsnap.so")
SOURCES = ["api.hip", "perm.hip", "scd.hip", "linalg.hip", "stream.hip", "grouped.hip", "dense_tiles.hip", "probe.hip"]


def build(verbose: bool = False, out: str = LIB_PATH, defines=()) -> str:
    os.makedirs(os.path.dirname(out), exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-munsafe-fp-atomics",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
           "-o", out] + ["-D" + d for d in defines] + [os.path.join(SRC_DIR, s) for s in SOURCES]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 target feature and says so: harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
