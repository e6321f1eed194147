"""Build libgwq.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libgwq.so")
SOURCES = ["gwq_api.hip", "gwq_pack.hip", "gwq_decode.hip", "gwq_gemm.hip", "gwq_quality.hip", "gwq_score.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, "-I", INCLUDE, "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode:
        # the host pass warns that it does not know the packed-fp32 feature; that is harmless
        noise = "is not a recognized feature for this target"
        print("\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l))
    if res.returncode:
        raise RuntimeError("hipcc failed building libgwq.so")
    return LIB


def stale() -> bool:
    """True when the built library is older than one of its sources or the public header."""
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(INCLUDE, "gwq.h")]
    return any(os.path.getmtime(d) > built for d in deps)


if __name__ == "__main__":
    print(build(verbose=True))
