"""Build libgwq.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libgwq.so")
SOURCES = ["gwq_api.hip", "gwq_pack.hip", "gwq_decode.hip", "gwq_gemm.hip", "gwq_quality.hip", "gwq_score.hip", "gwq_probe.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


STAMP_LIB = os.path.join(HERE, "libgwq_stamp.so")     # measurement build: kernels record device timestamps


def build(verbose: bool = False, stamps: bool = False) -> str:
    """Builds libgwq.so; with `stamps` the separate measurement library libgwq_stamp.so instead, whose
    decode kernels record the shader clock at their milestones (gwq_debug_read_stamps)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = STAMP_LIB if stamps else LIB
    cmd = [hipcc, *FLAGS, *(["-DGWQ_STAMP"] if stamps else []), "-I", INCLUDE, "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode:
        # the host pass warns that it does not know the packed-fp32 feature; that is harmless
        noise = "is not a recognized feature for this target"
        print("\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l))
    if res.returncode:
        raise RuntimeError("hipcc failed building " + os.path.basename(out))
    return out


def stale() -> bool:
    """True when the built library is older than one of its sources or the public header."""
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(INCLUDE, "gwq.h")]
    return any(os.path.getmtime(d) > built for d in deps)


if __name__ == "__main__":
    import sys
    print(build(verbose=True, stamps="--stamps" in sys.argv))
