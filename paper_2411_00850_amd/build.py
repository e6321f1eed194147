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


# Checking build for the CPU side: the host code of the library (argument checks, layout arithmetic, launch planning)
# under clang's address and undefined-behaviour sanitizers, every report fatal; the device code is built as usual.
# GWQ_SANITIZE_HOST=1 makes the binding load it; the Python process needs the sanitizer runtime loaded first:
#   python -m paper_2411_00850_amd.build --sanitize-host
#   LD_PRELOAD="$(/opt/rocm/lib/llvm/bin/clang -print-file-name=libclang_rt.asan-x86_64.so):$LD_PRELOAD" \
#       ASAN_OPTIONS=detect_leaks=0 GWQ_SANITIZE_HOST=1 python -m pytest tests/test_abi.py -q
SAN_LIB = os.path.join(HERE, "libgwq_san.so")
SAN_FLAGS = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-shared-libsan"]


def build(verbose: bool = False, stamps: bool = False, sanitize_host: bool = False) -> str:
    """Builds libgwq.so; with `stamps` the separate measurement library libgwq_stamp.so instead, whose
    decode kernels record the shader clock at their milestones (gwq_debug_read_stamps); with `sanitize_host`
    the checking build libgwq_san.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = SAN_LIB if sanitize_host else STAMP_LIB if stamps else LIB
    cmd = [hipcc, *FLAGS, *(SAN_FLAGS if sanitize_host else []), *(["-DGWQ_STAMP"] if stamps else []), "-I", INCLUDE, "-I", CSRC,
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
    print(build(verbose=True, stamps="--stamps" in sys.argv, sanitize_host="--sanitize-host" in sys.argv))
