"""Build the C-ABI library (HIP kernels + host code) for gfx950 into
paper_2211_13939_amd/libtts_pool.so.  Run on the CPU machine; hipcc cross-compiles."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libtts_pool.so")
SOURCES = ["kernels.hip", "tts_pool.cpp", "postnet.hip", "postnet.cpp", "vocoder.hip", "vocoder.cpp", "encoder.hip", "encoder.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the first 16 dwords of a kernel's arguments arrive in scalar registers with the wave (gfx950 preloads them):
         # the first loads of a kernel no longer wait for a cold read of the argument block
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-result"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale() -> bool:
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(HERE, "..", "include", "tts_pool.h"))
    deps.append(os.path.join(HERE, "..", "include", "tts_postnet.h"))
    deps.append(os.path.join(HERE, "..", "include", "tts_vocoder.h"))
    deps.append(os.path.join(HERE, "..", "include", "tts_encoder.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False) -> str:
    cmd = [HIPCC] + FLAGS + ["-x", "hip"] + sources() + ["-o", OUT]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
