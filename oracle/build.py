"""Compile the CPU oracle (plain C) into oracle/liboracle.so.  Test infrastructure only."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "tts_oracle.c")
SRC_POSTNET = os.path.join(HERE, "postnet_oracle.c")
SRC_VOCODER = os.path.join(HERE, "vocoder_oracle.c")
SRC_ENCODER = os.path.join(HERE, "encoder_oracle.c")
OUT = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    newest = max(os.path.getmtime(f) for f in (SRC, SRC_POSTNET, SRC_VOCODER, SRC_ENCODER))
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= newest:
        return OUT
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-o", OUT, SRC, SRC_POSTNET, SRC_VOCODER, SRC_ENCODER, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
