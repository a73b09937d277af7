"""Compile the CPU checker (oracle/dn_oracle.c, oracle/dn_conv_oracle.c) into oracle/libdn_oracle.so.

Each C file is built three times into one shared object: fp32 storage with
fp64 accumulation (symbols o32_*), all-fp64 (o64_*), and fp32 storage with fp32
accumulation (o32a_*: not a reference, a measure of fp32 rounding drift).  Flags avoid
-march=native and fused contraction so the library gives the same bits on any
x86-64-v3 host.  Test infrastructure only.
"""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "dn_oracle.c"), os.path.join(HERE, "dn_conv_oracle.c")]
LIB = os.path.join(HERE, "libdn_oracle.so")
CFLAGS = ["-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-fPIC", "-std=c11",
          "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SRCS):
        return LIB
    with tempfile.TemporaryDirectory() as tmp:
        objs = []
        for src in SRCS:
            for store, acc, pfx in (("float", "double", "o32_"), ("double", "double", "o64_"), ("float", "float", "o32a_")):
                obj = os.path.join(tmp, pfx + os.path.basename(src) + ".o")
                cmd = ["gcc", *CFLAGS, "-DSTORE_T=" + store, "-DACC_T=" + acc, "-DPFX(x)=" + pfx + "##x", "-c", src, "-o", obj]
                subprocess.run(cmd, check=True)
                objs.append(obj)
        subprocess.run(["gcc", "-shared", "-fopenmp", "-o", LIB, *objs, "-lm"], check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
