"""Compile the C part of the CPU oracle (test infrastructure, not product code).

The one source file is compiled twice, with REAL = float (the fp32 oracle) and
REAL = double (its twin), and linked into ``oracle/libs3oracle.so``.
"""
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "s3_oracle.c")
LIB = os.path.join(HERE, "libs3oracle.so")


def build_oracle(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    flags = ["-O2", "-fopenmp", "-fPIC", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]
    with tempfile.TemporaryDirectory() as tmp:
        objs = []
        for real, suf in (("float", "f32"), ("double", "f64")):
            obj = os.path.join(tmp, f"s3_oracle_{suf}.o")
            subprocess.check_call(["gcc", *flags, f"-DREAL={real}", f"-DSUF={suf}", "-c", SRC, "-o", obj])
            objs.append(obj)
        tmp_lib = LIB + ".tmp"
        subprocess.check_call(["gcc", "-shared", "-fopenmp", *objs, "-o", tmp_lib, "-lm"])
        os.replace(tmp_lib, LIB)
    return LIB


if __name__ == "__main__":
    print(build_oracle())
