"""Compile the CPU oracle (plain C, gcc + OpenMP) into oracle/liboracle.so.

Test infrastructure only: the product library never links or loads this file.
The source is compiled twice, once storing float and once storing double, so
that the double build can be checked tightly by finite differences and the
float build (the one the GPU path is compared with) is the same code.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle.c")
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    objs = []
    for real, suffix in (("float", "_f32"), ("double", "_f64")):
        obj = os.path.join(HERE, f"oracle{suffix}.o")
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-fPIC", "-std=c11", "-Wall", f"-DREAL={real}",
             f"-DSUFFIX={suffix}", "-c", SRC, "-o", obj])
        objs.append(obj)
    subprocess.check_call(["gcc", "-shared", "-fopenmp", "-o", LIB] + objs + ["-lm"])
    for o in objs:
        os.remove(o)
    return LIB


if __name__ == "__main__":
    print(build())
