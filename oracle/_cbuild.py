"""Compile one C file of the oracle into a shared library beside it (gcc, OpenMP)."""
import os
import subprocess


def compile_shared(src: str, lib: str, force: bool = False) -> str:
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(src):
        tmp = lib + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, src])
        os.replace(tmp, lib)
    return lib
