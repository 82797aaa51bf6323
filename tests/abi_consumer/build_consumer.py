"""Builds the plain-C consumer of the C ABI (gcc, C99; links libpgti.so and the HIP runtime)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "abi_consumer.c")
EXE = os.path.join(HERE, "abi_consumer")
LIBDIR = os.path.join(ROOT, "paper_2507_11683_amd")


def build(force: bool = False) -> str:
    lib = os.path.join(LIBDIR, "libpgti.so")
    stale = (not os.path.exists(EXE)) or os.path.getmtime(EXE) < max(os.path.getmtime(SRC), os.path.getmtime(lib))
    if force or stale:
        tmp = EXE + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                               "-I", "/opt/rocm/include", SRC, "-o", tmp, "-L", LIBDIR, "-lpgti", "-L", "/opt/rocm/lib",
                               "-lamdhip64", "-Wl,-rpath," + LIBDIR, "-Wl,-rpath,$ORIGIN/../../paper_2507_11683_amd",
                               "-Wl,-rpath,/opt/rocm/lib"])
        os.replace(tmp, EXE)
    return EXE


if __name__ == "__main__":
    print(build(force=True))
