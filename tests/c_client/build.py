"""Builds tests/c_client/step_client with gcc as C11: a plain-C program that calls the C
ABI of include/lioncub.h (links liblioncub.so and the HIP runtime, nothing else)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "step_client.c")
EXE = os.path.join(HERE, "step_client")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build():
    libdir = os.path.join(ROOT, "paper_2411_16462_amd")
    tmp = EXE + ".tmp.%d" % os.getpid()
    subprocess.check_call([
        "gcc", "-std=c11", "-O2", "-Wall", "-Wextra", "-Werror", "-pedantic", "-D__HIP_PLATFORM_AMD__",
        "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(ROCM, "include"), SRC, "-o", tmp,
        "-L", libdir, "-llioncub", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
        "-Wl,-rpath,$ORIGIN/../../paper_2411_16462_amd", "-Wl,-rpath," + os.path.join(ROCM, "lib")])
    os.replace(tmp, EXE)
    return EXE


if __name__ == "__main__":
    print(build())
