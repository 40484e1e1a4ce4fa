"""Compile the plain-C client of libduhl (tests/c_client/duhl_c_client.c) with gcc as C99."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
LIB = os.path.join(HERE, "libduhl_c_client.so")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build():
    pkg = os.path.join(ROOT, "paper_1708_05357_amd")
    subprocess.check_call([
        "gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fPIC", "-shared",
        "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(ROCM, "include"),
        os.path.join(HERE, "duhl_c_client.c"), "-o", LIB,
        "-L", pkg, "-lduhl", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
        "-Wl,-rpath,$ORIGIN/../../paper_1708_05357_amd", "-Wl,-rpath," + pkg,
        "-Wl,-rpath," + os.path.join(ROCM, "lib")])
    return LIB


if __name__ == "__main__":
    print(build())
