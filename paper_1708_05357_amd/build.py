"""Build libduhl.so (HIP, gfx950) in-tree with hipcc.  Run as ``python -m paper_1708_05357_amd.build``."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libduhl.so")
SOURCES = ["duhl_api.hip", "kernels_gap.hip", "kernels_select.hip", "kernels_cd.hip", "kernels_misc.hip",
           "host_sampler.hip", "host_stage.hip", "duhl_run.hip",
           "kernels_csr_blocked.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src, force):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    deps = [os.path.join(CSRC, src), os.path.join(CSRC, "duhl_internal.h"),
            os.path.join(ROOT, "include", "duhl.h")]
    if force or not os.path.exists(obj) or os.path.getmtime(obj) < max(map(os.path.getmtime, deps)):
        subprocess.check_call(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(force=True, jobs=6):
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs, "-lpthread"])
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
