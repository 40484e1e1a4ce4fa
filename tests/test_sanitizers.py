"""Host-side AddressSanitizer / UndefinedBehaviorSanitizer runs (no GPU is touched).

1. The CPU oracle (oracle/duhl_oracle.c) on the instances worked by hand from App. C, D, E.
2. The C ABI's argument checks: the library's host logic (entry points, round loop, host sampler,
   staging) compiled with the sanitizers on the host side only (-Xarch_host; GPU sanitizers are not
   available), linked with the kernels' ordinary objects, and driven by the plain-C client.
Each runs in a subprocess; any sanitizer report makes it exit non-zero."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(exe, env=ENV):
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
    return r.stdout


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", *SAN, os.path.join(HERE, "oracle_driver.c"),
                           os.path.join(ROOT, "oracle", "duhl_oracle.c"), "-o", exe, "-lm"])
    assert "ok" in _run(exe)


def test_sanitizer_build_catches_a_planted_overrun(tmp_path):
    """The harness itself: an oracle whose column dot product runs one entry too far must be reported."""
    src = open(os.path.join(ROOT, "oracle", "duhl_oracle.c")).read()
    old = "for (int64_t k = 0; k < M->d; ++k) s += (double)a[k] * v[k];"
    assert src.count(old) == 1
    bad = tmp_path / "bad_oracle.c"
    bad.write_text(src.replace(old, "for (int64_t k = 0; k <= M->d; ++k) s += (double)a[k] * v[k];"))
    exe = str(tmp_path / "bad_driver")
    subprocess.check_call(["gcc", "-std=c99", *SAN, os.path.join(HERE, "oracle_driver.c"), str(bad), "-o", exe, "-lm"])
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_c_abi_argument_checks_run_clean_under_asan_and_ubsan(tmp_path):
    sys.path.insert(0, ROOT)
    from paper_1708_05357_amd import build as b
    b.build(force=False)                                    # the kernels' ordinary objects
    host_logic = ["duhl_api.hip", "duhl_run.hip", "host_sampler.hip", "host_stage.hip"]
    flags = [f for f in b.FLAGS if f != "-O3"] + ["-O1", "-g", "-Xarch_host", "-fsanitize=address",
                                                   "-Xarch_host", "-fsanitize=undefined",
                                                   "-Xarch_host", "-fno-sanitize-recover=all"]
    procs, objs = [], []
    for src in b.SOURCES:
        if src in host_logic:
            obj = str(tmp_path / src.replace(".hip", ".o"))
            procs.append(subprocess.Popen(["hipcc", *flags, "-c", os.path.join(b.CSRC, src), "-o", obj],
                                          stderr=subprocess.DEVNULL))
        else:
            obj = os.path.join(b.CSRC, src.replace(".hip", ".o"))
        objs.append(obj)
    assert all(p.wait() == 0 for p in procs)
    lib = str(tmp_path / "libduhl_asan.so")
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address",
                           "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", lib, *objs, "-lpthread"],
                          stderr=subprocess.DEVNULL)
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    exe = str(tmp_path / "abi_driver")
    # (the client with the same compiler family as the library, so that both use one sanitizer runtime)
    clang = os.path.join(rocm, "llvm", "bin", "clang")
    subprocess.check_call([clang, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", *SAN,
                           "-I", os.path.join(ROOT, "include"), "-isystem", os.path.join(rocm, "include"),
                           os.path.join(HERE, "abi_driver.c"), os.path.join(ROOT, "tests", "c_client", "duhl_c_client.c"),
                           "-o", exe, lib, "-L", os.path.join(rocm, "lib"), "-lamdhip64",
                           "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath," + os.path.join(rocm, "lib")])
    assert "ok" in _run(exe)
