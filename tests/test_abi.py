"""The C-ABI library loads and exports every entry point that include/duhl.h declares.
No compute calls: this runs where no GPU is visible."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "duhl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(duhl_[a-z_]+)\s*\(", text)))


def test_header_declares_the_six_named_calls():
    names = declared_symbols()
    for must in ["duhl_create", "duhl_set_data_dense", "duhl_set_data_csr", "duhl_gap", "duhl_select",
                 "duhl_cd_epoch", "duhl_objective"]:
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_1708_05357_amd import duhl
    lib = duhl.load()
    names = declared_symbols()
    assert len(names) >= 15
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(duhl.EXPORTS) == names


def test_bad_arguments_are_rejected_without_a_gpu():
    """Argument checks that come before any device work."""
    from paper_1708_05357_amd import duhl
    lib = duhl.load()
    h = ctypes.c_void_p()
    assert lib.duhl_create(None, 0, 10, 10, 5, 0, None, None) == duhl.EINVAL
    assert lib.duhl_create(ctypes.byref(h), 7, 10, 10, 5, 0, None, None) == duhl.EINVAL
    assert lib.duhl_create(ctypes.byref(h), 0, 0, 10, 5, 0, None, None) == duhl.EINVAL
    assert lib.duhl_create(ctypes.byref(h), 0, 10, -1, 5, 0, None, None) == duhl.EINVAL
    assert lib.duhl_create(ctypes.byref(h), 0, 10, 10, 0, 0, None, None) == duhl.EINVAL
    assert lib.duhl_create(ctypes.byref(h), 0, 10, 10, 5, -1, None, None) in (duhl.EHIP, duhl.EINVAL)
    assert h.value is None
    assert lib.duhl_gap(None, None, 0, None) == duhl.EINVAL
    assert lib.duhl_objective(None, None) == duhl.EINVAL
    assert lib.duhl_set_eta(None, 0.5) == duhl.EINVAL
    assert lib.duhl_working_set_size(None) == 0
    assert lib.duhl_last_error(None) == b"null context"
    lib.duhl_destroy(None)


def test_product_path_does_not_reach_for_the_oracle():
    """The oracle is test infrastructure: nothing in the package may import, load or name it."""
    pkg = os.path.join(ROOT, "paper_1708_05357_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"import\s+oracle|from\s+oracle|duhl_oracle|oracle/", text), f


def test_header_is_plain_c_and_a_c_client_links():
    """include/duhl.h compiles as pedantic C99 with all warnings as errors, inside a client written
    in C that links against the library (gcc; no GPU needed to build)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location(
        "build_client", os.path.join(ROOT, "tests", "c_client", "build_client.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    from paper_1708_05357_amd import duhl
    duhl.load()                                              # the library the client links against
    lib = ctypes.CDLL(mod.build())
    assert hasattr(lib, "duhl_c_client_rounds")
