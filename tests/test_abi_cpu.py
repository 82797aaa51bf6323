"""CPU-only checks of the boundary: the built library loads and exports every symbol that
include/pgti.h declares, the Python binding covers each of them, and argument errors that are
detected before any device work come back as status codes (no GPU is touched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pgti.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pgti_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2507_11683_amd import build, pgti
    if not os.path.exists(pgti.LIB_PATH):
        build.build()
    return pgti.load_library()


def test_header_declares_the_three_calls_of_the_path():
    names = _declared_functions()
    for must in ("pgti_load_series", "pgti_epoch_indices", "pgti_build_batch"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2507_11683_amd import pgti
    names = _declared_functions()
    assert len(names) >= 9
    for name in names:
        assert hasattr(lib, name), f"{name} declared in pgti.h but not exported"
        assert name in pgti.SIGNATURES, f"{name} has no binding signature"
    assert sorted(pgti.SIGNATURES) == names


def test_null_context_is_an_argument_error(lib):
    from paper_2507_11683_amd import pgti
    assert lib.pgti_build_batch(None, 0, None, None, None) == pgti.PGTI_ERR_ARG
    assert b"context" in lib.pgti_last_error()
    assert lib.pgti_epoch_indices(None, 0, 0, 0, 1, None) == pgti.PGTI_ERR_ARG
    assert lib.pgti_num_batches(None) == pgti.PGTI_ERR_ARG
    assert lib.pgti_get_indices(None, None, 0) == pgti.PGTI_ERR_ARG
    assert lib.pgti_get_stats(None, None, None) == pgti.PGTI_ERR_ARG
    assert lib.pgti_load_series(None, None, 10, 1, 1, 1, 1, 1, 0, None, None) == pgti.PGTI_ERR_ARG
    assert lib.pgti_create(None, 0) == pgti.PGTI_ERR_ARG
    lib.pgti_destroy(None)  # documented no-op


def test_binding_has_no_fallback(tmp_path, monkeypatch):
    # a missing library must raise, never route anywhere else
    from paper_2507_11683_amd import pgti
    monkeypatch.setattr(pgti, "_lib", None)
    monkeypatch.setattr(pgti, "LIB_PATH", str(tmp_path / "libpgti.so"))
    with pytest.raises(ImportError):
        pgti.load_library()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2507_11683_amd")
    for dirpath, _dirs, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), f
                assert "pgti_oracle" not in text, f
    oracle_dir = os.path.join(ROOT, "oracle")
    for f in os.listdir(oracle_dir):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(oracle_dir, f)).read()
            assert "paper_2507_11683_amd" not in text and "pgti.h" not in text, f


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


@pytest.mark.parametrize("compiler,flags", [("gcc", ["-std=c99"]), ("g++", ["-std=c++11", "-x", "c++"])])
def test_header_is_plain_c_and_cxx(tmp_path, compiler, flags):
    # the boundary is usable from C99 and from C++ without HIP or torch headers
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_header.c"
    src.write_text('#include "pgti.h"\n'
                   "int main(void) { pgti_load_spec s; pgti_epoch_spec e; (void)s; (void)e;\n"
                   "  return pgti_create(0, 0) == PGTI_ERR_ARG ? 0 : 1; }\n")
    subprocess.check_call([compiler, *flags, "-Wall", "-Wextra", "-Werror", "-pedantic",
                           "-I", os.path.join(root, "include"), "-c", str(src), "-o", str(tmp_path / "use_header.o")])


def test_no_device_is_a_clean_error_not_a_fallback():
    # without a GPU the product path reports the HIP error; it never computes on the host
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from paper_2507_11683_amd import pgti
    with pytest.raises(pgti.PgtiError) as err:
        pgti.Context(0)
    assert err.value.status == pgti.PGTI_ERR_HIP and "device" in str(err.value)

