"""The C-ABI library loads and exports every symbol include/gids.h declares
(no compute call: this runs without a GPU)."""
import os
import re

import pytest

import paper_2306_16384_amd as gids

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gids.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gids_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = gids.lib()
    names = declared_symbols()
    assert len(names) >= 14
    for name in names:
        assert hasattr(L, name), name
    assert sorted(gids.EXPORTS) == names


def test_binding_has_the_same_names():
    for name in declared_symbols():
        assert callable(getattr(gids, name)), name


def test_host_only_entry_points():
    # pure host arithmetic (Section 3.2, Eq. 2-3): N = r / (1 - r) * IOPS * (Ti + Tt)
    n = gids.gids_accum_threshold(1.5e6, 25e-6, 5e-6, 0.95, 1)
    assert abs(n - 855.0) < 1e-6
    assert gids.gids_accum_threshold(1.5e6, 25e-6, 5e-6, 1.0, 1) < 0
    # argument validation happens before any device call
    with pytest.raises(gids.GidsError) as e:
        gids.gids_store_create(100, 24, 8)
    assert e.value.code == gids.GIDS_E_INVAL
    with pytest.raises(gids.GidsError) as e:
        gids.gids_store_create(100, 64, 3)
    assert e.value.code == gids.GIDS_E_INVAL
    with pytest.raises(gids.GidsError) as e:
        gids.gids_cache_create(None, 16, 4, 64)
    assert e.value.code == gids.GIDS_E_INVAL


def test_header_is_plain_c_and_links(tmp_path):
    """include/gids.h compiles as C99 and a C program links against the library."""
    import subprocess
    exe = tmp_path / "abi_check"
    lib_dir = os.path.dirname(gids.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "abi_check.c"), "-o", str(exe), "-L", lib_dir, "-lgids",
                           "-Wl,-rpath," + lib_dir, "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.startswith("abi ok 80")              # gids_stats is 7 x u64 + 2 x i32 + 2 x u64


def test_binding_struct_matches_the_header():
    import ctypes
    from paper_2306_16384_amd import binding
    assert ctypes.sizeof(binding.gids_stats) == 80            # the C program above prints the header's sizeof
