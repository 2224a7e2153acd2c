"""CPU-only checks of the C-ABI library: it loads, exports every symbol that
include/picasso.h declares, and its host-side logic (status strings, workspace
sizing, argument checks that need no device) behaves as documented."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2103_15076_amd as pk
    if not os.path.exists(pk.binding.LIB_PATH):
        from paper_2103_15076_amd import build
        build.build_library()
    return pk.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "picasso.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(picasso_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert "picasso_decimate" in names and "picasso_decimate_batch" in names and len(names) >= 10
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/picasso.h but not exported"
    from paper_2103_15076_amd.binding import EXPORTED_SYMBOLS
    assert sorted(EXPORTED_SYMBOLS) == names


def test_status_strings(lib):
    import paper_2103_15076_amd as pk
    seen = set()
    for st in (0, 1, -1, -2, -3, -4, -5, -6):
        s = pk.picasso_strerror(st)
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in pk.picasso_strerror(-99)


def test_workspace_sizing_is_monotone_and_linear(lib):
    import paper_2103_15076_amd as pk
    a = pk.picasso_workspace_bytes(115000, 231000, 1)
    b = pk.picasso_workspace_bytes(230000, 462000, 1)
    c = pk.picasso_workspace_bytes(115000, 231000, 16)
    assert 0 < a < b < 2.2 * a and a <= c < a + (1 << 20)
    assert a < 200 * (1 << 20)          # about 0.3 kB per vertex + 0.2 kB per facet


def test_host_side_argument_checks_need_no_device(lib):
    import paper_2103_15076_amd as pk
    n = ctypes.c_int32(0)
    # null context / null pointers are rejected before anything touches the device
    st = lib.picasso_decimate(None, None, None, 10, None, 10, 5, None, None, None, ctypes.byref(n), ctypes.byref(n), None)
    assert st == pk.PICASSO_ERR_INVALID_ARG
    assert lib.picasso_set_option(None, 0, 1) == pk.PICASSO_ERR_INVALID_ARG
    h = ctypes.c_void_p(0)
    assert lib.picasso_create(ctypes.byref(h), 0, 0, 10, 1) == pk.PICASSO_ERR_INVALID_ARG
    assert lib.picasso_create(ctypes.byref(h), 0, 10, 10, 0) == pk.PICASSO_ERR_INVALID_ARG
    assert lib.picasso_create(None, 0, 10, 10, 1) == pk.PICASSO_ERR_INVALID_ARG
    # capacities beyond what 32-bit indices address are refused before anything is allocated
    assert lib.picasso_create(ctypes.byref(h), 0, 10, (1 << 29) + 1, 1) == pk.PICASSO_ERR_INVALID_ARG
    assert lib.picasso_create(ctypes.byref(h), 0, 1 << 31, 10, 1) == pk.PICASSO_ERR_INVALID_ARG
    assert lib.picasso_device_copy(None, None, None, 16) == pk.PICASSO_ERR_INVALID_ARG
    # the entry point without a context checks its arguments and its size limit before it touches a device
    one = ctypes.c_void_p(16)
    f = lib.picasso_replace_mapping_static
    assert f(0, None, None, 4, 4, one, one, one) == pk.PICASSO_ERR_INVALID_ARG
    assert f(0, None, one, 4, 4, one, one, None) == pk.PICASSO_ERR_INVALID_ARG
    assert f(64, None, one, 4, 4, one, one, one) == pk.PICASSO_ERR_INVALID_ARG
    assert f(0, None, one, 4, pk.PICASSO_STATIC_MAX_CLUSTERS + 1, one, one, one) == pk.PICASSO_ERR_WORKSPACE


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2103_15076_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2103_15076_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle|picasso_oracle|libpicasso_oracle", src, flags=re.M), \
                    f"{f} reaches into the oracle"
