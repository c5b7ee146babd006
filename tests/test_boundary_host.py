"""CPU-side checks of the C-ABI library: it loads, exports every symbol that include/pilc.h
declares, and its host logic (geometry validation, sizes, messages) behaves.  No kernel runs."""
import ctypes as C
import os
import re

import pytest

from paper_2206_05279_amd import binding as pb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "pilc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pilc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = pb.lib()
    names = _declared_functions()
    assert set(names) == set(pb.EXPORTS)
    for name in names:
        assert hasattr(L, name), name


def test_library_was_built_from_the_current_sources():
    """The build records a digest of csrc/ and include/pilc.h beside the library; a library that
    was not rebuilt after a source change would be tested in place of the sources."""
    from paper_2206_05279_amd import build
    pb.lib()
    assert build.built_digest() == build.source_digest(), "run python -m paper_2206_05279_amd.build"


def test_version_and_messages():
    assert pb.pilc_version() == 1
    for code in range(-7, 1):
        assert pb.pilc_strerror(code) and "unknown" not in pb.pilc_strerror(code)
    assert "unknown" in pb.pilc_strerror(-99)


@pytest.mark.parametrize("geom,lanes", [
    ((64, 32, 32, 14, 0, 32, 0), 2048),
    ((50000, 32, 32, 14, 0, 16384, 0), 3125),
    ((16384, 64, 64, 15, 0, 64, 0), 1048576),
    ((30, 1080, 1920, 15, 1, 16, 16), 244800),
    ((8192, 256, 256, 12, 0, 64, 0), 8192 * 1024),
    ((3, 4, 4, 12, 0, 32, 0), 2),
])
def test_lane_count_and_sizes(geom, lanes):
    g = pb.make_geom(*geom)
    assert pb.pilc_lane_count(g) == lanes
    ws, mc = pb.pilc_workspace_size(g)
    sym = geom[0] * geom[1] * geom[2] * 3
    assert mc == 64 + 4 * (lanes + 1) + 4 * lanes + 2 * sym
    assert ws >= 8 * lanes + 2 * sym


@pytest.mark.parametrize("geom,code", [
    ((1, 4, 4, 9, 0, 16, 0), pb.PILC_E_ARG),
    ((1, 4, 4, 17, 0, 16, 0), pb.PILC_E_ARG),
    ((1, 4, 4, 12, 0, 5, 0), pb.PILC_E_ARG),
    ((1, 4, 4, 12, 0, 0, 0), pb.PILC_E_ARG),
    ((1, 4, 4, 12, 2, 4, 4), pb.PILC_E_ARG),
    ((1, 4, 4, 12, 1, 4, 0), pb.PILC_E_ARG),
    ((0, 4, 4, 12, 0, 16, 0), pb.PILC_E_ARG),
    ((65535, 4096, 4096, 12, 0, 4096, 0), pb.PILC_E_TOO_LARGE),
])
def test_bad_geometry_is_rejected(geom, code):
    g = pb.make_geom(*geom)
    assert pb.pilc_lane_count(g) == 0
    with pytest.raises(pb.PilcError) as e:
        pb.pilc_workspace_size(g)
    assert e.value.code == code


def test_null_and_misaligned_pointers_are_rejected_before_any_gpu_work():
    L = pb.lib()
    g = pb.make_geom(1, 4, 4, 12, 0, 16, 0)
    nb = C.c_uint64(0)
    good = pb.pilc_params(4096, 8192, 12288)
    big = 1 << 30
    assert L.pilc_encode(None, 4096, C.byref(good), 4096, big, 4096, big, C.byref(nb), None) == pb.PILC_E_ARG
    assert L.pilc_encode(C.byref(g), None, C.byref(good), 4096, big, 4096, big, C.byref(nb), None) == pb.PILC_E_ARG
    assert L.pilc_encode(C.byref(g), 4096, None, 4096, big, 4096, big, C.byref(nb), None) == pb.PILC_E_ARG
    assert L.pilc_encode(C.byref(g), 4096, C.byref(good), 4096 + 8, big, 4096, big, C.byref(nb), None) == pb.PILC_E_ARG
    assert L.pilc_encode(C.byref(g), 4096, C.byref(good), 4096, big, 4096 + 2, big, C.byref(nb), None) == pb.PILC_E_ARG
    odd = pb.pilc_params(4097, 8192, 12288)
    assert L.pilc_encode(C.byref(g), 4096, C.byref(odd), 4096, big, 4096, big, C.byref(nb), None) == pb.PILC_E_ARG
    assert L.pilc_encode(C.byref(g), 4096, C.byref(good), 4096, 16, 4096, big, C.byref(nb), None) == pb.PILC_E_WORKSPACE
    assert L.pilc_encode(C.byref(g), 4096, C.byref(good), 4096, big, 4096, 60, C.byref(nb), None) == pb.PILC_E_CAPACITY
    assert L.pilc_decode(C.byref(g), None, 100, C.byref(good), 4096, big, 4096, None) == pb.PILC_E_ARG
    assert L.pilc_decode(C.byref(g), 4096, 10, C.byref(good), 4096, big, 4096, None) == pb.PILC_E_FORMAT
    assert L.pilc_symbol_tables(C.byref(g), 4096, C.byref(good), None, 4096, None) == pb.PILC_E_ARG


def test_product_path_does_not_touch_the_oracle():
    """The package must never import the CPU oracle (no CPU fallback)."""
    pkg = os.path.join(ROOT, "paper_2206_05279_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"import\s+oracle|from\s+oracle|pilc_oracle|ac_bruteforce", text), \
                    os.path.join(dirpath, f)
