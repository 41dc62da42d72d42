"""CPU-side checks of the boundary: the library loads and exports every symbol the header declares."""
import os
import re

import paper_2310_03841_amd as ab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "abft.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(abft_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert "abft_gemm" in names and "abft_verify" in names and "abft_correct" in names and "abft_inject" in names
    L = ab.lib()
    for n in names:
        assert hasattr(L, n), n
    assert names == ab.exported_symbols()


def test_strerror_and_version_and_tile_shape():
    assert ab.abft_version() >= 100
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert ab.abft_strerror(code) not in ("", "unknown error")
    tm, tn = ab.abft_tile_shape(ab.ABFT_BF16, ab.make_shape(12608, 3072, 768))
    assert tm % 32 == 0 and tn % 32 == 0


def test_struct_layout_matches_header():
    import ctypes
    assert ctypes.sizeof(ab.abft_shape) == 11 * 8
    assert ctypes.sizeof(ab.abft_config) == 5 * 8
    assert ctypes.sizeof(ab.abft_result) == 4 * 8
